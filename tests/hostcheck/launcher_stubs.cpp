// Host-only stand-ins for the library's kernel launchers (test infrastructure): linked with csrc/api.hip they give
// a library whose entry points run their whole argument validation and sequencing on the CPU and launch nothing, so that
// tests/test_abi_host.py can drive it under AddressSanitizer / UndefinedBehaviorSanitizer (tests/test_sanitizers.py).
// Every stand-in counts its calls: a rejected call must not have reached any of them.
#include "launchers.h"
static int g_launches = 0;
extern "C" int quartet_hostcheck_launches(void) { return g_launches; }
namespace quartet {
hipError_t launch_quant(int, const void*, int64_t, int64_t, int64_t, int, const SrParams&, uint8_t*, uint8_t*, uint32_t*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_requant_transpose(int, const uint8_t*, const uint8_t*, int64_t, int64_t, const SrParams&, uint8_t*, uint8_t*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_fwd_operands(const void*, int64_t, const void*, int64_t, int64_t, uint8_t*, uint8_t*, uint32_t*, uint8_t*, uint8_t*, uint32_t*, const SrParams&, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_bwd_operands(int, const void*, int64_t, int64_t, int64_t, const uint8_t*, const uint8_t*, const uint8_t*, const uint8_t*, const SrParams&, const SrParams&, const SrParams&, uint8_t*, uint8_t*, uint8_t*, uint8_t*, uint8_t*, uint8_t*, const SrParams&, uint8_t*, uint8_t*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_dequant(const uint8_t*, const uint8_t*, int64_t, int64_t, float*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_gemm(const uint8_t*, const uint8_t*, const uint8_t*, const uint8_t*, int64_t, int64_t, int64_t, float, void*, int, int64_t, int, const uint32_t*, uint32_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_gemm_grad_pair(const GemmArgs&, const GemmArgs&, int, uint32_t, hipStream_t) { ++g_launches; return hipSuccess; }
void set_gemm_plan(int, int) {}
hipError_t launch_grad_epilogue(const float*, const uint32_t*, int64_t, int64_t, uint32_t, float, void*, int, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_mfma_ceiling(const uint8_t*, const uint8_t*, uint32_t, uint32_t, float*, uint64_t*, hipStream_t) { ++g_launches; return hipSuccess; }
void set_clock_counters(uint64_t*) {}
hipError_t launch_mxfp8_quant(const void*, int64_t, int64_t, int64_t, uint8_t*, uint8_t*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_mxfp8_gemm(const uint8_t*, const uint8_t*, const uint8_t*, const uint8_t*, int64_t, int64_t, int64_t, float, void*, int, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
}
