"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "quartet.h")
LIB = os.path.join(ROOT, "paper_2505_14669_amd", "libquartet.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="HIP library not built (run __graft_entry__.build())")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(quartet_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(LIB)
    names = declared_symbols()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), name


def test_binding_mirrors_the_header():
    from paper_2505_14669_amd import binding
    for name in declared_symbols():
        assert callable(getattr(binding, name)), name
    assert sorted(binding.EXPORTS) == declared_symbols()
    assert binding.quartet_sr_bits() == 22


def test_sign_word_is_philox_of_the_seed():
    # counter (0,0,0,0xFFFFFFFF), key = seed words; checked against the oracle's generator, which is
    # itself pinned to the published known-answer vectors
    import oracle
    from paper_2505_14669_amd import binding
    for seed in (0, 1, 77, 0x123456789ABCDEF0, 2 ** 64 - 1):
        assert binding.quartet_sign_word(seed) == oracle.sign_word(seed)


def launches(q):
    """kernel launches so far, if the library is the host-only build with counting stand-ins for the launchers; else None"""
    try:
        return q._lib.quartet_hostcheck_launches()
    except AttributeError:
        return None


def test_gemm_grad_pair_checks_both_products_before_launching():
    from paper_2505_14669_amd import binding as q
    P = 0x10000
    E = q.QUARTET_EINVAL
    good = lambda: q.gemm_grad_args(P, P, P, P, 64, 64, 64, P, 1.0, P, 64)
    before = launches(q)
    bad = []
    for field, value in (("a_codes", None), ("b_scales", None), ("d", None), ("k", 48), ("n", 48), ("ldd", 32), ("m", -1),
                         ("a_codes", P + 8), ("mask", P + 2), ("a_scales", P + 1)):
        g = good()
        setattr(g, field, value)
        bad.append(g)
    for g in bad:
        assert q.quartet_mxfp4_gemm_grad_pair(g, good(), q.QUARTET_DTYPE_F32, 0) == E
        assert q.quartet_mxfp4_gemm_grad_pair(good(), g, q.QUARTET_DTYPE_F32, 0) == E
    assert q.quartet_mxfp4_gemm_grad_pair(None, good(), q.QUARTET_DTYPE_F32, 0) == E
    assert q.quartet_mxfp4_gemm_grad_pair(good(), None, q.QUARTET_DTYPE_F32, 0) == E
    assert q.quartet_mxfp4_gemm_grad_pair(good(), good(), 7, 0) == E
    huge = good()
    huge.k = 2 ** 24
    assert q.quartet_mxfp4_gemm_grad_pair(good(), huge, q.QUARTET_DTYPE_F32, 0) == q.QUARTET_ENOTSUP
    assert launches(q) == before


def test_bad_arguments_are_rejected_on_the_host():
    from paper_2505_14669_amd import binding as q
    P = 0x10000  # fake, aligned, never dereferenced: validation fails first
    E = q.QUARTET_EINVAL
    before = launches(q)
    assert q.quartet_quant_fwd(None, 4, 32, 32, 0, P, P, P, 0) == E
    assert q.quartet_quant_fwd(P, 4, 48, 48, 0, P, P, P, 0) == E          # k % 32
    assert q.quartet_quant_fwd(P, 4, 64, 32, 0, P, P, P, 0) == E          # ldx < k
    assert q.quartet_quant_fwd(P, 4, 64, 68, 0, P, P, P, 0) == E          # ldx % 8
    assert q.quartet_quant_fwd(P + 2, 4, 64, 64, 0, P, P, P, 0) == E      # alignment
    assert q.quartet_quant_fwd(P, -1, 64, 64, 0, P, P, P, 0) == E
    assert q.quartet_quant_fwd(P, 12, 64, 16, 1, P, P, P, 0) == E         # transposed: rows % 8
    assert q.quartet_quant_fwd(P, 2 ** 40, 2 ** 20, 2 ** 20, 0, P, P, P, 0) == q.QUARTET_ENOTSUP
    assert q.quartet_quant_bwd_sr(P, 4, 64, 64, 0, 0, 0, 0, 2, P, P, 0) == E  # rounding
    assert q.quartet_quant_bwd_sr(P, 4, 64, 64, 0, 0, 0, 0, 0, None, P, 0) == E
    assert q.quartet_requant_transpose_sr(P, P, 48, 64, 0, 0, 0, 0, P, P, 0) == E  # rows % 32
    assert q.quartet_fwd_operands(P, P, 4, 48, 8, P, P, P, P, P, P, 0) == E                          # in % 32
    assert q.quartet_fwd_operands(P, P, 4, 64, 8, P, P, None, P, P, P, 0) == E                        # both masks required
    assert q.quartet_fwd_operands(P, P + 2, 4, 64, 8, P, P, P, P, P, P, 0) == E                       # alignment
    assert q.quartet_fwd_operands(P, P, 2 ** 40, 2 ** 20, 8, P, P, P, P, P, P, 0) == q.QUARTET_ENOTSUP
    assert q.quartet_bwd_operands(P, 64, 64, 48, P, P, P, P, 0, 0, 0, P, P, P, P, P, P, 0) == E     # out % 32
    assert q.quartet_bwd_operands(P, 64, 64, 64, P, P, P, P, 0, 0, 2, P, P, P, P, P, P, 0) == E     # rounding
    assert q.quartet_bwd_operands(P, 64, 64, 64, P, P, P, None, 0, 0, 0, P, P, P, P, P, P, 0) == E
    assert q.quartet_bwd_operands(P, 64, 64, 64, P, P, P, P, 0, 0, 0, P, P + 2, P, P, P, P, 0) == E # scale alignment
    assert q.quartet_bwd_operands(P, 64, 2 ** 24, 64, P, P, P, P, 0, 0, 0, P, P, P, P, P, P, 0) == q.QUARTET_ENOTSUP
    assert q.quartet_mxfp4_gemm(P, P, P, P, 4, 4, 40, 1.0, P, 0, 4, 0) == E
    assert q.quartet_mxfp4_gemm(P, P, P, P, 4, 8, 64, 1.0, P, 0, 4, 0) == E    # ldd < n
    assert q.quartet_mxfp4_gemm(P, P, P, P, 4, 8, 64, 1.0, P, 7, 8, 0) == E    # dtype
    assert q.quartet_mxfp4_gemm_grad(P, P, P, P, 4, 40, 64, None, 1.0, P, 0, 40, 0) == E    # n % 32
    assert q.quartet_mxfp4_gemm_grad(P, P, P, P, 4, 64, 48, None, 1.0, P, 0, 64, 0) == E    # k % 32
    assert q.quartet_mxfp4_gemm_grad(P, P, P, P, 4, 64, 64, None, 1.0, P, 0, 32, 0) == E    # ldd < n
    assert q.quartet_grad_epilogue(P, None, 4, 40, 1.0, P, 0, 0) == E
    assert q.quartet_grad_epilogue(P, None, 4, 64, 1.0, P, 1, 0) == E          # bf16 in place
    assert q.quartet_mxfp4_dequant(P, None, 4, 64, P, 0) == E
    assert q.quartet_linear_fwd(P, P, 4, 48, 8, P, 0, P, P, P, P, P, P, 0) == E
    assert q.quartet_linear_workspace_bytes(100, 64, 64) == 0
    need = q.quartet_linear_workspace_bytes(64, 64, 96)
    assert need > 0 and need % 256 == 0
    assert q.quartet_linear_bwd(P, 64, 64, 96, P, P, P, P, P, P, 0, 0, P, P, 0, 0x10000, need - 1, 0) == E
    assert q.quartet_linear_bwd(P, 64, 64, 96, P, P, P, P, P, P, 0, 0, P, P, 0, None, need, 0) == E
    assert q.quartet_linear_bwd(P, 64, 60, 96, P, P, P, P, P, P, 0, 0, P, P, 0, 0x10000, need, 0) == E
    assert q.quartet_last_hip_error() == 0
    assert launches(q) == before          # (host-only build) nothing was launched by a rejected call


def test_empty_problems_are_accepted_without_a_gpu():
    from paper_2505_14669_amd import binding as q
    P = 0x10000
    assert q.quartet_quant_fwd(P, 0, 64, 64, 0, P, P, P, 0) == 0
    assert q.quartet_quant_bwd_sr(P, 0, 64, 64, 0, 0, 0, 0, 0, P, P, 0) == 0
    assert q.quartet_mxfp4_gemm(P, P, P, P, 0, 8, 64, 1.0, P, 0, 8, 0) == 0
    assert q.quartet_bwd_operands(P, 0, 0, 0, P, P, P, P, 0, 0, 0, P, P, P, P, P, P, 0) == 0
    assert q.quartet_fwd_operands(P, P, 0, 64, 0, P, P, P, P, P, P, 0) == 0
    assert q.quartet_grad_epilogue(P, None, 0, 64, 1.0, P, 0, 0) == 0


def test_block_entry_points_reject_bad_arguments_on_the_host():
    import oracle
    from paper_2505_14669_amd import binding as q
    P = 0x10000
    E = q.QUARTET_EINVAL
    sw = [0] * 8
    for seed in (0, 9, 2 ** 63 + 5):
        assert q.quartet_sign_words(seed) == [int(w) for w in oracle.sign_words(seed)]
    assert q.quartet_quant_fwd_block(P, 4, 128, 128, 0, 48, P, P, P, 0) == E          # unsupported block
    assert q.quartet_quant_fwd_block(P, 4, 96, 96, 0, 64, P, P, P, 0) == E            # k % block
    assert q.quartet_quant_fwd_block(None, 4, 128, 128, 0, 64, P, P, P, 0) == E
    assert q.quartet_quant_bwd_sr_block(P, 4, 192, 192, 0, 128, sw, 0, 0, 0, P, P, 0) == E    # k % block
    assert q.quartet_quant_bwd_sr_block(P, 4, 256, 256, 0, 128, sw, 0, 0, 3, P, P, 0) == E    # rounding
    assert q.quartet_requant_transpose_sr_block(P, P, 64, 96, 64, sw, 0, 0, 0, P, P, 0) == E  # k % block
    assert q.quartet_requant_transpose_sr_block(P, P, 48, 128, 64, sw, 0, 0, 0, P, P, 0) == E # rows % 32
    assert q.quartet_grad_epilogue_block(P, None, 4, 96, 64, 1.0, P, 0, 0) == E
    assert q.quartet_grad_epilogue_block(P, None, 4, 128, 16, 1.0, P, 0, 0) == E
    assert q.quartet_linear_fwd_block(P, P, 64, 96, 64, 64, P, 0, P, P, P, P, P, P, 0) == E   # in % block
    assert q.quartet_linear_workspace_bytes_block(64, 64, 96, 64) == 0                         # out % block
    assert q.quartet_linear_workspace_bytes_block(64, 64, 64, 32) == q.quartet_linear_workspace_bytes(64, 64, 64)
    assert q.quartet_linear_workspace_bytes_block(128, 128, 256, 128) == q.quartet_linear_workspace_bytes(128, 128, 256)
    need = q.quartet_linear_workspace_bytes_block(256, 256, 512, 256)
    assert need > q.quartet_linear_workspace_bytes(256, 256, 512)    # blocks of 256: room for the fp32 product
    assert q.quartet_linear_bwd_block(P, 256, 256, 512, 256, P, P, P, P, P, P, 0, 0, P, P, 0, 0x10000, need - 1, 0) == E
    assert q.quartet_linear_bwd_block(P, 128, 128, 192, 128, P, P, P, P, P, P, 0, 0, P, P, 0, 0x10000, need, 0) == E
    assert q.quartet_mxfp4_gemm_grad_block(P, P, P, P, 4, 128, 64, 256, None, 1.0, P, 0, 128, 0) == q.QUARTET_ENOTSUP
    assert q.quartet_mxfp4_gemm_grad_block(P, P, P, P, 4, 96, 64, 64, None, 1.0, P, 0, 96, 0) == E      # n % block
    assert q.quartet_mxfp4_gemm_grad_block(P, P, P, P, 4, 128, 64, 48, None, 1.0, P, 0, 128, 0) == E    # unsupported block
    assert q.quartet_last_hip_error() == 0


def test_static_scratch_backward_rejects_layers_beyond_its_array_on_the_host():
    from paper_2505_14669_amd import binding as q
    P = 0x10000
    assert q.quartet_static_scratch_bytes() == 64 << 20
    t, i, o = 16384, 4096, 4096
    assert q.quartet_linear_workspace_bytes(t, i, o) > q.quartet_static_scratch_bytes()
    args = lambda t, i, o: (P, t, i, o, P, P, P, P, P, P, 0, 0, P, P, q.QUARTET_DTYPE_F32, 0)
    assert q.quartet_linear_bwd_static(*args(t, i, o)) == q.QUARTET_ENOTSUP
    assert q.quartet_linear_bwd_static(*args(2 ** 40, 2 ** 30, 2 ** 30)) == q.QUARTET_ENOTSUP
    assert q.quartet_linear_bwd_static(*args(48, 32, 32)) == q.QUARTET_EINVAL
    assert q.quartet_linear_bwd_static(None, 32, 32, 32, P, P, P, P, P, P, 0, 0, P, P, 0, 0) == q.QUARTET_EINVAL
    assert q.quartet_debug_set_gemm_plan(3, 0) == q.QUARTET_EINVAL and q.quartet_debug_set_gemm_plan(-1, 0) == q.QUARTET_OK


def test_profile_record_can_be_set_up_and_dropped_without_a_gpu():
    # with no GPU the events cannot be created: the call must fail cleanly and free what it made (last in this file: it
    # leaves a HIP error in the thread's last-error slot, which the tests above expect to be clear)
    from paper_2505_14669_amd import binding as q
    assert q.quartet_profile_enable(-1) == q.QUARTET_EINVAL
    rc = q.quartet_profile_enable(3)
    assert rc in (q.QUARTET_OK, q.QUARTET_EHIP)
    assert q.quartet_profile_enable(0) == q.QUARTET_OK
    assert q.quartet_profile_read(None, None, 0) == 0
    assert q.quartet_profile_clock(None) == q.QUARTET_OK and q.quartet_profile_clock(0x10004) == q.QUARTET_EINVAL
    assert q.quartet_probe_mfma_ceiling(None, 0x10000, 1, 1, 0x10000, None, 0) == q.QUARTET_EINVAL
