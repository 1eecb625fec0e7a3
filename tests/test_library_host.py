"""CPU-side checks of the boundary: the shared library loads, exports every symbol the
header declares, and rejects bad arguments on the host before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2505_12044_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "flashbias.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(api.LIB_PATH):
        from paper_2505_12044_amd import build
        build.build(force=False)
    return api.load_library()


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fb_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_exported(lib):
    names = _declared_symbols()
    assert set(names) == set(api.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_status_strings(lib):
    assert lib.fb_version() >= 100
    assert lib.fb_status_string(0) == b"ok"
    seen = {lib.fb_status_string(i) for i in range(8)}
    assert len(seen) == 8
    assert lib.fb_status_string(99) == b"unknown status"


def _fwd(lib, **kw):
    a = dict(q=64, k=64, v=64, phi_q=64, phi_k=64, out=64, lse=64, B=1, H=1, N=16, C=64, R=4,
             causal=0, dtype=api.FB_BF16, phi_dtype=api.FB_BF16, bcast=0, scale=0.0)
    a.update(kw)
    return lib.fb_lowrank_attn_fwd(a["q"], a["k"], a["v"], a["phi_q"], a["phi_k"], a["out"], a["lse"],
                                   a["B"], a["H"], a["N"], a["C"], a["R"], a["causal"], a["dtype"],
                                   a["phi_dtype"], a["bcast"], a["scale"], None)


def test_forward_argument_errors(lib):
    # fake non-null addresses: every case below must be rejected before any device access
    assert _fwd(lib, q=None) == 1
    assert _fwd(lib, phi_k=None) == 1
    assert _fwd(lib, N=0) == 2
    assert _fwd(lib, R=-1) == 2
    assert _fwd(lib, B=1 << 20, H=1 << 10, N=1 << 12) == 2          # index overflow
    assert _fwd(lib, C=48) == 3
    assert _fwd(lib, R=65) == 3                                      # padded width > 64
    assert _fwd(lib, R=11, phi_dtype=api.FB_F32) == 3                # 6 R > 64 columns
    assert _fwd(lib, dtype=api.FB_F32, phi_dtype=api.FB_BF16) == 3
    assert _fwd(lib, dtype=7) == 3
    assert _fwd(lib, k=72) == 4                                      # misaligned


def test_dense_and_backward_argument_errors(lib):
    f = lib.fb_dense_bias_attn_fwd
    assert f(64, 64, 64, None, 64, 64, 1, 1, 16, 64, 0, api.FB_BF16, 0, 0.0, None) == 1
    assert f(64, 64, 64, 64, 64, 64, 1, 1, 16, 96, 0, api.FB_BF16, 0, 0.0, None) == 3
    assert f(64, 64, 64, 68, 64, 64, 1, 1, 16, 64, 0, api.FB_BF16, 0, 0.0, None) == 4
    db = lib.fb_dense_bias_attn_bwd
    wsd = lib.fb_dense_bias_attn_bwd_workspace_bytes(1, 1, 64, 64, api.FB_BF16)
    assert wsd == 64 * 8 + 2 * 64 * 64 * 2
    # head dimension 16: 32-channel operand rows plus widened copies of v and dO
    assert lib.fb_dense_bias_attn_bwd_workspace_bytes(1, 1, 64, 16, api.FB_BF16) == 64 * 8 + 2 * 64 * (32 + 32) * 2
    assert db(*([64] * 10), None, 1, 1, 64, 64, 0, api.FB_BF16, 0, 0.0, 64, wsd, None) == 1         # dbias NULL
    assert db(*([64] * 11), 1, 1, 60, 64, 0, api.FB_BF16, 0, 0.0, 64, wsd, None) == 3               # N % 8 != 0
    assert db(*([64] * 11), 1, 1, 64, 64, 0, api.FB_BF16, 0, 0.0, 64, wsd - 1, None) == 5
    a = lib.fb_alibi_attn_fwd
    assert a(64, 64, 64, None, 64, 64, 1, 1, 16, 64, 1, api.FB_BF16, 0.0, None) == 1      # slopes NULL
    assert a(64, 64, 64, 64, 64, 64, 1, 1, 16, 64, 1, api.FB_F32, 0.0, None) == 3         # bf16 only
    assert a(64, 64, 64, 66, 64, 64, 1, 1, 16, 64, 1, api.FB_BF16, 0.0, None) == 4        # slopes not 4-byte aligned
    assert a(64, 64, 64, 64, 64, 64, 1, 1, 0, 64, 1, api.FB_BF16, 0.0, None) == 2
    ws = lib.fb_lowrank_attn_bwd_workspace_bytes(2, 3, 100, 64, 8, api.FB_BF16)
    # (lse, D) pairs plus the two concatenated operand copies of width up to C + 64
    assert ws == 2 * 3 * 100 * 8 + 2 * (2 * 3 * 100) * (64 + 64) * 2
    assert lib.fb_lowrank_attn_bwd_workspace_bytes(0, 3, 100, 64, 8, api.FB_BF16) == 0
    # head dimension 16: 32-channel operand rows plus widened copies of v and dO
    assert lib.fb_lowrank_attn_bwd_workspace_bytes(1, 1, 10, 16, 9, api.FB_F32) == 10 * 8 + 2 * 10 * (32 + 64 + 32) * 2
    g = lib.fb_lowrank_attn_bwd
    ptrs = [64] * 13

    def bwd(ptrs=ptrs, B=2, H=3, N=100, C=64, R=8, dtype=api.FB_BF16, phi=api.FB_BF16, w=64, wb=ws):
        return g(*ptrs, B, H, N, C, R, 0, dtype, phi, 0, 0.0, w, wb, None)

    assert bwd(ptrs=[None] + [64] * 12) == 1
    assert bwd(dtype=api.FB_F32) == 3          # fp32 tensors need fp32 factors
    assert bwd(dtype=api.FB_F32, phi=api.FB_F32, R=70) == 3
    assert bwd(R=70) == 3                      # padded width > 64
    assert bwd(w=None) == 5
    assert bwd(wb=ws - 1) == 5
    assert bwd(w=72) == 4


def test_mulbias_argument_errors(lib):
    f = lib.fb_lowrank_mulbias_attn_fwd
    need = lib.fb_lowrank_mulbias_attn_fwd_workspace_bytes(1, 2, 100, 64, 2, api.FB_BF16)
    assert need == 4 * 1 * 2 * 100 * 64 * 2
    assert lib.fb_lowrank_mulbias_attn_fwd_workspace_bytes(1, 2, 100, 64, 0, api.FB_BF16) == 0

    def call(ptrs=None, C=64, R=2, dtype=api.FB_BF16, w=64, wb=need):
        ptrs = ptrs or [64] * 7
        return f(*ptrs, 1, 2, 100, C, R, 0, dtype, api.FB_F32, 0, 0.0, w, wb, None)

    assert call(ptrs=[64, 64, 64, None, 64, 64, 64]) == 1      # factors are required
    assert call(R=0) == 2
    assert call(R=4) == 3                                      # C (R - 1) = 192 > 128
    assert call(C=128, R=2) == 3                               # C = 128 takes no extra channels
    assert call(dtype=api.FB_F32) == 3
    assert call(ptrs=[64, 64, 64, 66, 64, 64, 64]) == 4        # factors not 4-byte aligned
    assert call(w=None) == 5
    assert call(wb=need - 1) == 5
    assert call(w=72) == 4


def test_mulbias_backward_argument_errors(lib):
    f = lib.fb_lowrank_mulbias_attn_bwd
    need = lib.fb_lowrank_mulbias_attn_bwd_workspace_bytes(1, 2, 100, 32, 3, api.FB_BF16)
    # q', k' in bf16, their gradients in float, and the additive backward's scratch for 64 extra channels
    assert need == 2 * 200 * 32 * 3 * (2 + 4) + lib.fb_lowrank_attn_bwd_workspace_bytes(1, 2, 100, 32, 64, api.FB_BF16)
    # more than 64 extra channels: operand rows of width C + 128
    need5 = lib.fb_lowrank_mulbias_attn_bwd_workspace_bytes(1, 2, 100, 32, 5, api.FB_BF16)
    assert need5 == 2 * 200 * 32 * 5 * 6 + 200 * 8 + 2 * 200 * (32 + 128) * 2

    def call(ptrs=None, C=32, R=3, dtype=api.FB_BF16, w=64, wb=need):
        ptrs = ptrs or [64] * 13
        return f(*ptrs, 1, 2, 100, C, R, 0, dtype, api.FB_BF16, 0, 0.0, w, wb, None)

    assert call(ptrs=[64] * 12 + [None]) == 1
    assert call(R=0) == 2
    assert call(R=6) == 3                      # C (R - 1) = 160 > 128
    assert call(dtype=api.FB_F32) == 3
    assert call(ptrs=[64] * 11 + [66, 64]) == 4
    assert call(wb=need - 1) == 5
    assert call(w=None) == 5


def test_alibi_backward_argument_errors(lib):
    f = lib.fb_alibi_attn_bwd
    need = lib.fb_alibi_attn_bwd_workspace_bytes(1, 2, 100, 64, api.FB_BF16)
    assert need == lib.fb_lowrank_attn_bwd_workspace_bytes(1, 2, 100, 64, 2, api.FB_BF16)

    def call(ptrs=None, C=64, dtype=api.FB_BF16, w=64, wb=need, N=100):
        ptrs = ptrs or [64] * 10 + [None]                       # dslope_rows NULL: not wanted
        if len(ptrs) == 10:
            ptrs = ptrs + [None]
        return f(*ptrs, 1, 2, N, C, 1, dtype, 0.0, w, wb, None)

    assert call(ptrs=[64, 64, 64, None] + [64] * 6) == 1       # slopes
    assert call(ptrs=[64] * 10 + [66]) == 4                    # dslope_rows not 4-byte aligned
    assert call(N=0) == 2
    assert call(C=48) == 3
    assert call(dtype=api.FB_F32) == 3
    assert call(ptrs=[64, 64, 64, 66] + [64] * 6) == 4
    assert call(wb=need - 1) == 5


def test_size_limits_follow_the_indexing(lib):
    """Offsets above the head level are 64-bit: tensors of 2^31 elements and more are accepted
    (the calls below pass the shape check and stop at the deliberately misaligned pointer);
    what is limited is the row count (32-bit counters) and the extent of one head (32-bit byte
    offsets)."""
    assert _fwd(lib, B=2, H=8, N=1 << 17, C=128, R=8, k=72) == 4        # 2^31 elements per tensor
    assert _fwd(lib, B=64, H=64, N=1 << 16, C=128, R=8, k=72) == 4      # 2^35 elements, 2^28 rows
    assert _fwd(lib, B=1 << 10, H=1 << 5, N=1 << 16, C=32, R=0, k=72) == 2     # 2^31 rows
    assert _fwd(lib, B=1, H=1, N=1 << 23, C=128, R=0, k=72) == 2        # one head: N C = 2^30 elements
    assert _fwd(lib, B=1, H=1, N=1 << 22, C=128, R=0, k=72) == 4
    assert _fwd(lib, B=1, H=1, N=1 << 26, C=16, R=16, k=72) == 2        # N R = 2^30 factor values
    a = lib.fb_alibi_attn_fwd
    assert a(64, 64, 64, 64, 64, 64, 1, 1, (1 << 24) + 1, 16, 1, api.FB_BF16, 0.0, None) == 3   # fp32 positions


def test_noalloc_backward_host_checks(lib):
    """The allocation-free backward rejects bad shapes and problems beyond its static scratch on
    the host, before any device call."""
    g = lib.fb_lowrank_attn_bwd_noalloc
    ptrs = [64] * 13
    assert g(*ptrs, 0, 1, 16, 64, 4, 0, api.FB_BF16, api.FB_BF16, 0, 0.0, None) == 2
    assert g(*ptrs, 1, 1, 16, 48, 4, 0, api.FB_BF16, api.FB_BF16, 0, 0.0, None) == 3
    B, H, N, C, R = 4, 16, 4096, 128, 2
    assert lib.fb_lowrank_attn_bwd_workspace_bytes(B, H, N, C, R, api.FB_BF16) > api.FB_STATIC_SCRATCH_BYTES
    st = g(*ptrs, B, H, N, C, R, 1, api.FB_BF16, api.FB_F32, 1, 0.0, None)
    assert st == 7 and b"static scratch" in lib.fb_status_string(st)
    text = open(HEADER).read()
    m = re.search(r"#define FB_STATIC_SCRATCH_BYTES \(\(size_t\)(\d+) << (\d+)\)", text)
    assert m and int(m.group(1)) << int(m.group(2)) == api.FB_STATIC_SCRATCH_BYTES


def test_only_the_c_abi_is_exported():
    """Built with hidden visibility: the dynamic symbol table defines the header's functions and
    nothing else of this library's own."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", api.LIB_PATH], capture_output=True, text=True, check=True).stdout
    defined = {line.split()[-1] for line in out.splitlines() if line.strip()}
    ours = {n for n in defined if not n.startswith("__hip") and n not in ("_init", "_fini")}
    assert ours == set(api.EXPORTS), sorted(ours ^ set(api.EXPORTS))


def test_tune_knob(lib):
    assert lib.fb_tune_set(b"fwd_qb", 2) == 0
    assert lib.fb_tune_set(b"fwd_qb", 0) == 0
    assert lib.fb_tune_set(b"fwd_qb", 3) == 2
    assert lib.fb_tune_set(b"fwd_qb", 4) == 2
    assert lib.fb_tune_set(b"fwd_qb", 8) == 0
    assert lib.fb_tune_set(b"fwd_qb", 0) == 0
    assert lib.fb_tune_set(b"fwd_causal_up", 0) == 0
    assert lib.fb_tune_set(b"fwd_causal_up", 2) == 2
    assert lib.fb_tune_set(b"fwd_causal_up", 1) == 0
    assert lib.fb_tune_set(b"fwd_lds_pad", 0) == 3          # probe knob removed
    assert lib.fb_tune_set(b"nope", 1) == 3
    assert lib.fb_tune_set(None, 1) == 1


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(api.FlashBiasError):
        api.load_library(str(tmp_path / "libflashbias.so"))


def test_hand_placed_mfma_forms_keep_their_wait_states():
    """The backward's inline-assembly MFMA forms are invisible to the compiler's hazard padding: the
    generated code must show no instruction touching such a result inside its wait-state window
    (compiles one source to assembly, about a minute and a half).  The scanner itself is checked on
    a planted violation first."""
    from paper_2505_12044_amd import check_mfma_hazards as chk
    planted = ("_Zk:\n\tv_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], v[0:15]\n"
               "\tv_mfma_f32_32x32x16_bf16 v[0:15], v[24:27], v[20:23], v[0:15]\n"
               "\tv_add_f32_e32 v40, v3, v41\n")
    seen, found = chk.scan_asm(planted)
    assert seen == 2 and len(found) == 1
    fenced = planted.replace("\tv_add_f32", "\ts_nop 7\n\ts_nop 2\n\tv_add_f32")
    assert chk.scan_asm(fenced)[1] == []
    seen, found = chk.check()
    assert seen > 0 and found == [], found[:3]
