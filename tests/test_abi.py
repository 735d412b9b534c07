"""Host-side checks that need no GPU: the library loads, exports what include/vfa.h declares,
and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pkg():
    import paper_2604_12798_amd as p
    if not os.path.exists(p.LIB_PATH):
        from paper_2604_12798_amd import build
        build.build_lib()
    return p


def test_every_declared_symbol_is_exported(pkg):
    hdr = open(os.path.join(ROOT, "include", "vfa.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(vfa_\w+|vsa_\w+|fa_\w+)\s*\(", hdr))
    assert names == set(pkg.EXPORTS)
    L = pkg.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_strerror_and_workspace(pkg):
    assert pkg.strerror(0) == "ok"
    assert "invalid" in pkg.strerror(-1) and "unsupported" in pkg.strerror(-2) and "HIP" in pkg.strerror(-3)
    assert pkg.workspace_bytes(2, 8, 16384, 128, 64) == 2 * 8 * 256 * 128 * 2
    assert pkg.workspace_bytes(1, 1, 65, 64, 64) == 256          # 2 blocks * 64 * 2 bytes, rounded up
    assert pkg.workspace_bytes(0, 1, 64, 64, 64) == 0


def test_bad_arguments_are_rejected_before_launch(pkg):
    L = pkg.lib()
    p = ctypes.c_void_p(0x1000)     # never dereferenced: every call below fails validation first
    odd = ctypes.c_void_p(0x1004)
    none = ctypes.c_void_p(0)
    fa = lambda *a: L.fa_baseline_fwd(*a)
    ok_shape = (1, 4, 2, 256, 128, 128, 64, 1)
    assert fa(none, p, p, p, none, *ok_shape, 0.0, none) == -1                 # null Q
    assert fa(odd, p, p, p, none, *ok_shape, 0.0, none) == -1                  # misaligned
    assert fa(p, p, p, p, none, 1, 4, 3, 256, 128, 128, 64, 1, 0.0, none) == -1  # Hq % Hkv
    assert fa(p, p, p, p, none, 1, 4, 2, -1, 128, 128, 64, 1, 0.0, none) == -1   # negative N
    assert fa(p, p, p, p, none, 1, 4, 2, 256, 96, 128, 64, 1, 0.0, none) == -2   # d
    assert fa(p, p, p, p, none, 1, 4, 2, 256, 128, 128, 128, 1, 0.0, none) == -2  # block pair
    assert fa(p, p, p, p, none, 1, 4, 2, 256, 128, 32, 64, 1, 0.0, none) == -2
    assert fa(p, p, p, p, none, 0, 4, 2, 256, 128, 128, 64, 1, 0.0, none) == 0   # empty batch: no-op
    assert fa(none, none, none, none, none, 1, 4, 2, 0, 128, 128, 64, 1, 0.0, none) == 0  # N = 0: no-op
    lz = lambda *a: L.fa_lazy_rescale_fwd(*a)
    assert lz(p, p, p, p, none, *ok_shape, 0.0, -1.0, none) == -1                  # tau < 0
    assert lz(p, p, p, p, none, *ok_shape, 0.0, float("nan"), none) == -1
    assert lz(p, p, p, p, none, *ok_shape, 0.0, float("inf"), none) == -1
    assert lz(none, p, p, p, none, *ok_shape, 0.0, 8.0, none) == -1
    assert lz(p, p, p, p, none, 0, 4, 2, 256, 128, 128, 64, 1, 0.0, 8.0, none) == 0
    se = lambda *a: L.fa_lazy_rescale_softexp_fwd(*a)
    assert se(p, p, p, p, none, *ok_shape, 0.0, -1.0, none) == -1
    assert se(p, p, p, p, none, *ok_shape, 0.0, float("nan"), none) == -1
    assert se(none, p, p, p, none, *ok_shape, 0.0, 8.0, none) == -1
    assert se(p, p, p, p, none, 1, 4, 2, 256, 96, 128, 64, 1, 0.0, 8.0, none) == -2
    assert se(p, p, p, p, none, 0, 4, 2, 256, 128, 128, 64, 1, 0.0, 8.0, none) == 0
    vf = lambda *a: L.vfa_attn_fwd(*a)
    base = (p, p, p, p, none, *ok_shape)
    assert vf(*base, 1, 1, 1, 0.0, none, 0, none) == -1                           # workspace missing
    assert vf(*base, 1, 1, 1, 0.0, p, 16, none) == -1                             # workspace too small
    assert vf(*base, -1, 1, 1, 0.0, p, 1 << 20, none) == -1                       # n_sink < 0
    assert vf(*base, 0, 0, 0, 0.0, p, 1 << 20, none) == -1                        # max would stay -inf
    assert vf(*base, 1, 1, 1, float("nan"), p, 1 << 20, none) == -1
    vs = lambda *a: L.vsa_attn_fwd(*a)
    assert vs(*base, 1, 1, 1, 0.0, 0.0, none, p, 1 << 20, none) == -1             # threshold must be > 0
    assert vs(*base, 1, 1, 1, 0.0, float("nan"), none, p, 1 << 20, none) == -1
    assert vs(*base, 1, 1, 1, 0.0, float("inf"), none, p, 1 << 20, none) == -1
    va = lambda *a: L.vfa_variant_fwd(*a)
    # after the shape: n_sink, n_local, use_minit, repr_mode, q_repr_mode, reorder, freeze, rowskip, tau, scale, threshold
    assert va(*base, 1, 1, 1, 4, 0, 1, 1, 0, -1.0, 0.0, 0.0, none, p, 1 << 20, none) == -1      # repr_mode out of range
    assert va(*base, 1, 1, 1, 0, 4, 1, 1, 0, -1.0, 0.0, 0.0, none, p, 1 << 20, none) == -1      # q_repr_mode out of range
    assert va(*base, 1, 1, 0, 0, 1, 1, 1, 0, -1.0, 0.0, 0.0, none, p, 1 << 20, none) == -1      # q_repr without m-init
    assert va(*base, 1, 1, 2, 0, 1, 1, 1, 0, -1.0, 0.0, 0.0, none, p, 1 << 20, none) == -1      # q_repr with caller's summaries
    assert va(*base, 1, 1, 1, 0, 2, 1, 1, 0, -1.0, 0.0, 0.0, none, p, 2048, none) == -1         # room for k_repr only
    assert va(*base, 0, 0, 0, 0, 0, 1, 1, 0, -1.0, 0.0, 0.0, none, p, 1 << 20, none) == -1      # frozen max would stay -inf
    assert va(*base, 0, 2, 0, 0, 0, 0, 1, 0, -1.0, 0.0, 0.0, none, p, 1 << 20, none) == -1      # ascending, no seed, no sink: first tile frozen at -inf
    assert va(*base, 1, 1, 1, 0, 0, 0, 0, 0, -1.0, 0.0, -1.0, none, p, 1 << 20, none) == -1     # negative threshold
    assert va(*base, 0, 0, 0, 0, 0, 0, 0, 1, -1.0, 0.0, 0.0, none, p, 1 << 20, none) == -1      # row skip without a threshold
    assert va(*base, 1, 1, 1, 0, 0, 1, 1, 1, -1.0, 0.0, 4.0, none, p, 1 << 20, none) == -1      # row skip needs freeze = 0
    assert va(*base, 0, 0, 0, 0, 0, 0, 0, 0, float("nan"), 0.0, 4.0, none, p, 1 << 20, none) == -1
    assert va(none, p, p, p, none, *ok_shape, 1, 1, 1, 0, 0, 0, 0, 0, -1.0, 0.0, 0.0, none, p, 1 << 20, none) == -1
    ap = lambda *a: L.vfa_kblock_summary_append(*a)
    assert ap(p, p, 1, 1, 256, 10, 5, 128, 64, none) == -1                          # n_new < n_old
    assert ap(p, p, 1, 1, 256, 0, 300, 128, 64, none) == -1                         # beyond the capacity
    assert ap(p, p, 1, 1, 256, 5, 5, 128, 64, none) == 0                            # nothing appended: no-op
    assert ap(none, p, 1, 1, 256, 0, 5, 128, 64, none) == -1
    dc = lambda *a: L.vfa_decode_fwd(*a)
    dshape = (1, 8, 2, 1024)                                                        # B, Hq, Hkv, n_cap
    assert dc(p, p, p, p, p, none, *dshape, 0, 128, 64, 1, 1, 1, 4, 0.0, p, 1 << 20, none) == -1     # no keys
    assert dc(p, p, p, p, p, none, *dshape, 2000, 128, 64, 1, 1, 1, 4, 0.0, p, 1 << 20, none) == -1  # n_keys > n_cap
    assert dc(p, p, p, p, p, none, *dshape, 100, 128, 64, 0, 0, 0, 4, 0.0, p, 1 << 20, none) == -1   # max would stay -inf
    assert dc(p, p, p, p, p, none, *dshape, 100, 128, 64, 1, 1, 1, 0, 0.0, p, 1 << 20, none) == -1   # n_splits < 1
    assert dc(p, p, p, p, p, none, *dshape, 100, 128, 64, 1, 1, 1, 4, 0.0, p, 64, none) == -1        # workspace too small
    assert dc(p, p, p, none, p, none, *dshape, 100, 128, 64, 1, 1, 1, 4, 0.0, p, 1 << 20, none) == -1  # summaries missing
    assert dc(p, p, p, p, p, none, 1, 64, 1, 1024, 100, 128, 64, 1, 1, 1, 4, 0.0, p, 1 << 22, none) == -2  # 64 heads per KV head
    assert dc(p, p, p, p, p, none, *dshape, 100, 128, 32, 1, 1, 1, 4, 0.0, p, 1 << 20, none) == -2   # block_n
    assert dc(p, p, p, p, p, none, 0, 8, 2, 1024, 100, 128, 64, 1, 1, 1, 4, 0.0, p, 1 << 20, none) == 0
    dv = lambda *a: L.vfa_decode_varlen_fwd(*a)
    assert dv(p, p, p, p, p, none, *dshape, none, 128, 64, 1, 1, 1, 4, 0.0, p, 1 << 20, none) == -1   # lengths missing
    assert dv(p, p, p, p, p, none, *dshape, ctypes.c_void_p(0x1002), 128, 64, 1, 1, 1, 4, 0.0, p, 1 << 20, none) == -1
    assert dv(p, p, p, p, p, none, 0, 8, 2, 1024, none, 128, 64, 1, 1, 1, 4, 0.0, p, 1 << 20, none) == 0
    assert L.vfa_kblock_summary_append_varlen(p, p, 1, 1, 256, none, p, 128, 64, none) == -1
    assert L.vfa_kblock_summary_append_varlen(p, p, 0, 1, 256, none, none, 128, 64, none) == 0
    assert pkg.decode_workspace_bytes(1, 8, 128, 4) >= 1 * 8 * 4 * 130 * 4
    f8 = lambda *a: L.vfa_fp8_attn_fwd(*a)
    f8shape = (1, 4, 2, 256, 128, 128, 64, 1)
    assert f8(1, p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, 1.0, 1.0, none, 0, none) == -1        # summaries need a workspace
    assert f8(1, p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 0.0, 1.0, 1.0, p, 1 << 20, none) == -1      # descale must be > 0
    assert f8(2, p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, 1.0, 1.0, p, 1 << 20, none) == -1      # frozen is 0 or 1
    assert f8(1, p, p, p, p, none, *f8shape, 0, 0, 0, 0.0, 1.0, 1.0, 1.0, p, 1 << 20, none) == -1      # max would stay -inf
    assert f8(0, p, p, p, p, none, 1, 4, 2, 256, 64, 128, 64, 1, 1, 1, 1, 0.0, 1.0, 1.0, 1.0, p, 1 << 20, none) == -2   # d = 64
    assert f8(0, none, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, 1.0, 1.0, p, 1 << 20, none) == -1
    assert f8(0, p, p, p, p, none, 0, 4, 2, 256, 128, 128, 64, 1, 1, 1, 1, 0.0, 1.0, 1.0, 1.0, none, 0, none) == 0
    nx = lambda *a: L.vfa_fp8_attn_noexp_fwd(*a)
    # descale_q * descale_k * scale * log2(e): 2^-3.5 * log2(e) is no power of two -> refused before any launch
    assert nx(p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, 1.0, 1.0, p, 1 << 20, none) == -1
    assert nx(p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, 1.0, 1.0, none, 0, none) == -1            # workspace missing
    assert nx(none, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, 1.0, 1.0, p, 1 << 20, none) == -1
    assert nx(p, p, p, p, none, 0, 4, 2, 256, 128, 128, 64, 1, 1, 1, 1, 0.0, 1.0, 1.0, 1.0, none, 0, none) == 0
    m4 = lambda *a: L.vfa_mxfp4_attn_fwd(*a)
    # frozen, Q4, QS, K4, KS, Vt8, O, LSE, shape, n_sink, n_local, use_minit, softmax_scale, descale_v, workspace, bytes, stream
    assert m4(1, p, p, p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, none, 0, none) == -1             # summaries need a workspace
    assert m4(1, p, p, p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, p, 256, none) == -1              # ... of 4 * 132 * 2 bytes
    assert m4(1, p, p, p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 0.0, p, 1 << 20, none) == -1          # descale_v must be > 0
    assert m4(2, p, p, p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, p, 1 << 20, none) == -1          # frozen is 0 or 1
    assert m4(1, p, p, p, p, p, p, none, *f8shape, 0, 0, 0, 0.0, 1.0, p, 1 << 20, none) == -1          # max would stay -inf
    assert m4(0, p, none, p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, p, 1 << 20, none) == -1       # scales missing
    assert m4(0, p, ctypes.c_void_p(0x1002), p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, p, 1 << 20, none) == -1
    assert m4(0, p, p, p, p, p, p, none, 1, 4, 2, 256, 64, 128, 64, 1, 1, 1, 1, 0.0, 1.0, p, 1 << 20, none) == -2   # d = 64
    assert m4(0, p, p, p, p, p, p, none, 0, 4, 2, 256, 128, 128, 64, 1, 1, 1, 1, 0.0, 1.0, none, 0, none) == 0
    mn = lambda *a: L.vfa_mxfp4_attn_noexp_fwd(*a)
    ln2 = 0.6931471805599453
    assert mn(p, p, p, p, p, p, none, *f8shape, 1, 1, 1, 0.0, 1.0, p, 1 << 20, none) == -1             # scale 2^-3.5: scores not in log2 units
    assert mn(p, p, p, p, p, p, none, *f8shape, 1, 1, 1, ln2, 1.0, none, 0, none) == -1                 # workspace missing
    assert mn(p, p, p, p, p, p, none, 0, 4, 2, 256, 128, 128, 64, 1, 1, 1, 1, ln2, 1.0, none, 0, none) == 0
    assert L.vfa_mxfp4_quantize(p, p, p, 48, 1.0, none) == -1                                         # not a multiple of 32
    assert L.vfa_mxfp4_quantize(p, p, p, 64, 0.0, none) == -1
    assert L.vfa_mxfp4_quantize(p, none, p, 64, 1.0, none) == -1
    assert L.vfa_mxfp4_quantize(p, p, p, 0, 1.0, none) == 0
    assert L.vfa_mxfp4_workspace_bytes(1, 2, 256) == 1280 and L.vfa_mxfp4_workspace_bytes(0, 2, 256) == 0
    assert L.vfa_fp8_quantize(p, p, 12, 1.0, none) == -1                                              # not a multiple of 8
    assert L.vfa_fp8_quantize(p, p, 16, -1.0, none) == -1
    assert L.vfa_fp8_quantize(p, p, 0, 1.0, none) == 0
    assert L.vfa_fp8_pack_v(p, p, 1, 1, 64, 64, 1.0, none) == -2
    assert L.vfa_fp8_pack_v(none, p, 1, 1, 64, 128, 1.0, none) == -1
    assert L.vfa_fp8_v_bytes(2, 4, 100) == 2 * 4 * 2 * 8192
    assert L.vfa_kblock_summary_mode(p, p, 1, 1, 64, 128, 64, 7, none) == -1
    assert L.vfa_kblock_summary_mode(none, p, 1, 1, 64, 128, 64, 2, none) == -1
    assert L.vfa_kblock_summary(none, p, 1, 1, 64, 128, 64, none) == -1
    assert L.vfa_kblock_summary(p, p, 1, 1, 64, 100, 64, none) == -2
    assert L.vfa_kblock_summary(p, p, 0, 1, 64, 128, 64, none) == 0
