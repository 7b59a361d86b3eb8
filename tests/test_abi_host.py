"""C-ABI library on the host (no GPU): it loads, exports every symbol the header declares,
and rejects bad arguments before touching HIP."""
import ctypes
import pathlib
import re

import pytest

from paper_2507_00394_amd import binding as hx

ROOT = pathlib.Path(__file__).resolve().parents[1]


@pytest.fixture(scope="module")
def L():
    if not hx.LIB_PATH.exists():
        from paper_2507_00394_amd import build

        build.build()
    return hx.lib()


def declared_functions():
    text = (ROOT / "include" / "helix_attn.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(helix_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert set(names) == set(hx.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_status_strings(L):
    assert L.helix_attn_version() >= 100
    seen = {hx.status_string(s) for s in range(10)}
    assert len(seen) == 10 and hx.status_string(0) == "ok" and hx.status_string(99) == "unknown status"


def test_workspace_bytes(L):
    # two fp32 planes [B, H, S] (-delta and lse * log2(e)), each padded to 256 bytes
    assert hx.helix_attn_bwd_workspace_bytes(1, 2, 512, 64) == 2 * 4096
    assert hx.helix_attn_bwd_workspace_bytes(1, 1, 1, 64) == 2 * 256
    assert hx.helix_attn_bwd_workspace_bytes(1, 32, 131072, 128) == 2 * 32 * 131072 * 4
    assert hx.helix_attn_bwd_workspace_bytes(1, 1, 10, 96) == 0
    assert hx.helix_attn_bwd_workspace_bytes(0, 1, 10, 64) == 0


def test_validation_precedes_any_device_work(L):
    """Fake but aligned addresses: every call must fail in validation, never reach a launch."""
    p = ctypes.c_void_p(0x10000)
    odd = ctypes.c_void_p(0x10008)
    fwd = lambda **kw: L.helix_attn_fwd(kw.get("q", p), p, p, kw.get("o", p), kw.get("lse", p), kw.get("B", 1), kw.get("H", 1),
                                         kw.get("S", 8), kw.get("D", 64), kw.get("scale", 0.1), 1, None)
    assert fwd(q=None) == 1 and fwd(o=None) == 1 and fwd(lse=None) == 1
    assert fwd(B=0) == 2 and fwd(S=0) == 2 and fwd(H=-3) == 2 and fwd(S=(1 << 24) + 1) == 2
    assert fwd(D=96) == 3 and fwd(D=256) == 3
    assert fwd(q=odd) == 4 and fwd(lse=ctypes.c_void_p(0x10002)) == 4
    assert fwd(scale=0.0) == 5 and fwd(scale=-1.0) == 5 and fwd(scale=float("nan")) == 5 and fwd(scale=float("inf")) == 5
    bwd = lambda ws=p, wsb=1 << 20, **kw: L.helix_attn_bwd(p, p, p, p, p, kw.get("dO", p), p, p, kw.get("dv", p), ws, wsb, 1, 2, 512,
                                                          kw.get("D", 64), kw.get("scale", 0.1), 1, None)
    assert bwd(dO=None) == 1 and bwd(dv=None) == 1 and bwd(ws=None) == 1
    assert bwd(ws=ctypes.c_void_p(0x10010)) == 4
    assert bwd(wsb=4095) == 6
    assert bwd(D=32) == 3 and bwd(scale=0.0) == 5
    # the allocation-free variant validates the same way and refuses shapes beyond its built-in scratch
    static = lambda **kw: L.helix_attn_bwd_static(p, p, p, p, p, kw.get("dO", p), p, p, kw.get("dv", p), kw.get("B", 1), kw.get("H", 2),
                                                  kw.get("S", 512), kw.get("D", 64), kw.get("scale", 0.1), 1, None)
    assert static(dO=None) == 1 and static(dv=odd) == 4 and static(D=32) == 3 and static(scale=0.0) == 5 and static(S=0) == 2
    assert static(B=1, H=32, S=131072 + 64, D=128) == 9 and static(B=2, H=40, S=65536, D=128) == 9
    assert "4194304" in hx.status_string(9)
    assert bwd(wsb=2 * 4096 - 1) == 6 and bwd(wsb=2 * 4096) != 6     # two fp32 planes of B*H*S rows
    assert L.helix_attn_bwd_workspace_bytes(1, 2, 512, 64) == 2 * 4096
    assert L.helix_attn_bwd_workspace_bytes(1, 1, 3, 64) == 2 * 256  # each plane padded to 256 bytes
    assert L.helix_attn_bwd_preprocess(p, None, p, p, 1, 1, 8, 64, None) == 1
    assert L.helix_attn_bwd_preprocess(p, p, p, ctypes.c_void_p(0x10010), 1, 1, 8, 64, None) == 4   # stats need 256 bytes
    assert L.helix_attn_bwd_delta_head(p, p, p, p, p, p, -1, 1, 1, 8, 64, 0.1, 1, None) == 2
    assert L.helix_attn_bwd_dkdv(p, p, p, p, p, p, odd, 1, 1, 8, 64, 0.1, 1, None) == 4
    assert L.helix_attn_bwd_dkdv(p, p, p, p, None, p, p, 1, 1, 8, 64, 0.1, 1, None) == 1
    assert L.helix_attn_bwd_dq(p, p, p, p, p, p, 1, 1, 8, 128, -0.1, 1, None) == 5


def test_mfma_probe_validation(L):
    p = ctypes.c_void_p(0x10000)
    flops = ctypes.c_longlong(-1)
    call = lambda sink=p, wg=4, it=10, out=ctypes.byref(flops): L.helix_mfma_probe(sink, wg, it, 1, out, None)
    assert call(sink=None) == 1 and call(out=None) == 1
    assert call(sink=ctypes.c_void_p(0x10002)) == 4
    assert call(wg=0) == 2 and call(it=0) == 2 and call(wg=(1 << 20) + 1) == 2 and call(it=(1 << 24) + 1) == 2
    assert flops.value == -1          # nothing was written by a refused call
    mix = lambda sink=p, wg=4, it=10, out=ctypes.byref(flops): L.helix_mfma_mix_probe(sink, wg, it, 0, out, None)
    assert mix(sink=None) == 1 and mix(out=None) == 1 and mix(sink=ctypes.c_void_p(0x10002)) == 4
    assert mix(wg=0) == 2 and mix(it=0) == 2 and mix(wg=(1 << 20) + 1) == 2 and flops.value == -1


def test_stride_validation(L):
    """Strided entry points: the stride rules of the header, checked on the host."""
    p = ctypes.c_void_p(0x10000)
    B, H, S, D = 2, 4, 96, 64
    st = lambda b, h, r: ctypes.byref(hx.helix_strides(b, h, r))
    good = {
        "contiguous": st(H * S * D, S * D, D),
        "seq_major": st(H * D, D, B * H * D),                  # [S, B, H, D] viewed as [B, H, S, D]
        "fused_qkv": st(3 * H * D, D, B * 3 * H * D),          # a third of an [S, B, 3*H*D] buffer
        "interleaved_qkv": st(H * 3 * D, 3 * D, B * H * 3 * D),  # [S, B, H, 3*D]
        "padded_rows": st(H * S * (D + 8), S * (D + 8), D + 8),
    }
    def fwd(sq=None, so=None, **kw):
        return L.helix_attn_fwd_strided(kw.get("q", p), sq, p, None, p, None, p, so, p, B, H, S, kw.get("D", D), 0.1, 1, None)
    bad = {
        "row_below_D": st(H * S * D, S * D, D - 8),
        "not_multiple_of_8": st(H * S * D + 4, S * D, D),
        "negative": st(-H * S * D, S * D, D),
        "heads_overlap_rows": st(H * S * D, D, D),             # head stride inside the span of the rows
        "batch_overlaps": st(S * D, S * D, D),                  # batch and head strides coincide
        "row_too_large": st(0, 0, (1 << 24) + 8),
    }
    for name, s_ in bad.items():
        assert fwd(sq=s_) == 8, name
        assert fwd(so=s_) == 8, name
    assert fwd(sq=bad["row_below_D"], q=None) == 1              # pointer checks come first
    assert fwd(sq=bad["row_below_D"], D=96) == 3                # then the shape
    for name, s_ in good.items():
        assert L.helix_attn_check_strides(s_, B, H, S, D) == 0, name
    for name, s_ in bad.items():
        assert L.helix_attn_check_strides(s_, B, H, S, D) == 8, name
    assert L.helix_attn_check_strides(None, B, H, S, D) == 0
    assert L.helix_attn_check_strides(None, B, H, S, 80) == 3
    # extent-1 dimensions may carry any (aligned) stride, as torch views of size 1 do
    assert hx.helix_attn_check_strides((0, 64, 128), 1, 2, 96, 64) == 0
    assert hx.helix_attn_check_strides((8, 8, 64), 1, 1, 96, 64) == 0
    bwd = lambda s_, ws=1 << 20: L.helix_attn_bwd_strided(p, None, p, None, p, None, p, None, p, p, None, p, None, p, s_,
                                                         p, None, p, ws, B, H, S, D, 0.1, 1, None)
    assert bwd(bad["heads_overlap_rows"]) == 8 and bwd(bad["negative"]) == 8
    assert bwd(good["seq_major"], ws=16) == 6                   # workspace size is checked before the strides


def test_linear_layer_validation(L):
    p = ctypes.c_void_p(0x10000)
    fwd = lambda M=64, K=128, N=256, lda=128, ldw=256, ldo=256, a=p: L.helix_qkv_linear_fwd(a, lda, p, ldw, p, ldo, M, K, N, None)
    assert fwd(a=None) == 1 and fwd(a=ctypes.c_void_p(0x10008)) == 4
    assert fwd(M=0) == 2 and fwd(K=96) == 2 and fwd(N=200) == 2
    assert fwd(lda=120) == 8 and fwd(ldw=260) == 8 and fwd(ldo=(1 << 23) + 8) == 8
    bwd = lambda M=4096, ws=p, wsb=1 << 30, ldda=128: L.helix_qkv_linear_bwd(p, 128, p, 128, p, 128, p, ldda, p, 128, ws, wsb, M, 128, 128, None)
    assert bwd(M=4100) == 2                       # the weight gradient contracts over M in stages of 32
    assert bwd(ldda=64) == 8
    need = hx.helix_qkv_linear_bwd_workspace_bytes(4096, 128, 128)
    assert need == 128 * 128 * 2 + 2 * 128 * 128 * 4   # w^T, then two parts of 2048 tokens
    assert bwd(ws=None) == 1 and bwd(ws=ctypes.c_void_p(0x10010)) == 4 and bwd(wsb=need - 1) == 6
    assert hx.helix_qkv_linear_bwd_workspace_bytes(1024, 128, 128) == 128 * 128 * 2     # too few tokens to split: w^T only
    assert hx.helix_qkv_linear_bwd_workspace_bytes(131072, 4096, 1536) == 4096 * 1536 * 2 + 6 * 4096 * 1536 * 4
    assert hx.helix_qkv_linear_bwd_workspace_bytes(4096, 100, 128) == 0      # invalid shape


def test_binding_refuses_cpu_tensors(L):
    import torch

    x = torch.zeros(1, 1, 8, 64, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        hx.helix_attn_fwd(x, x, x, x, torch.zeros(1, 1, 8), 0.1)
