"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its argument validation and workspace planning work without a GPU (no compute calls)."""
import ctypes
import os
import re

import pytest

from paper_2509_24899_amd import hybrid_attn as ha
from paper_2509_24899_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000  # 4 KiB-aligned, never dereferenced by the host-side checks


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ha.LIB_PATH):
        from paper_2509_24899_amd.build import build_library
        build_library()
    return ha._lib()


def _problem(B=1, H=12, N=32760, d=128, dtype=ha.HA_BF16, bs=128, R=4, scale=None, strides=None, g=0, causal=0, window=0,
             reserved=0):
    sb, sh, sn = strides if strides else (H * N * d, N * d, d)
    return ha.ha_problem(B, H, N, d, dtype, bs, R, scale if scale is not None else d ** -0.5, sb, sh, sn, g, causal, window, reserved)


def _map(Hd=128, F=128, P=2, act=ha.HA_ACT_SOFTMAX, w1=FAKE, w2=FAKE + 0x100000, b1=None, b2=None):
    return ha.ha_feature_map(w1, b1, w2, b2, Hd, F, P, act)


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "hybrid_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(hybrid_attn_\w+)\s*\(", text)
    assert len(set(names)) == 19
    for n in set(names):
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
    assert ha.hybrid_attn_abi_version() == 7


def test_struct_layout_matches_header():
    # 7 int32 + float, then three int64 at offset 32; four pointers, four int32, two pointers, two int32
    assert ha.ha_problem.stride_b.offset == 32 and ctypes.sizeof(ha.ha_problem) == 72 and ha.ha_problem.split_granularity.offset == 56 and ha.ha_problem.local_window.offset == 64
    assert ha.ha_feature_map.d_hidden.offset == 32 and ha.ha_feature_map.w_mid.offset == 48 and ctypes.sizeof(ha.ha_feature_map) == 72


def test_valid_problems(lib):
    fm = _map()
    assert ha.hybrid_attn_validate(_problem(), fm, fm) == ha.HA_OK
    assert ha.hybrid_attn_validate(_problem(R=1), None, None) == ha.HA_OK           # full softmax needs no phi
    assert ha.hybrid_attn_validate(_problem(R=0), fm, fm) == ha.HA_OK
    assert ha.hybrid_attn_validate(_problem(R=3), fm, fm) == ha.HA_OK               # Fig. "method" uses rate 3
    # block-granular variant of the split: any group size up to N; fewer softmax keys to stage when groups are cut short
    assert ha.hybrid_attn_validate(_problem(g=128), fm, fm) == ha.HA_OK
    assert ha.hybrid_attn_validate(_problem(g=32760), fm, fm) == ha.HA_OK
    assert ha.hybrid_attn_validate(_problem(g=-1), fm, fm) == ha.HA_ERR_SHAPE
    assert ha.hybrid_attn_validate(_problem(g=32761), fm, fm) == ha.HA_ERR_SHAPE
    # chunk-causal variant: whole query tiles per chunk, fused feature-map kernels only, forward only
    assert ha.hybrid_attn_validate(_problem(causal=1536), fm, fm) == ha.HA_OK
    assert ha.hybrid_attn_validate(_problem(causal=128, bs=64), fm, fm) == ha.HA_OK
    assert ha.hybrid_attn_validate(_problem(causal=128), fm, fm) == ha.HA_ERR_UNSUPPORTED
    assert ha.hybrid_attn_validate(_problem(causal=1560), fm, fm) == ha.HA_ERR_UNSUPPORTED
    assert ha.hybrid_attn_validate(_problem(causal=-256), fm, fm) == ha.HA_ERR_SHAPE
    assert ha.hybrid_attn_validate(_problem(causal=1536), _map(256, 256), _map(256, 256)) == ha.HA_OK
    assert ha.hybrid_attn_validate(_problem(causal=1536), _map(384, 384, 3), _map(384, 384, 3)) == ha.HA_ERR_UNSUPPORTED
    assert ha.hybrid_attn_validate(_problem(causal=1536, R=1), None, None) == ha.HA_OK
    # local-window variant: rate 0 plus a window of whole query tiles; the other variants stay off
    assert ha.hybrid_attn_validate(_problem(R=0, window=1024), fm, fm) == ha.HA_OK
    assert ha.hybrid_attn_validate(_problem(R=0, window=128, bs=64), fm, fm) == ha.HA_OK
    assert ha.hybrid_attn_validate(_problem(R=4, window=1024), fm, fm) == ha.HA_ERR_SHAPE
    assert ha.hybrid_attn_validate(_problem(R=0, window=1024, causal=1024), fm, fm) == ha.HA_ERR_SHAPE
    assert ha.hybrid_attn_validate(_problem(R=0, window=1024, g=8), fm, fm) == ha.HA_ERR_SHAPE
    assert ha.hybrid_attn_validate(_problem(R=0, window=1000), fm, fm) == ha.HA_ERR_UNSUPPORTED
    assert ha.hybrid_attn_validate(_problem(R=0, window=-1), fm, fm) == ha.HA_ERR_SHAPE
    assert ha.hybrid_attn_validate(_problem(reserved=1), fm, fm) == ha.HA_ERR_SHAPE
    assert ha.hybrid_attn_validate(_problem(R=0, window=1024), _map(384, 384, 3), _map(384, 384, 3)) == ha.HA_ERR_UNSUPPORTED
    # one prefix state per chunk
    assert ha.hybrid_attn_workspace_bytes(_problem(causal=4096), fm, fm) > ha.hybrid_attn_workspace_bytes(_problem(), fm, fm)
    assert lib.hybrid_attn_value_distill_workspace_bytes(ctypes.byref(_problem(causal=4096)), ctypes.byref(fm), ctypes.byref(fm)) > 0
    assert ha.hybrid_attn_validate(_problem(N=75600, R=75600, g=75600), fm, fm) == ha.HA_ERR_UNSUPPORTED    # R g beyond 2^30
    assert ha.hybrid_attn_workspace_bytes(_problem(g=1), fm, fm) == ha.hybrid_attn_workspace_bytes(_problem(), fm, fm)
    fm64 = _map(64, 64)
    assert ha.hybrid_attn_validate(_problem(H=2, N=1024, d=64, dtype=ha.HA_F32, bs=64), fm64, fm64) == ha.HA_OK
    wide = _map(256, 256)
    assert ha.hybrid_attn_validate(_problem(), wide, wide) == ha.HA_OK              # Tab. "phi" default widths
    bnhd = _problem(strides=(32760 * 12 * 128, 128, 12 * 128))                       # [B, N, H, d] memory
    assert ha.hybrid_attn_validate(bnhd, fm, fm) == ha.HA_OK


@pytest.mark.parametrize("kw,status", [
    (dict(N=0), ha.HA_ERR_SHAPE), (dict(B=0), ha.HA_ERR_SHAPE), (dict(H=-1), ha.HA_ERR_SHAPE),
    (dict(R=-1), ha.HA_ERR_SHAPE), (dict(R=40000), ha.HA_ERR_SHAPE),
    (dict(scale=0.0), ha.HA_ERR_SHAPE), (dict(scale=-1.0), ha.HA_ERR_SHAPE), (dict(scale=float("nan")), ha.HA_ERR_SHAPE),
    (dict(d=96), ha.HA_ERR_UNSUPPORTED), (dict(bs=32), ha.HA_ERR_UNSUPPORTED), (dict(dtype=7), ha.HA_ERR_UNSUPPORTED),
    (dict(strides=(12 * 32760 * 128, 32760 * 128, 64)), ha.HA_ERR_SHAPE),           # rows overlap
    (dict(strides=(12 * 32760 * 132, 32760 * 132, 132)), ha.HA_ERR_ALIGN),          # 132*2 B is not 16-byte
])
def test_problem_errors(lib, kw, status):
    fm = _map()
    assert ha.hybrid_attn_validate(_problem(**kw), fm, fm) == status


def test_feature_map_errors(lib):
    p, fm = _problem(), _map()
    assert ha.hybrid_attn_validate(None, fm, fm) == ha.HA_ERR_NULL
    assert ha.hybrid_attn_validate(p, None, fm) == ha.HA_ERR_NULL
    assert ha.hybrid_attn_validate(p, fm, None) == ha.HA_ERR_NULL
    assert ha.hybrid_attn_validate(p, _map(w1=None), fm) == ha.HA_ERR_NULL
    assert ha.hybrid_attn_validate(p, fm, _map(P=3)) == ha.HA_ERR_SHAPE             # 3 does not divide 128
    assert ha.hybrid_attn_validate(p, fm, _map(P=0)) == ha.HA_ERR_SHAPE
    assert ha.hybrid_attn_validate(p, fm, _map(P=16)) == ha.HA_ERR_UNSUPPORTED
    assert ha.hybrid_attn_validate(p, fm, _map(act=9)) == ha.HA_ERR_UNSUPPORTED
    assert ha.hybrid_attn_validate(p, fm, _map(Hd=96)) == ha.HA_ERR_UNSUPPORTED
    assert ha.hybrid_attn_validate(p, fm, _map(256, 256)) == ha.HA_ERR_SHAPE        # phi_q / phi_k widths differ
    assert ha.hybrid_attn_validate(p, fm, _map(P=4)) == ha.HA_ERR_SHAPE             # degrees differ
    assert ha.hybrid_attn_validate(p, _map(w1=FAKE + 2), fm) == ha.HA_ERR_ALIGN
    assert ha.hybrid_attn_validate(p, _map(b1=FAKE + 1), fm) == ha.HA_ERR_ALIGN


def test_forward_rejects_bad_buffers_before_any_device_work(lib):
    p, fm = _problem(N=4096), _map()
    need = ha.hybrid_attn_workspace_bytes(p, fm, fm)
    f = lib.hybrid_attn_forward
    pq = ctypes.byref(fm)
    args_ok = [FAKE, FAKE + (1 << 30), FAKE + (2 << 30), pq, pq, FAKE + (3 << 30), FAKE + (4 << 30), need, None]
    bad = list(args_ok); bad[0] = None
    assert f(ctypes.byref(p), *bad) == ha.HA_ERR_NULL
    bad = list(args_ok); bad[5] = None
    assert f(ctypes.byref(p), *bad) == ha.HA_ERR_NULL
    bad = list(args_ok); bad[1] = FAKE + 8
    assert f(ctypes.byref(p), *bad) == ha.HA_ERR_ALIGN
    bad = list(args_ok); bad[6] = None
    assert f(ctypes.byref(p), *bad) == ha.HA_ERR_WORKSPACE
    bad = list(args_ok); bad[7] = need - 1
    assert f(ctypes.byref(p), *bad) == ha.HA_ERR_WORKSPACE
    bad = list(args_ok); bad[6] = FAKE + (4 << 30) + 16
    assert f(ctypes.byref(p), *bad) == ha.HA_ERR_ALIGN


def test_workspace_bytes(lib):
    fm = _map()
    assert ha.hybrid_attn_workspace_bytes(_problem(d=96), fm, fm) == 0
    w = W.WAN_480P_81F
    p = _problem()
    need = ha.hybrid_attn_workspace_bytes(p, fm, fm)
    ns_pad = -(-w.n_softmax // 128) * 128
    compact = 2 * w.B * w.H * ns_pad * w.d * 2                   # K_S and V_S in bf16, padded to key tiles
    assert compact <= need <= compact + 64 * 2 ** 20             # weights, partial states, S, z stay small
    assert ha.hybrid_attn_workspace_bytes(_problem(R=1), None, None) >= 2 * 12 * 32768 * 128 * 2
    assert ha.hybrid_attn_workspace_bytes(_problem(R=0), fm, fm) < 64 * 2 ** 20
    # more softmax keys -> more workspace
    sizes = [ha.hybrid_attn_workspace_bytes(_problem(R=R), fm, fm) for R in (16, 8, 4, 2)]
    assert sizes == sorted(sizes)


def test_status_strings(lib):
    seen = {ha.hybrid_attn_status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert ha.hybrid_attn_last_device_error() == 0


def test_binding_refuses_cpu_tensors(lib):
    import torch
    q = torch.zeros(1, 2, 64, 64)
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        ha.hybrid_attn_forward(q, q, q, None, None, 1)


def test_flop_and_byte_counts():
    assert abs(W.algorithmic_flops(W.WAN_480P_81F) / 1e9 - 1716.2) < 0.1
    assert abs(W.algorithmic_flops(W.WAN_480P_161F) / 1e9 - 3283.5) < 0.1
    assert abs(W.algorithmic_flops(W.TINY) / 1e9 - 0.223) < 1e-3
    assert abs(W.algorithmic_flops(W.with_rate(W.WAN_480P_81F, 0)) / 1e9 - 77.4) < 0.1
    assert W.WAN_480P_81F.n_softmax == 8190 and W.WAN_480P_161F.n_softmax == 7995


def test_mfma_probe_rejects_bad_arguments_on_the_host(lib):
    flops = ctypes.c_double(0.0)
    f = lib.hybrid_attn_mfma_probe
    assert f(1, 100, 1, None, 1 << 20, ctypes.byref(flops), None) == ha.HA_ERR_NULL
    assert f(1, 100, 1, FAKE, 1 << 20, None, None) == ha.HA_ERR_NULL
    assert f(1, 0, 1, FAKE, 1 << 20, ctypes.byref(flops), None) == ha.HA_ERR_SHAPE
    assert f(1, 100, 0, FAKE, 1 << 20, ctypes.byref(flops), None) == ha.HA_ERR_SHAPE
    assert f(1, 100, 1, FAKE + 4, 1 << 20, ctypes.byref(flops), None) == ha.HA_ERR_ALIGN


def test_value_distill_workspace_and_errors(lib):
    fm = _map()
    p = _problem()
    fwd = lib.hybrid_attn_workspace_bytes(ctypes.byref(p), ctypes.byref(fm), ctypes.byref(fm))
    both = lib.hybrid_attn_value_distill_workspace_bytes(ctypes.byref(p), ctypes.byref(fm), ctypes.byref(fm))
    teacher = _problem(R=1)
    fwd_teacher = lib.hybrid_attn_workspace_bytes(ctypes.byref(teacher), None, None)
    assert both >= max(fwd, fwd_teacher) + 12 * 64 * 8          # the larger forward plus the reduction partials
    assert lib.hybrid_attn_value_distill_workspace_bytes(ctypes.byref(_problem(N=0)), ctypes.byref(fm), ctypes.byref(fm)) == 0
    f = lib.hybrid_attn_value_distill_loss
    A = [FAKE + i * 0x10000000 for i in range(8)]
    args = lambda **kw: [ctypes.byref(kw.get("p", p)), A[0], A[1], A[2], ctypes.byref(fm), ctypes.byref(fm), 0,
                         kw.get("yt", A[3]), kw.get("ys", A[4]), kw.get("loss", A[5]), kw.get("ws", A[6]),
                         kw.get("wsb", both), None]
    assert f(*args(yt=None)) == ha.HA_ERR_NULL
    assert f(*args(loss=None)) == ha.HA_ERR_NULL
    assert f(*args(ys=A[3])) == ha.HA_ERR_SHAPE               # teacher and student outputs must be distinct
    assert f(*args(loss=A[5] + 4)) == ha.HA_ERR_ALIGN
    assert f(*args(wsb=both - 1)) == ha.HA_ERR_WORKSPACE
    assert f(*args(ws=None)) == ha.HA_ERR_WORKSPACE
    assert f(*args(p=_problem(d=96))) == ha.HA_ERR_UNSUPPORTED


def test_value_distill_grad_workspace_and_errors(lib):
    """Host-side checks of the gradient entry point: every error is reported before anything is enqueued."""
    fm = _map()
    p = _problem()
    loss_ws = lib.hybrid_attn_value_distill_workspace_bytes(ctypes.byref(p), ctypes.byref(fm), ctypes.byref(fm))
    need = lib.hybrid_attn_value_distill_grad_workspace_bytes(ctypes.byref(p), ctypes.byref(fm), ctypes.byref(fm))
    # beyond the loss's workspace: the sign tensor (one bf16 per element of q) and the partial tiles, at least
    assert need >= loss_ws + 12 * 32760 * 128 * 2
    # two-layer maps of the other supported widths go pass by pass and bring image buffers of their own
    wide = _map(256, 256)
    assert lib.hybrid_attn_value_distill_grad_workspace_bytes(ctypes.byref(p), ctypes.byref(wide), ctypes.byref(wide)) > need
    three = ha.ha_feature_map(FAKE, None, FAKE + 0x100000, None, 768, 768, 6, ha.HA_ACT_SOFTMAX, FAKE + 0x200000, None, 768, 0)
    f = lib.hybrid_attn_value_distill_grad
    A = [FAKE + i * 0x10000000 for i in range(16)]
    gq = ha.ha_feature_map_grad(A[8], A[9], A[10], A[11])
    gk = ha.ha_feature_map_grad(A[12], A[13], A[14], A[15])

    def args(**kw):
        return [ctypes.byref(kw.get("p", p)), A[0], A[1], A[2], ctypes.byref(kw.get("fq", fm)), ctypes.byref(kw.get("fk", fm)),
                0, 0, kw.get("yt", A[3]), kw.get("ys", A[4]), kw.get("den", A[5]), kw.get("loss", A[6]),
                ctypes.byref(kw.get("gq", gq)), ctypes.byref(kw.get("gk", gk)), kw.get("ws", A[7]), kw.get("wsb", need), None]
    assert f(*args(den=None)) == ha.HA_ERR_NULL
    assert f(*args(loss=None)) == ha.HA_ERR_NULL
    assert f(*args(gq=ha.ha_feature_map_grad(A[8], None, A[10], A[11]))) == ha.HA_ERR_NULL
    assert f(*args(gk=ha.ha_feature_map_grad(A[12], A[13], A[14] + 2, A[15]))) == ha.HA_ERR_ALIGN
    assert f(*args(ys=A[3])) == ha.HA_ERR_SHAPE
    assert f(*args(den=A[5] + 2)) == ha.HA_ERR_ALIGN
    assert f(*args(wsb=need - 1)) == ha.HA_ERR_WORKSPACE
    assert f(*args(ws=None)) == ha.HA_ERR_WORKSPACE
    assert f(*args(fq=three, fk=three)) == ha.HA_ERR_NULL           # a three-layer map needs w_mid, b_mid gradient buffers
    assert f(*args(fq=three, fk=wide)) == ha.HA_ERR_SHAPE
    assert ctypes.sizeof(ha.ha_feature_map_grad) == 48 and ha.ha_feature_map_grad.w_mid.offset == 32
    assert f(*args(fq=wide, fk=wide)) == ha.HA_ERR_WORKSPACE        # supported, but `need` was sized for the narrow map
    assert f(*args(fq=wide, fk=fm)) == ha.HA_ERR_SHAPE
    assert f(*args(p=_problem(d=96))) == ha.HA_ERR_UNSUPPORTED
    # rate 1: the maps are still required (they give the gradients their shapes)
    p1 = _problem(R=1)
    a = args(p=p1)
    a[4] = None
    assert f(*a) == ha.HA_ERR_NULL


def test_wider_and_three_layer_maps_validate(lib):
    """Host checks of the layer-by-layer path's shapes (Tab. "phi" rows beyond P = 2)."""
    p = _problem()
    for width in (384, 512, 768):
        fm = _map(width, width, width // 128)
        assert ha.hybrid_attn_validate(p, fm, fm) == ha.HA_OK
        assert lib.hybrid_attn_workspace_bytes(ctypes.byref(p), ctypes.byref(fm), ctypes.byref(fm)) > \
            lib.hybrid_attn_workspace_bytes(ctypes.byref(p), ctypes.byref(_map()), ctypes.byref(_map()))
    mixed = _map(384, 512)
    assert ha.hybrid_attn_validate(p, mixed, mixed) == ha.HA_OK
    assert ha.hybrid_attn_validate(p, _map(896, 896), _map(896, 896)) == ha.HA_ERR_UNSUPPORTED     # beyond 768
    assert ha.hybrid_attn_validate(p, _map(320, 320), _map(320, 320)) == ha.HA_ERR_UNSUPPORTED     # not a multiple of 128
    assert ha.hybrid_attn_validate(_problem(H=2, N=1024, d=64, dtype=ha.HA_F32, bs=64), _map(128, 128), _map(128, 128)) == \
        ha.HA_ERR_UNSUPPORTED                                                                      # wide maps need d_head = 128
    three = ha.ha_feature_map(FAKE, None, FAKE + 0x100000, None, 768, 768, 6, ha.HA_ACT_SOFTMAX, FAKE + 0x200000, None, 768, 0)
    assert ha.hybrid_attn_validate(p, three, three) == ha.HA_OK
    assert ha.hybrid_attn_validate(p, three, _map(768, 768, 6)) == ha.HA_ERR_SHAPE                 # depths differ
    bad = ha.ha_feature_map(FAKE, None, FAKE + 0x100000, None, 768, 768, 6, ha.HA_ACT_SOFTMAX, FAKE + 0x200000, None, 0, 0)
    assert ha.hybrid_attn_validate(p, bad, bad) == ha.HA_ERR_SHAPE
    odd = ha.ha_feature_map(FAKE, None, FAKE + 0x100000, None, 768, 768, 6, ha.HA_ACT_SOFTMAX, FAKE + 0x200000, None, 192, 0)
    assert ha.hybrid_attn_validate(p, odd, odd) == ha.HA_ERR_UNSUPPORTED
    # the gradient entry point takes them too
    assert lib.hybrid_attn_value_distill_grad_workspace_bytes(ctypes.byref(p), ctypes.byref(three), ctypes.byref(three)) > \
        lib.hybrid_attn_value_distill_workspace_bytes(ctypes.byref(p), ctypes.byref(three), ctypes.byref(three))


def test_param_update_host_errors(lib):
    """Host-side checks of the parameter update (Alg. 1's update line): every error is reported before anything is enqueued."""
    f = lib.hybrid_attn_param_update
    A = [FAKE + i * 0x1000000 for i in range(6)]
    assert ctypes.sizeof(ha.ha_optimizer) == 32

    def opt(**kw):
        d = dict(kind=ha.HA_OPT_ADAMW, step=1, lr=1e-3, grad_scale=1.0, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
        d.update(kw)
        return ctypes.byref(ha.ha_optimizer(d["kind"], d["step"], d["lr"], d["grad_scale"], d["beta1"], d["beta2"], d["eps"],
                                            d["weight_decay"]))
    assert f(None, 8, A[0], A[1], A[2], A[3], A[4], ha.HA_BF16, None) == ha.HA_ERR_NULL
    assert f(opt(), 8, None, A[1], A[2], A[3], A[4], ha.HA_BF16, None) == ha.HA_ERR_NULL
    assert f(opt(), 8, A[0], None, A[2], A[3], A[4], ha.HA_BF16, None) == ha.HA_ERR_NULL
    assert f(opt(), 8, A[0], A[1], None, A[3], A[4], ha.HA_BF16, None) == ha.HA_ERR_NULL          # AdamW needs its moments
    assert f(opt(kind=2), 8, A[0], A[1], A[2], A[3], A[4], ha.HA_BF16, None) == ha.HA_ERR_UNSUPPORTED
    assert f(opt(), 8, A[0], A[1], A[2], A[3], A[4], 7, None) == ha.HA_ERR_UNSUPPORTED
    assert f(opt(step=0), 8, A[0], A[1], A[2], A[3], A[4], ha.HA_BF16, None) == ha.HA_ERR_SHAPE
    assert f(opt(beta2=1.0), 8, A[0], A[1], A[2], A[3], A[4], ha.HA_BF16, None) == ha.HA_ERR_SHAPE
    assert f(opt(lr=-1.0), 8, A[0], A[1], A[2], A[3], A[4], ha.HA_BF16, None) == ha.HA_ERR_SHAPE
    assert f(opt(lr=float("nan")), 8, A[0], A[1], A[2], A[3], A[4], ha.HA_BF16, None) == ha.HA_ERR_SHAPE
    assert f(opt(), 8, A[0] + 2, A[1], A[2], A[3], A[4], ha.HA_BF16, None) == ha.HA_ERR_ALIGN
    assert f(opt(), 8, A[0], A[1], A[2], A[3], A[4] + 1, ha.HA_BF16, None) == ha.HA_ERR_ALIGN
    assert f(opt(), 8, A[0], A[1], A[2], A[3], A[4] + 2, ha.HA_F32, None) == ha.HA_ERR_ALIGN
    assert f(opt(), 8, A[0], A[1], A[2], A[3], A[0], ha.HA_F32, None) == ha.HA_ERR_SHAPE
    assert f(opt(), 0, A[0], A[1], A[2], A[3], A[4], ha.HA_BF16, None) == ha.HA_OK                 # nothing to do, nothing enqueued


# ---------------------------------------------------------------- binding-side checks of the feature-map tensors

def _cpu_map(H=3, d=128, Hd=128, F=128, dtype=None, mid=0):
    import torch
    dtype = dtype or torch.bfloat16
    kl = mid or Hd
    return ha.FeatureMap(torch.zeros(H, Hd, d, dtype=dtype), torch.zeros(H, Hd), torch.zeros(H, F, kl, dtype=dtype), torch.zeros(H, F), 2,
                         w_mid=torch.zeros(H, mid, Hd, dtype=dtype) if mid else None, b_mid=torch.zeros(H, mid) if mid else None)


def test_binding_checks_feature_map_tensors_against_the_problem():
    """The C ABI reads the weights through raw pointers: the binding must refuse tensors whose dtype, heads, widths or
    device differ from what the library will assume (host-only: CPU tensors, nothing is launched)."""
    import torch
    cpu = torch.device("cpu")
    _cpu_map().check(3, 128, torch.bfloat16, cpu)
    _cpu_map(Hd=256, F=256).check(3, 128, torch.bfloat16, cpu)
    _cpu_map(Hd=768, F=768, mid=768).check(3, 128, torch.bfloat16, cpu)
    bad = [
        (_cpu_map(dtype=torch.float32), "fp32 weights with bf16 q"),
        (_cpu_map(H=2), "maps for fewer heads"),
        (_cpu_map(d=64), "w1 inner width != d_head"),
    ]
    m = _cpu_map(); m.w2 = torch.zeros(3, 128, 64, dtype=torch.bfloat16); bad.append((m, "w2 inner width != d_hidden"))
    m = _cpu_map(); m.b1 = torch.zeros(3, 64); bad.append((m, "b1 too short"))
    m = _cpu_map(); m.b2 = torch.zeros(2, 128); bad.append((m, "b2 for fewer heads"))
    m = _cpu_map(mid=256); m.w2 = torch.zeros(3, 128, 128, dtype=torch.bfloat16); bad.append((m, "w2 inner width != d_mid"))
    m = _cpu_map(); m.b_mid = torch.zeros(3, 128); bad.append((m, "b_mid without w_mid"))
    m = _cpu_map(); m.poly_degree = 3; bad.append((m, "P does not divide F"))
    m = _cpu_map(); m.w1 = torch.zeros(3, 128 * 128, dtype=torch.bfloat16); bad.append((m, "w1 not 3-d"))
    for fm, why in bad:
        with pytest.raises(ValueError):
            fm.check(3, 128, torch.bfloat16, cpu)
            pytest.fail(why)
    with pytest.raises(ValueError):
        _cpu_map().check(3, 128, torch.bfloat16, torch.device("meta"))
    # the entry points run the check before anything else that touches the library's compute calls
    q = torch.zeros(1, 3, 16, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        ha._fm_ptr(_cpu_map(H=2), q)
