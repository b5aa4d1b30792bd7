"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
function nats.h declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2602_03681_amd import binding as nb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))

OK, E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_WS, E_UNSUP = 0, -1, -2, -3, -4, -5, -6
FAKE = 0x10000  # an aligned non-NULL "device pointer"; validation fails before it is ever used


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(nb.library_path()):
        from paper_2602_03681_amd.build import build_library
        build_library()
    return nb.load_library()


def declared_functions():
    text = "\n".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nats_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_function_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(nb.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_abi_version(lib):
    assert lib.nats_abi_version() == 113   # 101: nats_fwd_params gained `routing`; 102: nats_fwd_extra gained `W_out`;
    # 103: nats_fwd_params and nats_dec_params gained `linear_op` and `freeze_on_softmax`; 104: backward entry points; 105: Q_nla / K_nla; 106: weight_act; 107: combine_mode 2; 108: gdn_segments, nats_hybrid_attn_fwd_noalloc; 109: group, decode workspace;
    # 110: p->math selects the form of the backward's linear adjoint, C = 128 with routing per chunk; 111: the backward
    # pass takes p->group; 112: nats_bwd_extra gained Q_nla, K_nla, dQ_nla, dK_nla;
    # 113: the backward takes combine_mode 1 and 2 (nats_bwd_extra gained w_nla, w_la, dw_nla, dw_la)


def good_params(**over):
    kw = dict(B=1, H=2, L=256, d=64, C=64, dtype_code=nb.NATS_F32)
    kw.update(over)
    return nb.make_fwd_params(**kw)


def test_workspace_bytes(lib):
    p = good_params()
    n = nb.fwd_workspace_bytes(p)
    # at least cnt + idx + compacted K,V + fp32 linear-branch output
    assert n >= 2 * 512 * 4 + 2 * 512 * 64 * 4 + 512 * 64 * 4
    assert nb.fwd_workspace_bytes(good_params(L=100)) == 0          # L % C != 0
    assert nb.fwd_workspace_bytes(good_params(d=48)) == 0
    big = nb.fwd_workspace_bytes(good_params(B=2, H=16, L=8192, d=128, dtype_code=nb.NATS_BF16))
    assert big > n


def call_fwd(lib, p, ptrs=None, ws=FAKE, ws_bytes=1 << 40, extra=None):
    ptrs = [FAKE] * 7 if ptrs is None else ptrs
    return lib.nats_hybrid_attn_fwd_ex(ctypes.byref(p), *ptrs, extra, ws, ws_bytes, None)


@pytest.mark.parametrize("over,code", [
    (dict(L=100), E_SHAPE), (dict(L=0), E_SHAPE), (dict(B=0), E_SHAPE), (dict(d=96), E_SHAPE),
    (dict(dtype_code=7), E_DTYPE), (dict(C=32, L=256), E_UNSUP), (dict(combine_mode=3), E_SHAPE),
    (dict(math=9), E_SHAPE), (dict(B=70000, H=1), E_SHAPE), (dict(linear_op=2), E_SHAPE),
    (dict(freeze_on_softmax=3), E_SHAPE), (dict(weight_act=3), E_SHAPE),
])
def test_bad_params_are_rejected(lib, over, code):
    assert call_fwd(lib, good_params(**over)) == code
    assert lib.nats_last_error() != b""


def test_null_misaligned_and_workspace_errors(lib):
    p = good_params()
    assert lib.nats_hybrid_attn_fwd_ex(None, *([FAKE] * 7), None, FAKE, 1 << 40, None) == E_NULL
    for i in range(7):
        ptrs = [FAKE] * 7
        ptrs[i] = None
        assert call_fwd(lib, p, ptrs) == E_NULL
    ptrs = [FAKE] * 7
    ptrs[2] = FAKE + 4
    assert call_fwd(lib, p, ptrs) == E_ALIGN
    assert b"aligned" in lib.nats_last_error()
    assert call_fwd(lib, p, ws=None) == E_WS
    assert call_fwd(lib, p, ws_bytes=nb.fwd_workspace_bytes(p) - 1) == E_WS
    assert b"needed" in lib.nats_last_error()
    # O aliasing an input
    assert call_fwd(lib, p, [FAKE, FAKE + 16, FAKE + 32, FAKE + 48, FAKE + 64, FAKE + 80, FAKE]) == E_SHAPE
    # Kc without Vc
    ex = nb.FwdExtra()
    ex.Kc = FAKE
    assert call_fwd(lib, p, [FAKE + 16 * i for i in range(7)], extra=ctypes.byref(ex)) == E_NULL
    # Q_nla without K_nla
    ex = nb.FwdExtra()
    ex.Q_nla = FAKE + 4096
    assert call_fwd(lib, p, [FAKE + 16 * i for i in range(7)], extra=ctypes.byref(ex)) == E_NULL


def test_plain_fwd_goes_through_the_same_validation(lib):
    p = good_params(L=100)
    assert lib.nats_hybrid_attn_fwd(ctypes.byref(p), *([FAKE] * 7), FAKE, 1 << 40, None) == E_SHAPE


def test_decode_validation(lib):
    def call(p, ptrs=None):
        ptrs = [FAKE + 16 * i for i in range(14)] if ptrs is None else ptrs
        return lib.nats_hybrid_attn_decode(ctypes.byref(p), *ptrs, None)
    good = nb.DecParams(4, 2, 128, 512, nb.NATS_BF16, 0.0, 0.0, 0, 0.0)
    assert call(nb.DecParams(4, 2, 100, 512, nb.NATS_BF16, 0, 0, 0, 0)) == E_SHAPE
    assert call(nb.DecParams(4, 2, 128, 0, nb.NATS_BF16, 0, 0, 0, 0)) == E_SHAPE
    assert call(nb.DecParams(4, 2, 128, 512, 5, 0, 0, 0, 0)) == E_DTYPE
    assert call(nb.DecParams(4, 2, 128, 512, nb.NATS_BF16, 0, 0, 3, 0)) == E_SHAPE
    assert call(nb.DecParams(4, 2, 128, 512, nb.NATS_BF16, 0, 0, 0, 0, 5, 0)) == E_SHAPE     # linear_op
    assert call(nb.DecParams(4, 2, 128, 512, nb.NATS_BF16, 0, 0, 0, 0, 1, 2)) == E_SHAPE     # freeze_on_softmax
    assert call(nb.DecParams(4, 2, 128, 512, nb.NATS_BF16, 0, 0, 0, 0, 0, 0, FAKE, None)) == E_NULL   # q_nla alone
    ptrs = [FAKE + 16 * i for i in range(14)]
    ptrs[0] = None
    assert call(good, ptrs) == E_NULL
    ptrs = [FAKE + 16 * i for i in range(14)]
    ptrs[4] = FAKE + 2
    assert call(good, ptrs) == E_ALIGN


def test_chunk_routing_validation(lib):
    # forward: routing must be one of the two enumerators
    assert lib.nats_hybrid_attn_fwd_workspace_bytes(ctypes.byref(good_params(routing=7))) == 0
    assert lib.nats_hybrid_attn_fwd_workspace_bytes(ctypes.byref(good_params(routing=nb.NATS_ROUTE_CHUNK))) > 0
    # generation with routing per chunk: params, state struct and pointers are checked before any launch
    good = nb.DecParams(4, 2, 128, 512, nb.NATS_BF16, 0.0, 0.0, 0, 0.0)
    st = nb.DecChunkState(*[FAKE + 16 * i for i in range(7)])
    args = [FAKE + 256 + 16 * i for i in range(9)]

    def step(p, s, a=args):
        return lib.nats_hybrid_attn_decode_chunk(ctypes.byref(p), None if s is None else ctypes.byref(s), *a, None)

    assert step(nb.DecParams(4, 2, 100, 512, nb.NATS_BF16, 0, 0, 0, 0), st) == E_SHAPE
    assert step(good, None) == E_NULL
    assert step(good, nb.DecChunkState(*([None] + [FAKE + 16 * i for i in range(6)]))) == E_NULL
    assert step(good, nb.DecChunkState(*([FAKE + 2] + [FAKE + 16 * i for i in range(6)]))) == E_ALIGN
    assert step(good, st, [None] + args[1:]) == E_NULL
    assert lib.nats_hybrid_attn_decode_commit(ctypes.byref(good), ctypes.byref(st), None, None, None) == E_NULL
    assert lib.nats_hybrid_attn_decode_commit(ctypes.byref(good), None, FAKE, None, None) == E_NULL


def test_route_chunks_and_merge_weights_validation(lib):
    """Every rejected call returns before anything is launched (the pointers are fake)."""
    rc = lambda *a: lib.nats_route_chunks(*a, None)
    assert rc(2, 250, 64, 1536, 6, nb.NATS_BF16, FAKE, FAKE + 64, None, FAKE + 128) == E_SHAPE     # L % C
    assert rc(2, 256, 64, 1537, 6, nb.NATS_BF16, FAKE, FAKE + 64, None, FAKE + 128) == E_SHAPE     # d_model % 8
    assert rc(2, 256, 64, 65544, 6, nb.NATS_BF16, FAKE, FAKE + 64, None, FAKE + 128) == E_SHAPE    # d_model too large
    assert rc(2, 256, 64, 1536, 40, nb.NATS_BF16, FAKE, FAKE + 64, None, FAKE + 128) == E_SHAPE    # H
    assert rc(2, 256, 64, 1536, 6, 9, FAKE, FAKE + 64, None, FAKE + 128) == E_DTYPE
    assert rc(2, 256, 64, 1536, 6, nb.NATS_BF16, None, FAKE + 64, None, FAKE + 128) == E_NULL
    assert rc(2, 256, 64, 1536, 6, nb.NATS_BF16, FAKE + 4, FAKE + 64, None, FAKE + 128) == E_ALIGN
    p = good_params()
    mw = lambda *a: lib.nats_merge_weights(ctypes.byref(p), *a, None)
    assert mw(None, FAKE, FAKE, FAKE) == E_NULL
    assert mw(FAKE + 4, FAKE, FAKE, FAKE) == E_ALIGN
    assert lib.nats_merge_weights(ctypes.byref(good_params(d=96)), FAKE, FAKE, FAKE, FAKE, None) == E_SHAPE


def test_backward_validation(lib):
    p = good_params()
    need = lib.nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(p))
    assert need > nb.fwd_workspace_bytes(p) // 2
    # the token-by-token adjoint of the linear branch (routing per chunk, math = NATS_MATH_FP32) keeps d/16 partial
    # copies of dQ and dK; by chunks (the default with routing per token) the workspace is smaller
    need_tok = lib.nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(good_params(math=nb.NATS_MATH_FP32)))
    assert need_tok > need
    assert lib.nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(good_params(routing=nb.NATS_ROUTE_CHUNK))) > 0
    # the merges of Eq. 21 run on fp32 copies and keep both branches' rows: a larger workspace
    assert lib.nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(good_params(combine_mode=1))) > need
    assert lib.nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(good_params(combine_mode=3))) == 0

    def call(prm, ptrs=None, ws=FAKE, ws_bytes=1 << 40):
        ptrs = [FAKE + 16 * i for i in range(12)] if ptrs is None else ptrs
        return lib.nats_hybrid_attn_bwd(ctypes.byref(prm), *ptrs, None, ws, ws_bytes, None)

    # the per-token linear score gradient does not exist with routing per chunk (rejected before any launch)
    ex = nb.BwdExtra(None, None, None, FAKE, None, None)
    ptrs0 = [FAKE + 16 * i for i in range(12)]
    assert lib.nats_hybrid_attn_bwd(ctypes.byref(good_params(routing=nb.NATS_ROUTE_CHUNK)), *ptrs0, ctypes.byref(ex), FAKE,
                                    1 << 40, None) == E_UNSUP
    assert call(good_params(combine_mode=3)) == E_SHAPE
    # weights of the merge belong to combine_mode 1 and 2
    exw = nb.BwdExtra(None, None, None, None, None, None, None, None, None, None, FAKE, None, None, None)
    assert lib.nats_hybrid_attn_bwd(ctypes.byref(p), *ptrs0, ctypes.byref(exw), FAKE, 1 << 40, None) == E_SHAPE
    assert call(good_params(L=100)) == E_SHAPE
    ptrs = [FAKE + 16 * i for i in range(12)]
    ptrs[6] = None                                     # dO
    assert call(p, ptrs) == E_NULL
    ptrs = [FAKE + 16 * i for i in range(12)]
    ptrs[8] = FAKE + 4                                 # dK
    assert call(p, ptrs) == E_ALIGN
    ptrs = [FAKE + 16 * i for i in range(12)]
    ptrs[7] = ptrs[0]                                  # dQ aliases Q
    assert call(p, ptrs) == E_SHAPE
    assert call(p, ws_bytes=need - 1) == E_WS
    # routing chunks of 128 tokens: the forward takes them, the backward covers 64
    assert nb.fwd_workspace_bytes(good_params(C=128, routing=nb.NATS_ROUTE_CHUNK)) > 0
    assert call(good_params(C=128, routing=nb.NATS_ROUTE_CHUNK)) == E_UNSUP


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(nb, "_lib", None)
    monkeypatch.setattr(nb, "_LIB_PATH", str(tmp_path / "libnats.so"))
    with pytest.raises(FileNotFoundError):
        nb.load_library()


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros((1, 1, 64, 64))
    a = torch.zeros((1, 1, 64))
    m = torch.zeros((1, 1, 64), dtype=torch.uint8)
    with pytest.raises(ValueError):
        nb.hybrid_attn_fwd(x, x, x, a, a, m)


def test_autograd_wrapper_has_no_cpu_path():
    """The differentiable function is the same two library calls: CPU tensors are refused, nothing is computed here."""
    import torch
    import paper_2602_03681_amd as nats
    x = torch.zeros((1, 1, 64, 64), requires_grad=True)
    a = torch.zeros((1, 1, 64))
    m = torch.zeros((1, 1, 64), dtype=torch.uint8)
    with pytest.raises(ValueError):
        nats.hybrid_attn(x, x, x, a, a, m)


def test_noalloc_forward_rejects_large_problems_on_the_host(lib):
    """The entry point without allocation checks the size against its built-in buffer before anything touches a
    device: too large a problem is an error, and so are bad parameters."""
    big = good_params(B=2, H=16, L=8192, d=128, dtype_code=nb.NATS_BF16)
    assert nb.fwd_workspace_bytes(big) > nb.NOALLOC_SCRATCH_BYTES
    assert lib.nats_hybrid_attn_fwd_noalloc(ctypes.byref(big), *([FAKE] * 7), None) == -5     # NATS_ERR_WORKSPACE
    assert b"scratch" in lib.nats_last_error()
    assert lib.nats_hybrid_attn_fwd_noalloc(ctypes.byref(good_params(L=100)), *([FAKE] * 7), None) == E_SHAPE
    assert lib.nats_hybrid_attn_fwd_noalloc(None, *([FAKE] * 7), None) == E_NULL


def test_head_grouping_is_validated_on_the_host(lib):
    assert nb.fwd_workspace_bytes(good_params(group=9)) == 0
    assert nb.fwd_workspace_bytes(good_params(group=-1)) == 0
    one, three = nb.fwd_workspace_bytes(good_params(group=0)), nb.fwd_workspace_bytes(good_params(group=3))
    assert one == nb.fwd_workspace_bytes(good_params(group=1))
    assert one < three < 3 * one     # rows per output head grow with the group, the integers do not
    # the backward pass runs once per member of the groups: its own workspace plus one member's tensors
    b1 = lib.nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(good_params(group=1)))
    b2 = lib.nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(good_params(group=2)))
    b3 = lib.nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(good_params(group=3)))
    assert 0 < b1 < b2 == b3
    assert lib.nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(good_params(group=9))) == 0
    assert b"group" in lib.nats_last_error()


def test_decode_workspace_is_validated_on_the_host(lib):
    n = nb.decode_workspace_bytes(2, 3, 128, 1000, nb.NATS_BF16)
    assert n == 2 * 3 * (4 * (128 + 4) + 128) * 4          # 4 blocks of 256 rows: (acc, max, sum) each, then o_la
    assert nb.decode_workspace_bytes(2, 3, 100, 1000, nb.NATS_BF16) == 0
    p = nb.DecParams(2, 3, 128, 1000, nb.NATS_BF16, 0.0, 0.0, 0, 0.0, 0, 0, None, None, FAKE, n - 1)
    args = [FAKE] * 15
    assert lib.nats_hybrid_attn_decode(ctypes.byref(p), *args[:13], None, None) == -5      # NATS_ERR_WORKSPACE
    p = nb.DecParams(2, 3, 128, 40000, nb.NATS_BF16, 0.0, 0.0, 0, 0.0, 0, 0, None, None, FAKE, 1 << 40)
    assert lib.nats_hybrid_attn_decode(ctypes.byref(p), *args[:13], None, None) == -6      # cap beyond the form's limit
