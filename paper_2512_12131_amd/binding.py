"""ctypes binding of liblrboost.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their device pointers,
sizes and leading dimensions through the C ABI of include/lrboost.h and returns the output
tensors.  PyTorch is used for device memory and the current stream, nothing else: every step of
the computation runs in the library's kernels.  There is no CPU or PyTorch fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

LR_F32, LR_BF16 = 0, 1
LR_ACT_IDENTITY, LR_ACT_SILU = 0, 1
LR_NORM_NONE, LR_NORM_TWO_PASS, LR_NORM_ONLINE, LR_NORM_SHARD_LOCAL, LR_NORM_ONLINE_GATHER = 0, 1, 2, 3, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblrboost.so")
_lib = None

_vp, _i64, _int, _f32, _sz = C.c_void_p, C.c_int64, C.c_int, C.c_float, C.c_size_t


class LrError(RuntimeError):
    pass


class BlockDesc(C.Structure):
    _fields_ = [("batch", _i64), ("seq", _i64), ("d_model", _i64), ("n_heads", _i64), ("head_dim", _i64),
                ("ffn", _i64), ("ffn_ld", _i64), ("rank", _i64), ("eps", _f32), ("act", _int), ("norm", _int),
                ("dt", _int), ("grad_dt", _int), ("causal", _int), ("rope_cos", _vp), ("rope_sin", _vp),
                ("stat_x_ready", _int), ("stat_y_out", _vp), ("n_kv_heads", _i64)]


class BlockParams(C.Structure):
    _fields_ = [(n, _vp) for n in ("gamma1", "w_dn_qkv", "w_up_qkv", "w_dn_o", "w_up_o", "gamma2", "w_dn_gu",
                                   "w_up_gu", "w_dn_d", "w_up_d")]


class BlockCkpt(C.Structure):
    _fields_ = [(n, _vp) for n in ("z_qkv", "z_o", "z_gu", "z_d", "s1", "s2")]


class BlockSaved(C.Structure):
    _fields_ = [(n, _vp) for n in ("qkv", "o", "lse", "h1", "gu", "m")]


class BlockLax(C.Structure):
    _fields_ = [(k + "_" + n, _vp) for k in ("h_prev", "dz_next", "dh_prev") for n in ("qkv", "o", "gu", "d")]


PARAM_NAMES = tuple(n for n, _ in BlockParams._fields_)
LAX_PARTS = ("qkv", "o", "gu", "d")

_SIGS = {
    "lr_version": (_int, []),
    "lr_status_string": (C.c_char_p, [_int]),
    "lr_linear_workspace_bytes": (_sz, [_i64, _i64, _i64, _i64, _int, _int]),
    "lr_linear_fwd": (_int, [_vp, _i64, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _int, _int, _vp, _sz, _vp]),
    "lr_linear_fwd_static": (_int, [_vp, _i64, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _int, _int, _vp]),
    "lr_linear_bwd": (_int, [_vp, _i64, _vp, _vp, _vp, _vp, _i64, _vp, _i64, _vp, _vp, _i64, _i64, _i64, _i64, _int,
                             _int, _int, _int, _vp, _sz, _vp]),
    "lr_group_workspace_bytes": (_sz, [_int, _i64, _i64, _i64, _i64, _int, _int]),
    "lr_group_fwd": (_int, [_vp, _i64, _vp, _f32, _int, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _int, _i64, _i64, _i64,
                            _i64, _int, _int, _vp, _sz, _vp]),
    "lr_group_bwd": (_int, [_vp, _i64, _vp, _f32, _int, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _vp, _i64, _vp, _vp, _vp,
                            _int, _i64, _i64, _i64, _i64, _int, _int, _int, _int, _vp, _sz, _vp]),
    "lr_block_workspace_bytes": (_sz, [C.POINTER(BlockDesc), _int]),
    "lr_block_ckpt_bytes": (_sz, [C.POINTER(BlockDesc)]),
    "lr_block_fwd": (_int, [C.POINTER(BlockDesc), C.POINTER(BlockParams), _vp, _vp, C.POINTER(BlockCkpt), _vp, _sz,
                            _vp]),
    "lr_block_bwd": (_int, [C.POINTER(BlockDesc), C.POINTER(BlockParams), _vp, _vp, C.POINTER(BlockCkpt), _vp,
                            C.POINTER(BlockParams), _int, _vp, _sz, _vp]),
    "lr_block_saved_workspace_bytes": (_sz, [C.POINTER(BlockDesc), _int]),
    "lr_block_fwd_save": (_int, [C.POINTER(BlockDesc), C.POINTER(BlockParams), _vp, _vp, C.POINTER(BlockCkpt),
                                 C.POINTER(BlockSaved), _vp, _sz, _vp]),
    "lr_block_bwd_saved": (_int, [C.POINTER(BlockDesc), C.POINTER(BlockParams), _vp, _vp, C.POINTER(BlockCkpt),
                                  C.POINTER(BlockSaved), _vp, C.POINTER(BlockParams), _int, _vp, _sz, _vp]),
    "lr_block_lax_fwd": (_int, [C.POINTER(BlockDesc), C.POINTER(BlockParams), _vp, _vp, C.POINTER(BlockCkpt),
                                C.POINTER(BlockLax), _vp, _sz, _vp]),
    "lr_block_lax_bwd": (_int, [C.POINTER(BlockDesc), C.POINTER(BlockParams), _vp, _vp, C.POINTER(BlockCkpt), _vp,
                                C.POINTER(BlockParams), _int, C.POINTER(BlockLax), _vp, _sz, _vp]),
    "lr_rope": (_int, [_vp, _i64, _vp, _vp, _i64, _i64, _i64, _i64, _int, _int, _vp]),
    "lr_attention_fwd": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _int, _int, _vp]),
    "lr_attention_bwd_workspace_bytes": (_sz, [_i64, _i64, _i64, _i64]),
    "lr_attention_bwd": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _int, _int,
                                _vp, _sz, _vp]),
    "lr_attention_gqa_fwd": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _i64, _i64, _int, _int, _vp]),
    "lr_attention_gqa_bwd_workspace_bytes": (_sz, [_i64, _i64, _i64, _i64, _i64]),
    "lr_attention_gqa_bwd": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _i64, _i64,
                                    _int, _int, _vp, _sz, _vp]),
    "lr_launch_timer_begin": (_int, [_int]),
    "lr_launch_timer_end": (_int, [_vp, _int, C.POINTER(_int)]),
    "lr_mfma_probe": (_int, [_int, _int, _int, C.POINTER(C.c_double), _vp]),
    "lr_rms_stat": (_int, [_vp, _i64, _vp, _i64, _i64, _int, _vp]),
    "lr_rmsnorm_apply": (_int, [_vp, _i64, _vp, _vp, _f32, _vp, _i64, _i64, _i64, _int, _vp]),
    "lr_online_rmsnorm_finish": (_int, [_vp, _i64, _vp, _i64, _f32, _vp, _i64, _i64, _i64, _int, _vp]),
    "lr_rmsnorm_bwd_parts": (_i64, [_i64]),
    "lr_rmsnorm_bwd": (_int, [_vp, _i64, _vp, _vp, _f32, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _i64, _int, _vp]),
    "lr_act_fwd": (_int, [_vp, _i64, _vp, _i64, _i64, _i64, _int, _int, _vp]),
    "lr_swiglu_fwd": (_int, [_vp, _vp, _vp, _i64, _i64, _i64, _int, _vp]),
    "lr_swiglu_bwd": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _vp]),
}
EXPORTS = tuple(_SIGS)


def lib():
    """Loads liblrboost.so on first use.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise LrError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(status: int, what: str):
    if status != 0:
        raise LrError(f"{what} failed: {lib().lr_status_string(status).decode()}")


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return LR_F32
    if t.dtype == torch.bfloat16:
        return LR_BF16
    raise LrError(f"unsupported dtype {t.dtype}")


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(nbytes: int, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _rowmajor(t: torch.Tensor):
    assert t.dim() == 2 and t.stride(1) == 1, "row-major 2-D tensor expected"
    return t.stride(0)


# ---- one bottleneck layer ------------------------------------------------------------------
def lr_linear_workspace_bytes(T, d_in, r, d_out, dt, backward):
    return lib().lr_linear_workspace_bytes(T, d_in, r, d_out, dt, int(backward))


def lr_linear_fwd(x, w_down, w_up, act=LR_ACT_SILU):
    """Returns (z[T, r], y[T, d_out])."""
    T, d_in = x.shape
    r, d_out = w_down.shape[0], w_up.shape[0]
    dt = _dt(x)
    z = torch.empty((T, r), dtype=x.dtype, device=x.device)
    y = torch.empty((T, d_out), dtype=x.dtype, device=x.device)
    nb = lr_linear_workspace_bytes(T, d_in, r, d_out, dt, 0)
    ws = _ws(nb, x.device)
    _check(lib().lr_linear_fwd(_p(x), _rowmajor(x), _p(w_down), _p(w_up), _p(z), _p(y), d_out, T, d_in, r, d_out, act,
                               dt, _p(ws), nb, _stream()), "lr_linear_fwd")
    return z, y


def lr_linear_fwd_static(x, w_down, w_up, z, y, act=LR_ACT_SILU):
    """The forward of one bottleneck layer through the entry point that allocates nothing: the caller
    passes the outputs z[T, r] and y[T, d_out]; the library's scratch is a device array of its own."""
    T, d_in = x.shape
    r, d_out = w_down.shape[0], w_up.shape[0]
    assert z.shape == (T, r) and y.shape == (T, d_out) and z.is_contiguous() and y.is_contiguous()
    _check(lib().lr_linear_fwd_static(_p(x), _rowmajor(x), _p(w_down), _p(w_up), _p(z), _p(y), d_out, T, d_in, r, d_out,
                                      act, _dt(x), _stream()), "lr_linear_fwd_static")
    return z, y


def _tdt(dt):
    return torch.float32 if dt == LR_F32 else torch.bfloat16


def lr_linear_bwd(x, w_down, w_up, z, dy, act=LR_ACT_SILU, grads=None, grad_dt=LR_F32):
    """Returns (dx, dw_down, dw_up).  With grads=(dw_down, dw_up) the weight grads are accumulated."""
    T, d_in = x.shape
    r, d_out = w_down.shape[0], w_up.shape[0]
    dt = _dt(x)
    dx = torch.empty((T, d_in), dtype=x.dtype, device=x.device)
    acc = grads is not None
    dwd, dwu = grads if acc else (torch.empty_like(w_down, dtype=_tdt(grad_dt)),
                                  torch.empty_like(w_up, dtype=_tdt(grad_dt)))
    nb = lr_linear_workspace_bytes(T, d_in, r, d_out, dt, 1)
    ws = _ws(nb, x.device)
    _check(lib().lr_linear_bwd(_p(x), _rowmajor(x), _p(w_down), _p(w_up), _p(z), _p(dy), _rowmajor(dy), _p(dx), d_in,
                               _p(dwd), _p(dwu), T, d_in, r, d_out, act, dt, grad_dt, int(acc), _p(ws), nb, _stream()),
           "lr_linear_bwd")
    return dx, dwd, dwu


# ---- G projections sharing one input ---------------------------------------------------------
def lr_group_workspace_bytes(G, T, d_in, r, d_out, dt, backward):
    return lib().lr_group_workspace_bytes(G, T, d_in, r, d_out, dt, int(backward))


def lr_group_fwd(x, gamma, eps, norm, w_down_cat, w_up_stack, act=LR_ACT_SILU):
    """Returns (z_cat[T, G*r], stat[T] fp32, y_stack[G, T, d_out])."""
    T, d_in = x.shape
    G, d_out, r = w_up_stack.shape
    dt = _dt(x)
    z = torch.empty((T, G * r), dtype=x.dtype, device=x.device)
    stat = torch.empty((T,), dtype=torch.float32, device=x.device)
    y = torch.empty((G, T, d_out), dtype=x.dtype, device=x.device)
    nb = lr_group_workspace_bytes(G, T, d_in, r, d_out, dt, 0)
    ws = _ws(nb, x.device)
    _check(lib().lr_group_fwd(_p(x), _rowmajor(x), _p(gamma), eps, norm, _p(w_down_cat), _p(w_up_stack), _p(z),
                              _p(stat), _p(y), d_out, T * d_out, G, T, d_in, r, d_out, act, dt, _p(ws), nb, _stream()),
           "lr_group_fwd")
    return z, stat, y


def lr_group_bwd(x, gamma, eps, norm, w_down_cat, w_up_stack, z_cat, stat, dy_stack, act=LR_ACT_SILU, grads=None,
                 grad_dt=LR_F32):
    """Returns (dx, dgamma, dw_down_cat, dw_up_stack)."""
    T, d_in = x.shape
    G, d_out, r = w_up_stack.shape
    dt = _dt(x)
    dx = torch.empty((T, d_in), dtype=x.dtype, device=x.device)
    acc = grads is not None
    if acc:
        dgamma, dwd, dwu = grads
    else:
        gt = _tdt(grad_dt)
        dgamma = torch.empty((d_in,), dtype=gt, device=x.device)
        dwd, dwu = torch.empty_like(w_down_cat, dtype=gt), torch.empty_like(w_up_stack, dtype=gt)
    nb = lr_group_workspace_bytes(G, T, d_in, r, d_out, dt, 1)
    ws = _ws(nb, x.device)
    _check(lib().lr_group_bwd(_p(x), _rowmajor(x), _p(gamma), eps, norm, _p(w_down_cat), _p(w_up_stack), _p(z_cat),
                              _p(stat), _p(dy_stack), d_out, T * d_out, _p(dx), d_in, _p(dgamma), _p(dwd), _p(dwu), G,
                              T, d_in, r, d_out, act, dt, grad_dt, int(acc), _p(ws), nb, _stream()), "lr_group_bwd")
    return dx, dgamma, dwd, dwu


# ---- the decoder block -----------------------------------------------------------------------
def make_block_desc(batch, seq, d_model, n_heads, head_dim, ffn, ffn_ld, rank, eps=1e-5, act=LR_ACT_SILU,
                    norm=LR_NORM_ONLINE, dt=LR_BF16, grad_dt=LR_F32, causal=1, rope=None, stat_x_ready=False,
                    stat_y_out=None, n_kv_heads=0):
    """n_kv_heads: 0 (= n_heads) or a divisor of n_heads (grouped-query attention; w_up_qkv is then the
    packed [d_model + 2 * n_kv_heads * head_dim, rank] matrix: q rows, k rows, v rows).  rope: None, or (cos, sin) device tensors [seq, head_dim / 2] fp32.  stat_y_out: None or a device
    tensor [T] fp32 that receives sum y^2; stat_x_ready: ckpt["s1"] arrives filled.  The descriptor holds
    addresses only: keep the tensors alive while the descriptor is in use (desc._keep does)."""
    cos_p = sin_p = None
    if rope is not None:
        cos_p, sin_p = rope[0].data_ptr(), rope[1].data_ptr()
    desc = BlockDesc(batch, seq, d_model, n_heads, head_dim, ffn, ffn_ld, rank, eps, act, norm, dt, grad_dt, causal,
                     cos_p, sin_p, int(bool(stat_x_ready)), None if stat_y_out is None else stat_y_out.data_ptr(),
                     int(n_kv_heads))
    desc._keep = (rope, stat_y_out)
    return desc


def _params_struct(params: dict):
    return BlockParams(*[C.c_void_p(params[n].data_ptr()) for n in PARAM_NAMES])


def lr_block_workspace_bytes(desc, backward):
    return lib().lr_block_workspace_bytes(C.byref(desc), int(backward))


def lr_block_ckpt_bytes(desc):
    return lib().lr_block_ckpt_bytes(C.byref(desc))


def alloc_block_ckpt(desc, device):
    T, r = desc.batch * desc.seq, desc.rank
    tdt = torch.bfloat16 if desc.dt == LR_BF16 else torch.float32
    return {
        "z_qkv": torch.empty((T, 3 * r), dtype=tdt, device=device),
        "z_o": torch.empty((T, r), dtype=tdt, device=device),
        "z_gu": torch.empty((T, 2 * r), dtype=tdt, device=device),
        "z_d": torch.empty((T, r), dtype=tdt, device=device),
        "s1": torch.empty((T,), dtype=torch.float32, device=device),
        "s2": torch.empty((T,), dtype=torch.float32, device=device),
    }


def _ckpt_struct(ck: dict):
    return BlockCkpt(*[C.c_void_p(ck[n].data_ptr()) for n, _ in BlockCkpt._fields_])


def lr_block_fwd(desc, params: dict, x, ckpt: dict = None, ws=None, y=None):
    """Returns (y, ckpt).  `params` maps the lr_block_params field names to device tensors."""
    if ckpt is None:
        ckpt = alloc_block_ckpt(desc, x.device)
    if y is None:
        y = torch.empty_like(x)
    nb = lr_block_workspace_bytes(desc, 0)
    if nb == 0:
        raise LrError("lr_block_workspace_bytes: invalid or unsupported block descriptor")
    if ws is None:
        ws = _ws(nb, x.device)
    ps, cs = _params_struct(params), _ckpt_struct(ckpt)
    _check(lib().lr_block_fwd(C.byref(desc), C.byref(ps), _p(x), _p(y), C.byref(cs), _p(ws), ws.numel(), _stream()),
           "lr_block_fwd")
    return y, ckpt


def lr_block_bwd(desc, params: dict, x, dy, ckpt: dict, grads: dict = None, accumulate=False, ws=None, dx=None):
    """Returns (dx, grads) with grads keyed like params."""
    if grads is None:
        grads = {n: torch.empty_like(params[n], dtype=_tdt(desc.grad_dt)) for n in PARAM_NAMES}
    if dx is None:
        dx = torch.empty_like(x)
    nb = lr_block_workspace_bytes(desc, 1)
    if nb == 0:
        raise LrError("lr_block_workspace_bytes: invalid or unsupported block descriptor")
    if ws is None:
        ws = _ws(nb, x.device)
    ps, cs, gs = _params_struct(params), _ckpt_struct(ckpt), _params_struct(grads)
    _check(lib().lr_block_bwd(C.byref(desc), C.byref(ps), _p(x), _p(dy), C.byref(cs), _p(dx), C.byref(gs),
                              int(accumulate), _p(ws), ws.numel(), _stream()), "lr_block_bwd")
    return dx, grads


# ---- block with every wide activation kept ---------------------------------------------------
def alloc_block_saved(desc, device):
    T, d, f = desc.batch * desc.seq, desc.d_model, desc.ffn_ld
    dkv = (desc.n_kv_heads or desc.n_heads) * desc.head_dim
    bf = torch.bfloat16
    return {"qkv": torch.empty((T * (d + 2 * dkv),), dtype=bf, device=device),
            "o": torch.empty((T, d), dtype=bf, device=device),
            "lse": torch.empty((desc.batch, desc.n_heads, desc.seq), dtype=torch.float32, device=device),
            "h1": torch.empty((T, d), dtype=bf, device=device),
            "gu": torch.empty((2, T, f), dtype=bf, device=device),
            "m": torch.empty((T, f), dtype=bf, device=device)}


def _saved_struct(sv: dict):
    return BlockSaved(*[C.c_void_p(sv[n].data_ptr()) for n, _ in BlockSaved._fields_])


def lr_block_fwd_save(desc, params: dict, x, ckpt: dict = None, saved: dict = None, ws=None, y=None):
    """Returns (y, ckpt, saved): the forward that also keeps every wide activation."""
    ckpt = alloc_block_ckpt(desc, x.device) if ckpt is None else ckpt
    saved = alloc_block_saved(desc, x.device) if saved is None else saved
    y = torch.empty_like(x) if y is None else y
    nb = lib().lr_block_saved_workspace_bytes(C.byref(desc), 0)
    if nb == 0:
        raise LrError("lr_block_saved_workspace_bytes: invalid or unsupported block descriptor")
    ws = _ws(nb, x.device) if ws is None else ws
    ps, cs, ss = _params_struct(params), _ckpt_struct(ckpt), _saved_struct(saved)
    _check(lib().lr_block_fwd_save(C.byref(desc), C.byref(ps), _p(x), _p(y), C.byref(cs), C.byref(ss), _p(ws),
                                   ws.numel(), _stream()), "lr_block_fwd_save")
    return y, ckpt, saved


def lr_block_bwd_saved(desc, params: dict, x, dy, ckpt: dict, saved: dict, grads: dict = None, accumulate=False,
                       ws=None, dx=None):
    """Returns (dx, grads): the backward that reads the kept activations instead of re-forwarding."""
    if grads is None:
        grads = {n: torch.empty_like(params[n], dtype=_tdt(desc.grad_dt)) for n in PARAM_NAMES}
    dx = torch.empty_like(x) if dx is None else dx
    nb = lib().lr_block_saved_workspace_bytes(C.byref(desc), 1)
    if nb == 0:
        raise LrError("lr_block_saved_workspace_bytes: invalid or unsupported block descriptor")
    ws = _ws(nb, x.device) if ws is None else ws
    ps, cs, gs, ss = _params_struct(params), _ckpt_struct(ckpt), _params_struct(grads), _saved_struct(saved)
    _check(lib().lr_block_bwd_saved(C.byref(desc), C.byref(ps), _p(x), _p(dy), C.byref(cs), C.byref(ss), _p(dx),
                                    C.byref(gs), int(accumulate), _p(ws), ws.numel(), _stream()), "lr_block_bwd_saved")
    return dx, grads


# ---- block, LaX variant ----------------------------------------------------------------------
def _lax_struct(h_prev=None, dz_next=None, dh_prev=None):
    """Each argument: None or a dict keyed "qkv", "o", "gu", "d" of device tensors (missing keys = NULL)."""
    vals = []
    for d in (h_prev, dz_next, dh_prev):
        for n in LAX_PARTS:
            t = None if d is None else d.get(n)
            vals.append(C.c_void_p(None if t is None else t.data_ptr()))
    return BlockLax(*vals)


def lr_block_lax_fwd(desc, params: dict, x, h_prev: dict = None, ckpt: dict = None, ws=None, y=None):
    """Returns (y, ckpt); ckpt["z_qkv"], ["z_o"], ["z_gu"], ["z_d"] are the h_prev of the block above."""
    if ckpt is None:
        ckpt = alloc_block_ckpt(desc, x.device)
    if y is None:
        y = torch.empty_like(x)
    nb = lr_block_workspace_bytes(desc, 0)
    if nb == 0:
        raise LrError("lr_block_workspace_bytes: invalid or unsupported block descriptor")
    if ws is None:
        ws = _ws(nb, x.device)
    ps, cs, lx = _params_struct(params), _ckpt_struct(ckpt), _lax_struct(h_prev)
    _check(lib().lr_block_lax_fwd(C.byref(desc), C.byref(ps), _p(x), _p(y), C.byref(cs), C.byref(lx), _p(ws),
                                  ws.numel(), _stream()), "lr_block_lax_fwd")
    return y, ckpt


def lr_block_lax_bwd(desc, params: dict, x, dy, ckpt: dict, h_prev: dict = None, dz_next: dict = None,
                     want_dh_prev=True, grads: dict = None, accumulate=False, ws=None, dx=None):
    """Returns (dx, grads, dh_prev) with dh_prev keyed "qkv", "o", "gu", "d" (None if not wanted)."""
    if grads is None:
        grads = {n: torch.empty_like(params[n], dtype=_tdt(desc.grad_dt)) for n in PARAM_NAMES}
    if dx is None:
        dx = torch.empty_like(x)
    dh = None
    if want_dh_prev:
        dh = {n: torch.empty_like(ckpt["z_" + n]) for n in LAX_PARTS}
    nb = lr_block_workspace_bytes(desc, 1)
    if nb == 0:
        raise LrError("lr_block_workspace_bytes: invalid or unsupported block descriptor")
    if ws is None:
        ws = _ws(nb, x.device)
    ps, cs, gs = _params_struct(params), _ckpt_struct(ckpt), _params_struct(grads)
    lx = _lax_struct(h_prev, dz_next, dh)
    _check(lib().lr_block_lax_bwd(C.byref(desc), C.byref(ps), _p(x), _p(dy), C.byref(cs), _p(dx), C.byref(gs),
                                  int(accumulate), C.byref(lx), _p(ws), ws.numel(), _stream()), "lr_block_lax_bwd")
    return dx, grads, dh


# ---- rotary position embedding ----------------------------------------------------------------
def lr_rope(x, cos, sin, B, S, H, hd, inverse=False):
    """In place on x [B*S, >= H*hd] bf16; cos, sin [S, hd/2] fp32 device tensors.  Returns x."""
    _check(lib().lr_rope(_p(x), _rowmajor(x), _p(cos), _p(sin), B, S, H, hd, int(inverse), _dt(x), _stream()), "lr_rope")
    return x


# ---- attention -----------------------------------------------------------------------------
def lr_attention_fwd(q, k, v, B, S, H, hd, causal=True):
    o = torch.empty_like(q)
    lse = torch.empty((B, H, S), dtype=torch.float32, device=q.device)
    _check(lib().lr_attention_fwd(_p(q), _p(k), _p(v), _p(o), _p(lse), _rowmajor(q), B, S, H, hd, int(causal), _dt(q),
                                  _stream()), "lr_attention_fwd")
    return o, lse


def lr_attention_bwd(q, k, v, o, dout, lse, B, S, H, hd, causal=True):
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    nb = lib().lr_attention_bwd_workspace_bytes(B, S, H, hd)
    ws = _ws(nb, q.device)
    _check(lib().lr_attention_bwd(_p(q), _p(k), _p(v), _p(o), _p(dout), _p(lse), _p(dq), _p(dk), _p(dv), _rowmajor(q),
                                  B, S, H, hd, int(causal), _dt(q), _p(ws), ws.numel(), _stream()), "lr_attention_bwd")
    return dq, dk, dv


def lr_attention_gqa_fwd(q, k, v, B, S, H, Hkv, hd, causal=True):
    """q [B*S, >= H*hd], k and v [B*S, >= Hkv*hd] (k and v with the same row stride)."""
    o = torch.empty_like(q)
    lse = torch.empty((B, H, S), dtype=torch.float32, device=q.device)
    assert _rowmajor(k) == _rowmajor(v)
    _check(lib().lr_attention_gqa_fwd(_p(q), _p(k), _p(v), _p(o), _p(lse), _rowmajor(q), _rowmajor(k), B, S, H, Hkv, hd,
                                      int(causal), _dt(q), _stream()), "lr_attention_gqa_fwd")
    return o, lse


def lr_attention_gqa_bwd(q, k, v, o, dout, lse, B, S, H, Hkv, hd, causal=True):
    assert _rowmajor(k) == _rowmajor(v)
    dq = torch.empty_like(q)
    dk, dv = (torch.empty_strided(k.shape, k.stride(), dtype=k.dtype, device=k.device) for _ in range(2))   # rows of ldkv
    nb = lib().lr_attention_gqa_bwd_workspace_bytes(B, S, H, Hkv, hd)
    ws = _ws(nb, q.device)
    _check(lib().lr_attention_gqa_bwd(_p(q), _p(k), _p(v), _p(o), _p(dout), _p(lse), _p(dq), _p(dk), _p(dv), _rowmajor(q),
                                      _rowmajor(k), B, S, H, Hkv, hd, int(causal), _dt(q), _p(ws), ws.numel(), _stream()),
           "lr_attention_gqa_bwd")
    return dq, dk, dv


# ---- measurement aid -----------------------------------------------------------------------
class LaunchRecord(C.Structure):
    _fields_ = [("tag", _int), ("M", _int), ("N", _int), ("K", _int), ("batch", _int), ("ms", _f32),
                ("flops", C.c_double)]


LR_TAG_ATTN_FWD, LR_TAG_ATTN_BWD = 32, 33
_timer_cap = 0


def lr_launch_timer_begin(max_launches=4096):
    global _timer_cap
    _check(lib().lr_launch_timer_begin(int(max_launches)), "lr_launch_timer_begin")
    _timer_cap = int(max_launches)


def lr_launch_timer_end():
    """Returns the list of (tag, M, N, K, batch, ms, flops) of every bracketed launch since begin."""
    buf = (LaunchRecord * _timer_cap)()
    n = _int(0)
    _check(lib().lr_launch_timer_end(C.cast(buf, _vp), _timer_cap, C.byref(n)), "lr_launch_timer_end")
    return [(r.tag, r.M, r.N, r.K, r.batch, r.ms, r.flops) for r in buf[:min(n.value, _timer_cap)]]


def lr_mfma_probe(random_operands=True, iters=20000, launches=20):
    """TFLOP/s the bf16 matrix pipes sustain from registers alone (waits for its own launches)."""
    tf = C.c_double(0.0)
    _check(lib().lr_mfma_probe(int(bool(random_operands)), iters, launches, C.byref(tf), _stream()), "lr_mfma_probe")
    return tf.value


# ---- standalone memory-bound kernels ---------------------------------------------------------
def lr_rms_stat(x):
    T, d = x.shape
    stat = torch.empty((T,), dtype=torch.float32, device=x.device)
    _check(lib().lr_rms_stat(_p(x), _rowmajor(x), _p(stat), T, d, _dt(x), _stream()), "lr_rms_stat")
    return stat


def lr_rmsnorm_apply(x, gamma, stat, eps):
    T, d = x.shape
    out = torch.empty_like(x)
    _check(lib().lr_rmsnorm_apply(_p(x), _rowmajor(x), _p(gamma), _p(stat), eps, _p(out), d, T, d, _dt(x), _stream()),
           "lr_rmsnorm_apply")
    return out


def lr_shard_down_fwd(x_shard, gamma_shard, eps, w_down_cat_shard):
    """One rank's part of the feature-sharded grouped down-projection (lr_group_fwd with
    LR_NORM_SHARD_LOCAL).  Returns (partial product [T, G*r], local sum of squares [T])."""
    T, d_in = x_shard.shape
    GR = w_down_cat_shard.shape[0]
    dt = _dt(x_shard)
    h = torch.empty((T, GR), dtype=x_shard.dtype, device=x_shard.device)
    stat = torch.empty((T,), dtype=torch.float32, device=x_shard.device)
    nb = lr_group_workspace_bytes(1, T, d_in, GR, 8, dt, 0)
    ws = _ws(nb, x_shard.device)
    _check(lib().lr_group_fwd(_p(x_shard), _rowmajor(x_shard), _p(gamma_shard), eps, LR_NORM_SHARD_LOCAL,
                              _p(w_down_cat_shard), None, _p(h), _p(stat), None, 0, 0, 1, T, d_in, GR, 8, LR_ACT_IDENTITY,
                              dt, _p(ws), nb, _stream()), "lr_group_fwd (shard-local)")
    return h, stat


def lr_online_rmsnorm_finish(h_sum, stat_sum, d_total, eps):
    T, n = h_sum.shape
    z = torch.empty_like(h_sum)
    _check(lib().lr_online_rmsnorm_finish(_p(h_sum), _rowmajor(h_sum), _p(stat_sum), d_total, eps, _p(z), n, T, n,
                                          _dt(h_sum), _stream()), "lr_online_rmsnorm_finish")
    return z


def lr_rmsnorm_bwd(x, gamma, stat, eps, dxhat, dres=None):
    """Returns (dx, dgamma_part[nparts, d] fp32)."""
    T, d = x.shape
    dx = torch.empty_like(x)
    nparts = lib().lr_rmsnorm_bwd_parts(T)
    part = torch.empty((max(nparts, 1), d), dtype=torch.float32, device=x.device)
    _check(lib().lr_rmsnorm_bwd(_p(x), _rowmajor(x), _p(gamma), _p(stat), eps, _p(dxhat), _rowmajor(dxhat), _p(dres),
                                _rowmajor(dres) if dres is not None else 0, _p(dx), d, _p(part), T, d, _dt(x),
                                _stream()), "lr_rmsnorm_bwd")
    return dx, part


def lr_act_fwd(z, act=LR_ACT_SILU):
    T, n = z.shape
    a = torch.empty_like(z)
    _check(lib().lr_act_fwd(_p(z), _rowmajor(z), _p(a), n, T, n, act, _dt(z), _stream()), "lr_act_fwd")
    return a


def lr_swiglu_fwd(g, u):
    T, f = g.shape
    m = torch.empty_like(g)
    _check(lib().lr_swiglu_fwd(_p(g), _p(u), _p(m), _rowmajor(g), T, f, _dt(g), _stream()), "lr_swiglu_fwd")
    return m


def lr_swiglu_bwd(g, u, dm):
    T, f = g.shape
    dg, du = torch.empty_like(g), torch.empty_like(u)
    _check(lib().lr_swiglu_bwd(_p(g), _p(u), _p(dm), _p(dg), _p(du), _rowmajor(g), T, f, _dt(g), _stream()),
           "lr_swiglu_bwd")
    return dg, du
