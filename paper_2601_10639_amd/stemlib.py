"""ctypes binding of libstem's C ABI (include/stem.h): same names, argument marshalling only.

Every function takes torch tensors (device memory unless the C header says host),
checks dtype / contiguity, and passes raw pointers plus the current torch stream.
Nothing is computed here; if the shared library is missing the import of any entry
point fails loudly — there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstem.so")

STEM_OK = 0
STEM_ERR_INVALID_ARG, STEM_ERR_SHAPE, STEM_ERR_ID_RANGE, STEM_ERR_WORKSPACE, STEM_ERR_UNSUPPORTED, STEM_ERR_HIP = range(1, 7)
STEM_F32, STEM_BF16 = 0, 1

SYMBOLS = [
    "stem_create", "stem_reserve", "stem_set_prefetch_mode", "stem_destroy", "stem_last_error", "stem_status_string", "stem_sync_status",
    "stem_ffn_forward", "stem_ffn_forward_residual", "stem_ffn_backward", "stem_ffn_up_forward", "stem_ffn_up_backward",
    "stem_embed_grad", "stem_embed_grad_presorted", "stem_embed_grad_noalloc", "stem_embed_sparse_adamw",
    "stem_prefetch_rows", "stem_cache_init", "stem_prefetch_rows_cached", "stem_cache_state",
    "stem_edit_rows", "stem_profile_enable", "stem_profile_kernels", "stem_profile_read",
    "stem_profile_reset", "stem_measure_peak",
]


class stem_layer_desc(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("vocab", ctypes.c_int32),
                ("dtype", ctypes.c_int32)]


class stem_adamw_hparams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("step", ctypes.c_int64)]


class StemError(RuntimeError):
    def __init__(self, status: int, where: str, text: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}: {text}")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2601_10639_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.stem_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(stem_layer_desc), i64, i32]
        L.stem_create.restype = i32
        L.stem_reserve.argtypes = [vp, ctypes.c_uint32]
        L.stem_reserve.restype = i32
        L.stem_set_prefetch_mode.argtypes = [vp, i32]
        L.stem_set_prefetch_mode.restype = i32
        L.stem_destroy.argtypes = [vp]
        L.stem_destroy.restype = None
        L.stem_last_error.argtypes = [vp]
        L.stem_last_error.restype = ctypes.c_char_p
        L.stem_status_string.argtypes = [i32]
        L.stem_status_string.restype = ctypes.c_char_p
        L.stem_sync_status.argtypes = [vp, vp]
        L.stem_sync_status.restype = i32
        L.stem_ffn_forward.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp, vp]
        L.stem_ffn_forward.restype = i32
        L.stem_ffn_forward_residual.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, vp, vp, vp]
        L.stem_ffn_forward_residual.restype = i32
        L.stem_ffn_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, vp, vp, i64, vp, vp, vp, vp, i32, vp]
        L.stem_ffn_backward.restype = i32
        L.stem_ffn_up_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp, vp]
        L.stem_ffn_up_forward.restype = i32
        L.stem_ffn_up_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, vp, vp, i64, vp, vp, vp, vp, vp,
                                           i32, vp]
        L.stem_ffn_up_backward.restype = i32
        L.stem_embed_grad.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp]
        L.stem_embed_grad.restype = i32
        L.stem_embed_grad_presorted.argtypes = [vp, vp, i64, vp, vp, vp, vp]
        L.stem_embed_grad_presorted.restype = i32
        L.stem_embed_grad_noalloc.argtypes = [i32, i32, i32, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp]
        L.stem_embed_grad_noalloc.restype = i32
        L.stem_embed_sparse_adamw.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp,
                                              ctypes.POINTER(stem_adamw_hparams), vp]
        L.stem_embed_sparse_adamw.restype = i32
        L.stem_prefetch_rows.argtypes = [vp, vp, vp, i64, vp, i64, vp, ctypes.POINTER(i64), vp,
                                         ctypes.POINTER(vp)]
        L.stem_prefetch_rows.restype = i32
        L.stem_cache_init.argtypes = [vp, i64]
        L.stem_cache_init.restype = i32
        L.stem_prefetch_rows_cached.argtypes = [vp, vp, vp, i64, vp, i64, vp, ctypes.POINTER(i64),
                                                ctypes.POINTER(i64), ctypes.POINTER(vp)]
        L.stem_prefetch_rows_cached.restype = i32
        L.stem_cache_state.argtypes = [vp, vp, i64]
        L.stem_cache_state.restype = i32
        L.stem_edit_rows.argtypes = [vp, vp, vp, i64, vp, i64, i32, i32, vp, vp]
        L.stem_edit_rows.restype = i32
        L.stem_profile_enable.argtypes = [vp, i32]
        L.stem_profile_enable.restype = i32
        L.stem_profile_kernels.argtypes = []
        L.stem_profile_kernels.restype = i32
        L.stem_profile_read.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_char_p),
                                        ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        L.stem_profile_read.restype = i32
        L.stem_profile_reset.argtypes = [vp]
        L.stem_profile_reset.restype = i32
        L.stem_measure_peak.argtypes = [i32, vp, vp, i64, i32, vp, ctypes.POINTER(ctypes.c_double)]
        L.stem_measure_peak.restype = i32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().stem_status_string(status).decode()


class StemCtx:
    """Owner of one stem_ctx*; frees it on close() or garbage collection."""

    def __init__(self, handle: int, d_model: int, d_ff: int, vocab: int, dtype: int, max_tokens: int, device: int):
        self.handle = ctypes.c_void_p(handle)
        self.d_model, self.d_ff, self.vocab, self.dtype = d_model, d_ff, vocab, dtype
        self.max_tokens, self.device = max_tokens, device

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.dtype == STEM_BF16 else torch.float32

    def close(self):
        if self.handle:
            lib().stem_destroy(self.handle)
            self.handle = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _check(ctx, status: int, where: str):
    if status != STEM_OK:
        h = ctx.handle if ctx is not None else None
        raise StemError(status, where, lib().stem_last_error(h).decode())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ptr(t, dtype=None, cuda=True, name="tensor") -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(None)
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if cuda == "or_pinned":
        if not (t.is_cuda or t.is_pinned()):
            raise ValueError(f"{name}: must be device memory or pinned host memory")
        return ctypes.c_void_p(t.data_ptr())
    if cuda and not t.is_cuda:
        raise ValueError(f"{name}: must be device memory")
    if not cuda and t.is_cuda:
        raise ValueError(f"{name}: must be host memory")
    return ctypes.c_void_p(t.data_ptr())


STEM_RESERVE_UP, STEM_RESERVE_EDIT = 1, 2
STEM_NOALLOC_MAX_TOKENS = 65536
STEM_PREFETCH_KERNEL, STEM_PREFETCH_MEMCPY = 0, 1


def stem_create(d_model: int, d_ff: int, vocab: int, dtype: int, max_tokens: int, device: int = 0,
                reserve: int = 0) -> StemCtx:
    """reserve: a sum of STEM_RESERVE_* bits passed on to stem_reserve."""
    desc = stem_layer_desc(d_model, d_ff, vocab, dtype)
    out = ctypes.c_void_p(None)
    st = lib().stem_create(ctypes.byref(out), ctypes.byref(desc), max_tokens, device)
    _check(None, st, "stem_create")
    ctx = StemCtx(out.value, d_model, d_ff, vocab, dtype, max_tokens, device)
    if reserve:
        stem_reserve(ctx, reserve)
    return ctx


def stem_reserve(ctx: StemCtx, what: int):
    _check(ctx, lib().stem_reserve(ctx.handle, what), "stem_reserve")


def stem_set_prefetch_mode(ctx: StemCtx, mode: int):
    _check(ctx, lib().stem_set_prefetch_mode(ctx.handle, mode), "stem_set_prefetch_mode")


def stem_destroy(ctx: StemCtx):
    ctx.close()


def stem_sync_status(ctx: StemCtx, stream=None):
    _check(ctx, lib().stem_sync_status(ctx.handle, _stream(stream)), "stem_sync_status")


def stem_ffn_forward(ctx: StemCtx, x, ids, W_gate, W_down, E, y, save_G=None, save_H=None, wait_event=None,
                     stream=None, E_rows=None, T=None):
    dt = ctx.torch_dtype
    T = x.shape[0] if T is None else T
    E_rows = E.shape[0] if E_rows is None else E_rows
    st = lib().stem_ffn_forward(ctx.handle, _ptr(x, dt, name="x"), _ptr(ids, torch.int32, name="ids"),
                                _ptr(W_gate, dt, name="W_gate"), _ptr(W_down, dt, name="W_down"),
                                _ptr(E, dt, name="E"), E_rows, T, _ptr(y, dt, name="y"),
                                _ptr(save_G, dt, name="save_G"), _ptr(save_H, dt, name="save_H"),
                                ctypes.c_void_p(wait_event), _stream(stream))
    _check(ctx, st, "stem_ffn_forward")


def stem_ffn_forward_residual(ctx: StemCtx, x, ids, W_gate, W_down, E, residual, y, stream=None, E_rows=None, T=None):
    """y = residual + layer(x); y may be residual (and x) itself."""
    dt = ctx.torch_dtype
    T = x.shape[0] if T is None else T
    E_rows = E.shape[0] if E_rows is None else E_rows
    st = lib().stem_ffn_forward_residual(ctx.handle, _ptr(x, dt, name="x"), _ptr(ids, torch.int32, name="ids"),
                                         _ptr(W_gate, dt, name="W_gate"), _ptr(W_down, dt, name="W_down"),
                                         _ptr(E, dt, name="E"), E_rows, T, _ptr(residual, dt, name="residual"),
                                         _ptr(y, dt, name="y"), _stream(stream))
    _check(ctx, st, "stem_ffn_forward_residual")


def stem_ffn_backward(ctx: StemCtx, dy, x, ids, W_gate, W_down, E, saved_G, saved_H, dx, dW_gate, dW_down, dU,
                      accumulate: bool = False, stream=None, E_rows=None, T=None):
    dt = ctx.torch_dtype
    T = dy.shape[0] if T is None else T
    E_rows = E.shape[0] if E_rows is None else E_rows
    st = lib().stem_ffn_backward(ctx.handle, _ptr(dy, dt, name="dy"), _ptr(x, dt, name="x"),
                                 _ptr(ids, torch.int32, name="ids"), _ptr(W_gate, dt, name="W_gate"),
                                 _ptr(W_down, dt, name="W_down"), _ptr(E, dt, name="E"), E_rows,
                                 _ptr(saved_G, dt, name="saved_G"), _ptr(saved_H, dt, name="saved_H"), T,
                                 _ptr(dx, dt, name="dx"), _ptr(dW_gate, torch.float32, name="dW_gate"),
                                 _ptr(dW_down, torch.float32, name="dW_down"), _ptr(dU, dt, name="dU"),
                                 1 if accumulate else 0, _stream(stream))
    _check(ctx, st, "stem_ffn_backward")


def stem_ffn_up_forward(ctx: StemCtx, x, ids, W_gate, W_up, W_down, E, y, save_G=None, save_Up=None, save_H=None,
                        stream=None, E_rows=None, T=None):
    """E (and ids) may be None: the dense SwiGLU FFN."""
    dt = ctx.torch_dtype
    T = x.shape[0] if T is None else T
    E_rows = (E.shape[0] if E is not None else 0) if E_rows is None else E_rows
    st = lib().stem_ffn_up_forward(ctx.handle, _ptr(x, dt, name="x"), _ptr(ids, torch.int32, name="ids"),
                                   _ptr(W_gate, dt, name="W_gate"), _ptr(W_up, dt, name="W_up"),
                                   _ptr(W_down, dt, name="W_down"), _ptr(E, dt, name="E"), E_rows, T,
                                   _ptr(y, dt, name="y"), _ptr(save_G, dt, name="save_G"),
                                   _ptr(save_Up, dt, name="save_Up"), _ptr(save_H, dt, name="save_H"), _stream(stream))
    _check(ctx, st, "stem_ffn_up_forward")


def stem_ffn_up_backward(ctx: StemCtx, dy, x, ids, W_gate, W_up, W_down, E, saved_G, saved_Up, saved_H, dx, dW_gate,
                         dW_up, dW_down, dV, accumulate: bool = False, stream=None, E_rows=None, T=None):
    dt = ctx.torch_dtype
    f32 = torch.float32
    T = dy.shape[0] if T is None else T
    E_rows = (E.shape[0] if E is not None else 0) if E_rows is None else E_rows
    st = lib().stem_ffn_up_backward(ctx.handle, _ptr(dy, dt, name="dy"), _ptr(x, dt, name="x"),
                                    _ptr(ids, torch.int32, name="ids"), _ptr(W_gate, dt, name="W_gate"),
                                    _ptr(W_up, dt, name="W_up"), _ptr(W_down, dt, name="W_down"),
                                    _ptr(E, dt, name="E"), E_rows, _ptr(saved_G, dt, name="saved_G"),
                                    _ptr(saved_Up, dt, name="saved_Up"), _ptr(saved_H, dt, name="saved_H"), T,
                                    _ptr(dx, dt, name="dx"), _ptr(dW_gate, f32, name="dW_gate"),
                                    _ptr(dW_up, f32, name="dW_up"), _ptr(dW_down, f32, name="dW_down"),
                                    _ptr(dV, dt, name="dV"), 1 if accumulate else 0, _stream(stream))
    _check(ctx, st, "stem_ffn_up_backward")


def stem_embed_grad(ctx: StemCtx, ids, dU, sorted_ids, perm, uniq_ids, seg_offsets, n_uniq, dE_rows, stream=None,
                    T=None):
    i32 = torch.int32
    T = ids.shape[0] if T is None else T
    st = lib().stem_embed_grad(ctx.handle, _ptr(ids, i32, name="ids"), _ptr(dU, ctx.torch_dtype, name="dU"), T,
                               _ptr(sorted_ids, i32, name="sorted_ids"), _ptr(perm, i32, name="perm"),
                               _ptr(uniq_ids, i32, name="uniq_ids"), _ptr(seg_offsets, i32, name="seg_offsets"),
                               _ptr(n_uniq, i32, name="n_uniq"), _ptr(dE_rows, torch.float32, name="dE_rows"),
                               _stream(stream))
    _check(ctx, st, "stem_embed_grad")


def stem_embed_grad_presorted(ctx: StemCtx, dU, perm, seg_offsets, dE_rows, stream=None, T=None):
    """The row sums alone, after a stem_embed_grad(dU=None) call on the same context and T."""
    T = dU.shape[0] if T is None else T
    st = lib().stem_embed_grad_presorted(ctx.handle, _ptr(dU, ctx.torch_dtype, name="dU"), T,
                                         _ptr(perm, torch.int32, name="perm"),
                                         _ptr(seg_offsets, torch.int32, name="seg_offsets"),
                                         _ptr(dE_rows, torch.float32, name="dE_rows"), _stream(stream))
    _check(ctx, st, "stem_embed_grad_presorted")


def stem_embed_grad_noalloc(dtype: int, vocab: int, d_ff: int, ids, dU, sorted_ids, perm, uniq_ids, seg_offsets,
                            n_uniq, dE_rows, id_flag=None, stream=None, T=None):
    """stem_embed_grad on the library's static scratch: no context, no allocation; current device."""
    i32 = torch.int32
    T = ids.shape[0] if T is None else T
    dt = torch.bfloat16 if dtype == STEM_BF16 else torch.float32
    st = lib().stem_embed_grad_noalloc(dtype, vocab, d_ff, _ptr(ids, i32, name="ids"), _ptr(dU, dt, name="dU"), T,
                                       _ptr(sorted_ids, i32, name="sorted_ids"), _ptr(perm, i32, name="perm"),
                                       _ptr(uniq_ids, i32, name="uniq_ids"), _ptr(seg_offsets, i32, name="seg_offsets"),
                                       _ptr(n_uniq, i32, name="n_uniq"), _ptr(dE_rows, torch.float32, name="dE_rows"),
                                       _ptr(id_flag, i32, name="id_flag"), _stream(stream))
    _check(None, st, "stem_embed_grad_noalloc")


def stem_embed_sparse_adamw(ctx: StemCtx, uniq_ids, n_uniq, dE_rows, E, master, m, v, lr, beta1, beta2, eps,
                            weight_decay, step, stream=None, max_rows=None):
    """E, master, m, v may be pinned host tensors (table and optimiser state resident in host memory)."""
    hp = stem_adamw_hparams(lr, beta1, beta2, eps, weight_decay, step)
    f32 = torch.float32
    max_rows = dE_rows.shape[0] if max_rows is None else max_rows
    st = lib().stem_embed_sparse_adamw(ctx.handle, _ptr(uniq_ids, torch.int32, name="uniq_ids"),
                                       _ptr(n_uniq, torch.int32, name="n_uniq"), max_rows,
                                       _ptr(dE_rows, f32, name="dE_rows"),
                                       _ptr(E, ctx.torch_dtype, cuda="or_pinned", name="E"),
                                       _ptr(master, f32, cuda="or_pinned", name="master"),
                                       _ptr(m, f32, cuda="or_pinned", name="m"),
                                       _ptr(v, f32, cuda="or_pinned", name="v"), ctypes.byref(hp), _stream(stream))
    _check(ctx, st, "stem_embed_sparse_adamw")


def stem_prefetch_rows(ctx: StemCtx, E_host, ids_host, E_compact, remap, uniq_ids_host=None, T=None):
    """Returns (n_uniq, ready_event handle)."""
    if not E_host.is_pinned():
        raise ValueError("E_host must be pinned host memory")
    T = ids_host.shape[0] if T is None else T
    n = ctypes.c_int64(0)
    ev = ctypes.c_void_p(None)
    st = lib().stem_prefetch_rows(ctx.handle, _ptr(E_host, ctx.torch_dtype, cuda=False, name="E_host"),
                                  _ptr(ids_host, torch.int32, cuda=False, name="ids_host"), T,
                                  _ptr(E_compact, ctx.torch_dtype, name="E_compact"), E_compact.shape[0],
                                  _ptr(remap, torch.int32, name="remap"), ctypes.byref(n),
                                  _ptr(uniq_ids_host, torch.int32, cuda=False, name="uniq_ids_host"),
                                  ctypes.byref(ev))
    _check(ctx, st, "stem_prefetch_rows")
    return n.value, ev.value


def stem_cache_init(ctx: StemCtx, n_slots: int):
    _check(ctx, lib().stem_cache_init(ctx.handle, n_slots), "stem_cache_init")


def stem_prefetch_rows_cached(ctx: StemCtx, E_host, ids_host, E_dev, n_slots: int, remap, T=None):
    """E_dev holds n_slots cache rows followed by the staging area.  Returns (n_uniq, n_miss, ready_event)."""
    if not E_host.is_pinned():
        raise ValueError("E_host must be pinned host memory")
    T = ids_host.shape[0] if T is None else T
    n = ctypes.c_int64(0)
    nm = ctypes.c_int64(0)
    ev = ctypes.c_void_p(None)
    st = lib().stem_prefetch_rows_cached(ctx.handle, _ptr(E_host, ctx.torch_dtype, cuda=False, name="E_host"),
                                         _ptr(ids_host, torch.int32, cuda=False, name="ids_host"), T,
                                         _ptr(E_dev, ctx.torch_dtype, name="E_dev"), E_dev.shape[0] - n_slots,
                                         _ptr(remap, torch.int32, name="remap"), ctypes.byref(n), ctypes.byref(nm),
                                         ctypes.byref(ev))
    _check(ctx, st, "stem_prefetch_rows_cached")
    return n.value, nm.value, ev.value


def stem_cache_state(ctx: StemCtx, n_slots: int):
    """Table row held by each cache slot (-1 = free), as a CPU int32 tensor."""
    out = torch.empty(n_slots, dtype=torch.int32)
    _check(ctx, lib().stem_cache_state(ctx.handle, _ptr(out, torch.int32, cuda=False, name="out"), n_slots),
           "stem_cache_state")
    return out


STEM_EDIT_REPLACE, STEM_EDIT_PAD_LEFT, STEM_EDIT_COPY, STEM_EDIT_AVERAGE = 0, 1, 2, 3


def stem_edit_rows(ctx: StemCtx, E, src_ids, tgt_ids, mode: int, pad_id: int = 0, backup=None, stream=None):
    """src_ids, tgt_ids: sequences of token ids (host).  E: the layer's table on the device."""
    src = (ctypes.c_int32 * len(src_ids))(*[int(t) for t in src_ids])
    tgt = (ctypes.c_int32 * len(tgt_ids))(*[int(t) for t in tgt_ids])
    st = lib().stem_edit_rows(ctx.handle, _ptr(E, ctx.torch_dtype, name="E"), src, len(src_ids), tgt, len(tgt_ids),
                              mode, pad_id, _ptr(backup, ctx.torch_dtype, name="backup"), _stream(stream))
    _check(ctx, st, "stem_edit_rows")


def stem_profile_enable(ctx: StemCtx, on: bool):
    _check(ctx, lib().stem_profile_enable(ctx.handle, 1 if on else 0), "stem_profile_enable")


def stem_profile_reset(ctx: StemCtx):
    _check(ctx, lib().stem_profile_reset(ctx.handle), "stem_profile_reset")


def stem_profile_read(ctx: StemCtx) -> dict:
    """{kernel name: (total_ms, launches)} for every kernel that was launched."""
    out = {}
    for k in range(lib().stem_profile_kernels()):
        name = ctypes.c_char_p()
        ms = ctypes.c_double()
        n = ctypes.c_int64()
        _check(ctx, lib().stem_profile_read(ctx.handle, k, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(n)),
               "stem_profile_read")
        if n.value:
            out[name.value.decode()] = (ms.value, n.value)
    return out


STEM_PEAK_MFMA_BF16, STEM_PEAK_HBM_READ, STEM_PEAK_HBM_COPY, STEM_PEAK_MFMA_BF16_DATA = 0, 1, 2, 3


def stem_measure_peak(what: int, buf_a, buf_b=None, repeats: int = 3, stream=None) -> float:
    """TFLOP/s (MFMA loop) or GB/s (streaming read of buf_a / copy buf_a -> buf_b) this GPU sustains."""
    out = ctypes.c_double(0.0)
    nbytes = buf_a.numel() * buf_a.element_size()
    st = lib().stem_measure_peak(what, _ptr(buf_a, name="buf_a"), _ptr(buf_b, name="buf_b"), nbytes, repeats,
                                 _stream(stream), ctypes.byref(out))
    _check(None, st, "stem_measure_peak")
    return out.value
