"""ctypes binding of libl2l.so: argument marshalling only, same names as include/l2l.h.

Every step of the path runs inside the library's HIP kernels; this module fails loudly if the
library has not been built (python -m paper_2002_05645_amd.build)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libl2l.so")

L2L_OK, L2L_E_ARG, L2L_E_STATE, L2L_E_HIP, L2L_E_NOMEM = 0, -1, -2, -3, -4
L2L_F32, L2L_BF16, L2L_FP16 = 0, 1, 2
DTYPES = {"fp32": L2L_F32, "bf16": L2L_BF16, "fp16": L2L_FP16}
PROF_GEMM, PROF_ATTN, PROF_ROWWISE, PROF_COLSUM, PROF_OTHER = range(5)
PROF_NAMES = ("gemm", "attn", "rowwise", "colsum", "other", "copy")
EPI_GELU, EPI_GELUGRAD, EPI_ACCUM, EPI_COLSUM, EPI_KEEPGRAD, EPI_MULAUX = 1, 2, 4, 8, 16, 32


class l2l_config(C.Structure):
    _fields_ = [("hidden", C.c_int), ("heads", C.c_int), ("ffn", C.c_int), ("seq", C.c_int),
                ("ubatch", C.c_int), ("num_ubatches", C.c_int), ("dtype", C.c_int),
                ("ln_eps", C.c_float), ("vocab", C.c_int), ("ubatch_group", C.c_int)]


class L2LError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"l2l error {code}: {msg}")
        self.code = code


_lib = None

_P = C.c_void_p
_CFGP = C.POINTER(l2l_config)
_SIGS = {
    "l2l_layer_tensor_count": (C.c_int, []),
    "l2l_embed_tensor_count": (C.c_int, []),
    "l2l_layer_tensor_offset": (C.c_longlong, [_CFGP, C.c_int]),
    "l2l_layer_tensor_size": (C.c_longlong, [_CFGP, C.c_int]),
    "l2l_layer_tensor_name": (C.c_char_p, [C.c_int]),
    "l2l_embed_tensor_offset": (C.c_longlong, [_CFGP, C.c_int]),
    "l2l_embed_tensor_size": (C.c_longlong, [_CFGP, C.c_int]),
    "l2l_embed_tensor_name": (C.c_char_p, [C.c_int]),
    "l2l_layer_param_count": (C.c_size_t, [_CFGP]),
    "l2l_layer_packed_elems": (C.c_size_t, [_CFGP]),
    "l2l_layer_param_bytes": (C.c_size_t, [_CFGP]),
    "l2l_layer_grad_bytes": (C.c_size_t, [_CFGP]),
    "l2l_embed_packed_elems": (C.c_size_t, [_CFGP]),
    "l2l_embed_param_bytes": (C.c_size_t, [_CFGP]),
    "l2l_embed_grad_bytes": (C.c_size_t, [_CFGP]),
    "l2l_config_check": (C.c_int, [_CFGP]),
    "l2l_create": (C.c_int, [_CFGP, _P, _P, C.POINTER(_P)]),
    "l2l_destroy": (C.c_int, [_P]),
    "l2l_device_bytes": (C.c_size_t, [_P]),
    "l2l_last_error": (C.c_char_p, [_P]),
    "l2l_sync": (C.c_int, [_P]),
    "l2l_param_stage": (C.c_int, [_P, C.c_int, _P, C.c_int]),
    "l2l_layer_fwd": (C.c_int, [_P, C.c_int, C.c_int, _P, _P]),
    "l2l_layer_bwd": (C.c_int, [_P, C.c_int, C.c_int, _P, _P]),
    "l2l_layer_fwd_stats": (C.c_int, [_P, C.c_int, C.c_int, _P, _P, _P]),
    "l2l_layer_bwd_stats": (C.c_int, [_P, C.c_int, C.c_int, _P, _P, _P, _P]),
    "l2l_grad_drain": (C.c_int, [_P, C.c_int, _P]),
    "l2l_drain_wait": (C.c_int, [_P, C.c_int]),
    "l2l_embed_stage": (C.c_int, [_P, _P]),
    "l2l_embed_fwd": (C.c_int, [_P, _P, _P]),
    "l2l_head_loss": (C.c_int, [_P, _P, _P, _P, _P]),
    "l2l_embed_bwd": (C.c_int, [_P, _P, _P]),
    "l2l_embed_grad_drain": (C.c_int, [_P, _P]),
    "l2l_embed_grad_drain_part": (C.c_int, [_P, _P, C.c_longlong, C.c_longlong]),
    "l2l_embed_stage_part": (C.c_int, [_P, _P, C.c_longlong, C.c_longlong]),
    "l2l_embed_drain_wait": (C.c_int, [_P]),
    "l2l_profile": (C.c_int, [_P, C.c_int]),
    "l2l_profile_overlap": (C.c_int, [_P, C.c_double, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double),
                                      C.POINTER(C.c_double)]),
    "l2l_profile_gemm_table": (C.c_int, [_P, C.c_char_p, C.c_size_t]),
    "l2l_profile_read": (C.c_int, [_P, C.c_int, C.POINTER(C.c_longlong), C.POINTER(C.c_double),
                                   C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "l2l_op_gemm": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _P, C.c_longlong,
                              _P, C.c_longlong, _P, C.c_longlong, C.c_float, _P, _P, C.c_int, C.c_int, C.c_int]),
    "l2l_op_gemm_ex": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _P, C.c_longlong,
                                 _P, C.c_longlong, _P, C.c_longlong, C.c_float, _P, _P, C.c_longlong, C.c_int, _P, _P,
                                 C.c_longlong, _P, C.c_longlong, C.POINTER(C.c_int), C.c_int]),
    "l2l_op_gemm_accum_noalloc": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _P, C.c_longlong, _P,
                                            C.c_longlong, _P, C.c_longlong]),
    "l2l_noalloc_scratch_bytes": (C.c_size_t, []),
    "l2l_noalloc_last_error": (C.c_char_p, []),
    "l2l_op_layernorm": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, _P, _P, _P, C.c_float, _P, _P, _P]),
    "eps_create": (C.c_int, [C.c_int, C.POINTER(C.c_size_t), C.c_int, C.c_int, C.POINTER(_P)]),
    "eps_destroy": (C.c_int, [_P]),
    "eps_master": (C.POINTER(C.c_float), [_P, C.c_int]),
    "eps_ship": (_P, [_P, C.c_int]),
    "eps_grad": (C.POINTER(C.c_float), [_P, C.c_int]),
    "eps_moment": (C.POINTER(C.c_float), [_P, C.c_int, C.c_int]),
    "eps_refresh_ship": (C.c_int, [_P, C.c_int, C.c_int]),
    "l2l_cls_tensor_count": (C.c_int, []),
    "l2l_cls_tensor_name": (C.c_char_p, [C.c_int]),
    "l2l_cls_tensor_offset": (C.c_longlong, [_CFGP, C.c_int, C.c_int]),
    "l2l_cls_tensor_size": (C.c_longlong, [_CFGP, C.c_int, C.c_int]),
    "l2l_cls_packed_elems": (C.c_size_t, [_CFGP, C.c_int]),
    "l2l_cls_stage": (C.c_int, [_P, _P, C.c_int]),
    "l2l_cls_head_loss": (C.c_int, [_P, _P, _P, _P, _P]),
    "l2l_cls_grad_drain": (C.c_int, [_P, _P]),
    "l2l_cls_drain_wait": (C.c_int, [_P]),
    "l2l_set_loss_scale": (C.c_int, [_P, C.c_float]),
    "l2l_stream_create_cu_masked": (C.c_int, [C.c_int, C.POINTER(C.c_void_p)]),
    "l2l_stream_destroy": (C.c_int, [C.c_void_p]),
    "l2l_memcpy_rows_async": (C.c_int, [_P, _P, C.c_size_t, C.c_int, _P]),
    "eps_adam_step": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_double, C.c_double, C.c_double, C.c_double]),
    "eps_adam_step_range": (C.c_int, [_P, C.c_int, C.c_longlong, C.c_longlong, C.c_int, C.c_double, C.c_double, C.c_double,
                                      C.c_double]),
    "eps_grad_unscale": (C.c_int, [_P, C.c_int, C.c_int, C.c_double, C.POINTER(C.c_int)]),
    "eps_grad_unscale_range": (C.c_int, [_P, C.c_int, C.c_longlong, C.c_longlong, C.c_double, C.POINTER(C.c_int)]),
    "eps_adam_step_range16": (C.c_int, [_P, C.c_int, C.c_longlong, C.c_longlong, C.c_int, C.c_double, C.c_double, C.c_double,
                                        C.c_double, C.c_int]),
    "eps_enable_grad16": (C.c_int, [_P]),
    "eps_grad16": (C.c_void_p, [_P, C.c_int]),
    "eps_grad_widen": (C.c_int, [_P, C.c_int, C.c_int, C.c_int]),
    "eps_grad_widen_range": (C.c_int, [_P, C.c_int, C.c_longlong, C.c_longlong, C.c_int]),
    "l2l_set_drain_dtype": (C.c_int, [_P, C.c_int]),
    "eps_lamb_step": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_double, C.c_double, C.c_double, C.c_double, C.c_double,
                                C.c_int, C.POINTER(C.c_longlong), C.POINTER(C.c_longlong), C.POINTER(C.c_double)]),
    "eps_host_bytes": (C.c_size_t, [_P]),
    "eps_is_pinned": (C.c_int, [_P]),
}
EXPORTS = tuple(_SIGS)


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2002_05645_amd.build` "
                              "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def make_config(hidden, heads, ffn, seq, ubatch, num_ubatches, dtype, ln_eps=1e-12, vocab=0, ubatch_group=0):
    d = DTYPES.get(dtype, dtype)
    return l2l_config(hidden, heads, ffn, seq, ubatch, num_ubatches, d, ln_eps, vocab, ubatch_group)


def layer_layout(cfg):
    """{name: (element offset, element count)} of the packed layer block."""
    L = lib()
    return {L.l2l_layer_tensor_name(i).decode(): (L.l2l_layer_tensor_offset(C.byref(cfg), i),
                                                   L.l2l_layer_tensor_size(C.byref(cfg), i))
            for i in range(L.l2l_layer_tensor_count())}


def embed_layout(cfg):
    L = lib()
    return {L.l2l_embed_tensor_name(i).decode(): (L.l2l_embed_tensor_offset(C.byref(cfg), i),
                                                   L.l2l_embed_tensor_size(C.byref(cfg), i))
            for i in range(L.l2l_embed_tensor_count())}


def cls_layout(cfg, num_classes):
    """{name: (element offset, element count)} of the sequence-classification head's packed block."""
    L = lib()
    return {L.l2l_cls_tensor_name(i).decode(): (L.l2l_cls_tensor_offset(C.byref(cfg), num_classes, i),
                                                 L.l2l_cls_tensor_size(C.byref(cfg), num_classes, i))
            for i in range(L.l2l_cls_tensor_count())}


def stream_create_cu_masked(cus_per_32: int) -> int:
    """hipStream_t (as an int) restricted to cus_per_32 of every 32 compute units; see include/l2l.h."""
    out = C.c_void_p()
    rc = lib().l2l_stream_create_cu_masked(cus_per_32, C.byref(out))
    if rc != L2L_OK:
        raise L2LError(rc, "l2l_stream_create_cu_masked")
    return out.value


def stream_destroy(handle: int):
    rc = lib().l2l_stream_destroy(handle)
    if rc != L2L_OK:
        raise L2LError(rc, "l2l_stream_destroy")


def memcpy_rows_async(dst, src, nbytes, to_host, stream):
    """pinned host <-> device copy through a DMA engine in either direction; see include/l2l.h"""
    rc = lib().l2l_memcpy_rows_async(_ptr(dst), _ptr(src), int(nbytes), int(bool(to_host)), stream or None)
    if rc != L2L_OK:
        raise L2LError(rc, "l2l_memcpy_rows_async")


def _ptr(x):
    """Address of a torch tensor, a numpy array, an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return C.cast(x, C.c_void_p).value


def op_gemm_accum_noalloc(stream, in_dtype, a_kc, b_kc, M, N, K, A, lda, B, ldb, Cm, ldc):
    """C += A B (fp32 C) without a context and without any allocation; see include/l2l.h."""
    rc = lib().l2l_op_gemm_accum_noalloc(stream or None, in_dtype, int(a_kc), int(b_kc), M, N, K, _ptr(A), lda, _ptr(B), ldb,
                                         _ptr(Cm), ldc)
    if rc != L2L_OK:
        raise L2LError(rc, lib().l2l_noalloc_last_error().decode())


class Context:
    """Owner of one l2l_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, cfg, compute_stream=0, copy_stream=0):
        self.cfg = cfg
        self._h = _P()
        rc = lib().l2l_create(C.byref(cfg), compute_stream or None, copy_stream or None, C.byref(self._h))
        if rc != L2L_OK:
            msg = lib().l2l_last_error(self._h).decode() if self._h else "l2l_create failed (bad config or no GPU)"
            if self._h:
                lib().l2l_destroy(self._h)
                self._h = _P()
            raise L2LError(rc, msg)

    def close(self):
        if self._h:
            lib().l2l_destroy(self._h)
            self._h = _P()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ck(self, rc):
        if rc != L2L_OK:
            raise L2LError(rc, lib().l2l_last_error(self._h).decode())

    def device_bytes(self):
        return lib().l2l_device_bytes(self._h)

    def sync(self):
        self._ck(lib().l2l_sync(self._h))

    def param_stage(self, layer, host_params, slot):
        self._ck(lib().l2l_param_stage(self._h, layer, _ptr(host_params), slot))

    def layer_fwd(self, layer, slot, x_stash, y_out):
        self._ck(lib().l2l_layer_fwd(self._h, layer, slot, _ptr(x_stash), _ptr(y_out)))

    def layer_bwd(self, layer, slot, x_stash, dy_dx):
        self._ck(lib().l2l_layer_bwd(self._h, layer, slot, _ptr(x_stash), _ptr(dy_dx)))

    def layer_fwd_stats(self, layer, slot, x_stash, y_out, rstd_out):
        self._ck(lib().l2l_layer_fwd_stats(self._h, layer, slot, _ptr(x_stash), _ptr(y_out), _ptr(rstd_out)))

    def layer_bwd_stats(self, layer, slot, x_stash, y_stash, rstd, dy_dx):
        self._ck(lib().l2l_layer_bwd_stats(self._h, layer, slot, _ptr(x_stash), _ptr(y_stash), _ptr(rstd), _ptr(dy_dx)))

    def grad_drain(self, layer, host_grads):
        self._ck(lib().l2l_grad_drain(self._h, layer, _ptr(host_grads)))

    def drain_wait(self, layer):
        self._ck(lib().l2l_drain_wait(self._h, layer))

    def embed_stage(self, host_embed):
        self._ck(lib().l2l_embed_stage(self._h, _ptr(host_embed)))

    def embed_stage_part(self, host_embed, first, count):
        self._ck(lib().l2l_embed_stage_part(self._h, _ptr(host_embed), int(first), int(count)))

    def embed_fwd(self, tokens, x_out):
        self._ck(lib().l2l_embed_fwd(self._h, _ptr(tokens), _ptr(x_out)))

    def head_loss(self, x_last, labels, dy_out, loss_out):
        self._ck(lib().l2l_head_loss(self._h, _ptr(x_last), _ptr(labels), _ptr(dy_out), _ptr(loss_out)))

    def embed_bwd(self, tokens, dy):
        self._ck(lib().l2l_embed_bwd(self._h, _ptr(tokens), _ptr(dy)))

    def embed_grad_drain(self, host_grads):
        self._ck(lib().l2l_embed_grad_drain(self._h, _ptr(host_grads)))

    def embed_grad_drain_part(self, host_grads, first, count):
        self._ck(lib().l2l_embed_grad_drain_part(self._h, _ptr(host_grads), int(first), int(count)))

    def set_drain_dtype(self, dtype):
        self._ck(lib().l2l_set_drain_dtype(self._h, DTYPES[dtype] if isinstance(dtype, str) else int(dtype)))

    def embed_drain_wait(self):
        self._ck(lib().l2l_embed_drain_wait(self._h))

    def profile(self, on):
        self._ck(lib().l2l_profile(self._h, int(on)))

    def profile_read(self):
        """{class name: dict(launches, ms, flops, bytes)}"""
        out = {}
        for i, name in enumerate(PROF_NAMES):
            n, ms, fl, by = C.c_longlong(), C.c_double(), C.c_double(), C.c_double()
            self._ck(lib().l2l_profile_read(self._h, i, C.byref(n), C.byref(ms), C.byref(fl), C.byref(by)))
            out[name] = dict(launches=n.value, ms=ms.value, flops=fl.value, bytes=by.value)
        return out

    def profile_gemm_table(self):
        """[dict(M, N, K, a_kc, b_kc, epi, out_f32, pass, launches, ms)] per distinct GEMM launch shape since profile(1 or 2)"""
        buf = C.create_string_buffer(1 << 16)
        self._ck(lib().l2l_profile_gemm_table(self._h, buf, len(buf)))
        rows = []
        for line in buf.value.decode().splitlines():
            f = line.split()
            rows.append(dict(zip(("M", "N", "K", "a_kc", "b_kc", "epi", "out_f32", "pass", "launches"), map(int, f[:9])), ms=float(f[9])))
        return rows

    def cls_stage(self, host_params, num_classes):
        self._ck(lib().l2l_cls_stage(self._h, _ptr(host_params), num_classes))

    def cls_head_loss(self, x_last, seq_labels, dy_out, loss_out):
        self._ck(lib().l2l_cls_head_loss(self._h, _ptr(x_last), _ptr(seq_labels), _ptr(dy_out), _ptr(loss_out)))

    def cls_grad_drain(self, host_grads):
        self._ck(lib().l2l_cls_grad_drain(self._h, _ptr(host_grads)))

    def cls_drain_wait(self):
        self._ck(lib().l2l_cls_drain_wait(self._h))

    def set_loss_scale(self, scale):
        self._ck(lib().l2l_set_loss_scale(self._h, float(scale)))

    def profile_overlap(self, merge_gap_ms=0.0):
        """dict(compute_busy_ms, copy_busy_ms, copy_hidden_ms, span_ms) since profile(1)"""
        v = [C.c_double() for _ in range(4)]
        self._ck(lib().l2l_profile_overlap(self._h, merge_gap_ms, *[C.byref(x) for x in v]))
        return dict(zip(("compute_busy_ms", "copy_busy_ms", "copy_hidden_ms", "span_ms"), [x.value for x in v]))

    def op_gemm(self, in_dtype, out_f32, a_kc, b_kc, M, N, K, A, lda, B, ldb, Cm, ldc, alpha=1.0, bias=None,
                resid=None, gelu=False, accumulate=False, impl=0):
        self._ck(lib().l2l_op_gemm(self._h, in_dtype, int(out_f32), int(a_kc), int(b_kc), M, N, K, _ptr(A), lda,
                                   _ptr(B), ldb, _ptr(Cm), ldc, alpha, _ptr(bias), _ptr(resid), int(gelu),
                                   int(accumulate), impl))

    def op_gemm_ex(self, in_dtype, out_f32, a_kc, b_kc, M, N, K, A, lda, B, ldb, Cm, ldc, alpha=1.0, bias=None, resid=None,
                   ldr=0, epi=0, aux=None, aux_out=None, ldaux=0, colsum=None, colsum_rows=0, impl=0) -> int:
        """returns the number of rows of `colsum` that were written (0 without L2L_EPI_COLSUM)"""
        used = C.c_int(0)
        self._ck(lib().l2l_op_gemm_ex(self._h, in_dtype, int(out_f32), int(a_kc), int(b_kc), M, N, K, _ptr(A), lda, _ptr(B), ldb,
                                      _ptr(Cm), ldc, alpha, _ptr(bias), _ptr(resid), ldr, int(epi), _ptr(aux), _ptr(aux_out),
                                      ldaux, _ptr(colsum), int(colsum_rows), C.byref(used), impl))
        return used.value

    def op_layernorm(self, dtype, rows, n, x, gamma, beta, eps, y, mean=None, rstd=None):
        self._ck(lib().l2l_op_layernorm(self._h, dtype, rows, n, _ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(y),
                                        _ptr(mean), _ptr(rstd)))


class EPS:
    """Host eager param-server store: numpy views over the library's host buffers."""

    def __init__(self, elems, ship_dtype, threads=0):
        self.elems = [int(e) for e in elems]
        self.ship_dtype = DTYPES.get(ship_dtype, ship_dtype)
        arr = (C.c_size_t * len(self.elems))(*self.elems)
        self._h = _P()
        rc = lib().eps_create(len(self.elems), arr, self.ship_dtype, threads, C.byref(self._h))
        if rc != L2L_OK:
            raise L2LError(rc, "eps_create failed")

    def close(self):
        if self._h:
            lib().eps_destroy(self._h)
            self._h = _P()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _f32(self, p, n):
        return np.ctypeslib.as_array(p, shape=(n,))

    def master(self, i):
        return self._f32(lib().eps_master(self._h, i), self.elems[i])

    def grad(self, i):
        return self._f32(lib().eps_grad(self._h, i), self.elems[i])

    def moment(self, i, which):
        return self._f32(lib().eps_moment(self._h, i, which), self.elems[i])

    def ship_ptr(self, i):
        return lib().eps_ship(self._h, i)

    def grad_ptr(self, i):
        return C.cast(lib().eps_grad(self._h, i), C.c_void_p).value

    def ship(self, i):
        p = lib().eps_ship(self._h, i)
        if self.ship_dtype in (L2L_BF16, L2L_FP16):     # the 16-bit patterns
            return np.ctypeslib.as_array(C.cast(p, C.POINTER(C.c_uint16)), shape=(self.elems[i],))
        return np.ctypeslib.as_array(C.cast(p, C.POINTER(C.c_float)), shape=(self.elems[i],))

    def refresh_ship(self, first=0, last=None):
        last = len(self.elems) - 1 if last is None else last
        rc = lib().eps_refresh_ship(self._h, first, last)
        if rc != L2L_OK:
            raise L2LError(rc, "eps_refresh_ship")

    def adam_step(self, first, last, t, lr=1e-4, beta1=0.9, beta2=0.999, eps_a=1e-8):
        rc = lib().eps_adam_step(self._h, first, last, t, lr, beta1, beta2, eps_a)
        if rc != L2L_OK:
            raise L2LError(rc, "eps_adam_step")

    def adam_step_range(self, block, first_elem, count, t, lr=1e-4, beta1=0.9, beta2=0.999, eps_a=1e-8):
        rc = lib().eps_adam_step_range(self._h, block, int(first_elem), int(count), t, lr, beta1, beta2, eps_a)
        if rc != L2L_OK:
            raise L2LError(rc, "eps_adam_step_range")

    def adam_step_range16(self, block, first_elem, count, t, grad_dtype, lr=1e-4, beta1=0.9, beta2=0.999, eps_a=1e-8):
        rc = lib().eps_adam_step_range16(self._h, block, int(first_elem), int(count), t, lr, beta1, beta2, eps_a,
                                         DTYPES[grad_dtype] if isinstance(grad_dtype, str) else int(grad_dtype))
        if rc != L2L_OK:
            raise L2LError(rc, "eps_adam_step_range16")

    def enable_grad16(self):
        rc = lib().eps_enable_grad16(self._h)
        if rc != L2L_OK:
            raise L2LError(rc, "eps_enable_grad16")

    def grad16_ptr(self, block):
        return lib().eps_grad16(self._h, block)

    def grad16(self, block) -> np.ndarray:
        """the 16-bit landing buffer of a block, as raw bit patterns"""
        p = lib().eps_grad16(self._h, block)
        if not p:
            raise L2LError(L2L_E_STATE, "eps_grad16: not enabled")
        return np.ctypeslib.as_array(C.cast(p, C.POINTER(C.c_uint16)), shape=(self.elems[block],))

    def grad_widen(self, first, last, dtype):
        rc = lib().eps_grad_widen(self._h, first, last, DTYPES[dtype] if isinstance(dtype, str) else int(dtype))
        if rc != L2L_OK:
            raise L2LError(rc, "eps_grad_widen")

    def grad_widen_range(self, block, first_elem, count, dtype):
        rc = lib().eps_grad_widen_range(self._h, block, int(first_elem), int(count), DTYPES[dtype] if isinstance(dtype, str) else int(dtype))
        if rc != L2L_OK:
            raise L2LError(rc, "eps_grad_widen_range")

    def grad_unscale(self, first, last, inv_scale) -> bool:
        """landing buffers *= inv_scale; True if they hold an inf or NaN."""
        bad = C.c_int(0)
        rc = lib().eps_grad_unscale(self._h, first, last, inv_scale, C.byref(bad))
        if rc != L2L_OK:
            raise L2LError(rc, "eps_grad_unscale")
        return bool(bad.value)

    def grad_unscale_range(self, block, first_elem, count, inv_scale) -> bool:
        bad = C.c_int(0)
        rc = lib().eps_grad_unscale_range(self._h, block, int(first_elem), int(count), inv_scale, C.byref(bad))
        if rc != L2L_OK:
            raise L2LError(rc, "eps_grad_unscale_range")
        return bool(bad.value)

    def lamb_step(self, first, last, t, segments, lr=1e-3, beta1=0.9, beta2=0.999, eps_a=1e-6, weight_decay=0.0,
                  decay_mask=None):
        """segments: [(begin, end)] element ranges of the tensors inside each of the blocks [first, last];
        decay_mask: per-segment factor on weight_decay (None: 1 everywhere)."""
        n = len(segments)
        b = (C.c_longlong * n)(*[int(s[0]) for s in segments])
        e = (C.c_longlong * n)(*[int(s[1]) for s in segments])
        d = None if decay_mask is None else (C.c_double * n)(*[float(x) for x in decay_mask])
        rc = lib().eps_lamb_step(self._h, first, last, t, lr, beta1, beta2, eps_a, weight_decay, n, b, e, d)
        if rc != L2L_OK:
            raise L2LError(rc, "eps_lamb_step")

    def host_bytes(self):
        return lib().eps_host_bytes(self._h)

    def is_pinned(self):
        return bool(lib().eps_is_pinned(self._h))
