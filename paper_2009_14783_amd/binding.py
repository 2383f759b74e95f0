"""ctypes binding of libhetseq_hip.so: the same names as include/hetseq_hip.h, argument
marshalling only.  torch provides device memory and the stream; every step of the path runs
in the library's kernels.  A missing library is an error (there is no fallback)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhetseq_hip.so")

HS_FP32, HS_BF16 = 0, 1
STATUS = {0: "HS_OK", 1: "HS_ERR_INVALID_ARG", 2: "HS_ERR_SHAPE", 3: "HS_ERR_WORKSPACE", 4: "HS_ERR_STATE",
          5: "HS_ERR_HIP", 6: "HS_ERR_UNIMPLEMENTED"}


class hs_model_cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32), ("ffn", C.c_int32),
                ("vocab", C.c_int32), ("max_pos", C.c_int32), ("ln_eps", C.c_float), ("compute", C.c_int32)]


class hs_s2s_cfg(C.Structure):
    _fields_ = [("n_enc", C.c_int32), ("n_dec", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32), ("ffn", C.c_int32),
                ("vocab", C.c_int32), ("max_pos", C.c_int32), ("ln_eps", C.c_float), ("compute", C.c_int32)]


class hs_param_entry(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("offset", C.c_int64), ("rows", C.c_int32), ("cols", C.c_int32)]


class hs_profile_entry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("launches", C.c_int64), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


class hs_ckpt_header(C.Structure):
    _fields_ = [("cfg", hs_model_cfg), ("n_params", C.c_int64), ("epoch", C.c_int64), ("step", C.c_int64),
                ("seed", C.c_uint64), ("max_lr", C.c_double), ("warmup", C.c_int64), ("total", C.c_int64),
                ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double), ("weight_decay", C.c_double)]


class HsError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"{STATUS.get(status, status)}: {msg}")
        self.status = status


_lib = None

_P, _I32, _I64, _SZ, _F, _D = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float, C.c_double
_SIGNATURES = {
    "hs_ctx_create": (_I32, [C.POINTER(hs_model_cfg), C.POINTER(_P)]),
    "hs_ctx_destroy": (_I32, [_P]),
    "hs_last_error": (C.c_char_p, [_P]),
    "hs_param_count": (_SZ, [C.POINTER(hs_model_cfg)]),
    "hs_param_layout": (_I32, [C.POINTER(hs_model_cfg), C.POINTER(hs_param_entry), C.POINTER(_I32)]),
    "hs_acts_bytes": (_SZ, [C.POINTER(hs_model_cfg), _I32, _I32, _I32]),
    "hs_workspace_bytes": (_SZ, [C.POINTER(hs_model_cfg), _I32, _I32, _I32]),
    "hs_make_batches": (_I32, [_P, _I64, _I32, _I64, _I32, _P, _P, _P, C.POINTER(_I64)]),
    "hs_key_mask": (_I32, [_P, _I32, _I32, _P, _P]),
    "hs_encoder_fwd": (_I32, [_P, _P, _P, _P, _P, _I32, _I32, _P, _P, _P, _SZ, _P]),
    "hs_mlm_loss": (_I32, [_P, _P, _P, _P, _P, _I32, _I32, _I32, _P, _P, _P, _I32, _P, _SZ, _P]),
    "hs_encoder_bwd": (_I32, [_P, _P, _P, _P, _P, _I32, _I32, _P, _P, _I32, _P, _SZ, _P]),
    "hs_grad_accum_normalize": (_I32, [_P, _P, _SZ, _I32, _D, _P]),
    "hs_adam_step": (_I32, [_P, _P, _P, _P, _P, _SZ, _D, _D, _D, _D, _D, _I64, _P]),
    "hs_cast_params": (_I32, [_P, _P, _SZ, _I32, _P]),
    "hs_arm_update": (_I32, [_P, _P, _P, _P, _P, _P, _D, _D, _D, _D, _D, _D, _I64]),
    "hs_set_dropout": (_I32, [_P, _D, C.c_uint64, C.c_uint32]),
    "hs_dropout_keep_mask": (_I32, [_P, C.c_uint32, _SZ, _P, _P]),
    "hs_shard_write": (_I32, [C.c_char_p, _P, _I64, _P]),
    "hs_dataset_open": (_I32, [C.POINTER(C.c_char_p), _I32, _I64, _I32, C.POINTER(_P)]),
    "hs_dataset_close": (_I32, [_P]),
    "hs_dataset_size": (_I64, [_P]),
    "hs_dataset_lengths": (_I32, [_P, _P]),
    "hs_dataset_locate": (_I32, [_P, _I64, C.POINTER(_I32), C.POINTER(_I64)]),
    "hs_dataset_begin_epoch": (_I32, [_P, C.c_uint64, _I64, _I32, _I64, _I32, _I32, _I32, C.POINTER(_I64)]),
    "hs_dataset_peek": (_I32, [_P, C.POINTER(_I32), C.POINTER(_I32)]),
    "hs_dataset_next": (_I32, [_P, _P, _P, _P]),
    "hs_dataset_stats": (_I32, [_P, C.POINTER(_I64), C.POINTER(_I64)]),
    "hs_lr_linear": (_D, [_I64, _D, _I64, _I64]),
    "hs_checkpoint_write": (_I32, [C.c_char_p, C.POINTER(hs_ckpt_header), _P, _P, _P]),
    "hs_checkpoint_read_header": (_I32, [C.c_char_p, C.POINTER(hs_ckpt_header)]),
    "hs_checkpoint_read": (_I32, [C.c_char_p, C.POINTER(hs_ckpt_header), _P, _P, _P, _SZ]),
    "hs_profile_enable": (_I32, [_P, _I32]),
    "hs_profile_read": (_I32, [_P, C.POINTER(hs_profile_entry), C.POINTER(_I32)]),
    "hs_fill_zero": (_I32, [_P, _SZ, _P]),
    "hs_weighted_loss": (_I32, [_P, _I32, _D, _P, _P]),
    "hs_tune_gemm_variant": (_I32, [_I32]),
    "hs_op_gemm": (_I32, [_I32, _I32, _I32, _I32, _I32, _I32, _P, _I64, _P, _I64, _P, _I64, _I32, _F, _P, _I32, _P, _I64, _P, _P, _SZ, _P]),
    "hs_op_layernorm_fwd": (_I32, [_I32, _P, _P, _P, _P, _P, _I32, _I32, _F, _P]),
    "hs_op_layernorm_bwd_scratch": (_SZ, [_I32, _I32]),
    "hs_op_layernorm_bwd": (_I32, [_I32, _P, _P, _P, _P, _P, _P, _P, _P, _F, _I32, _I32, _P, _P]),
    "hs_op_layernorm_bwd_noalloc": (_I32, [_I32, _P, _P, _P, _P, _P, _P, _P, _P, _F, _I32, _I32, _P]),
    "hs_op_attention_fwd": (_I32, [_I32, _P, _P, _I32, _I32, _I32, _P, _P, _P]),
    "hs_op_attention_bwd": (_I32, [_I32, _P, _P, _P, _P, _P, _I32, _I32, _I32, _P, _P, _P]),
    "hs_s2s_ctx_create": (_I32, [C.POINTER(hs_s2s_cfg), C.POINTER(_P)]),
    "hs_s2s_param_count": (_SZ, [C.POINTER(hs_s2s_cfg)]),
    "hs_s2s_param_layout": (_I32, [C.POINTER(hs_s2s_cfg), C.POINTER(hs_param_entry), C.POINTER(_I32)]),
    "hs_s2s_acts_bytes": (_SZ, [C.POINTER(hs_s2s_cfg), _I32, _I32, _I32]),
    "hs_s2s_workspace_bytes": (_SZ, [C.POINTER(hs_s2s_cfg), _I32, _I32, _I32]),
    "hs_s2s_fwd": (_I32, [_P, _P, _P, _P, _P, _P, _I32, _I32, _I32, _P, _P, _P]),
    "hs_s2s_loss": (_I32, [_P, _P, _P, _P, _P, _P, _I32, _I32, _D, _P, _P, _P, _P, _I32, _P, _SZ, _P]),
    "hs_s2s_bwd": (_I32, [_P, _P, _P, _P, _P, _P, _P, _I32, _I32, _I32, _P, _P, _I32, _P, _SZ, _P]),
    "hs_op_attention_general_fwd": (_I32, [_I32, _P, _I64, _P, _P, _I64, _P, _P, _I32, _I32, _I32, _I32, _I32, _P, _P, _P]),
    "hs_op_attention_general_bwd": (_I32, [_I32, _P, _I64, _P, _P, _I64, _P, _P, _I32, _I32, _I32, _I32, _I32, _P, _P, _P, _P, _I64, _P,
                                           _P, _I64, _P, _P]),
}
EXPORTS = tuple(_SIGNATURES)


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise HsError(-1, f"{LIB_PATH} is missing: build it with `python -m paper_2009_14783_amd.build`")
        # torch ships its own HIP runtime under the same soname; it must be in the process first so
        # that this library binds to it (two runtimes in one process do not share devices or streams)
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def _ptr(t):
    """Device/host address of a torch tensor or numpy array (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _check(status, ctx=None):
    if status != 0:
        msg = lib().hs_last_error(ctx)
        raise HsError(status, msg.decode() if msg else "")


def make_cfg(n_layers, hidden, n_heads, ffn, vocab, max_pos, ln_eps=1e-12, compute=HS_BF16) -> hs_model_cfg:
    return hs_model_cfg(n_layers, hidden, n_heads, ffn, vocab, max_pos, ln_eps, compute)


# ---- host-only calls ---------------------------------------------------------------------
def hs_shard_write(path: str, sequences: list):
    lengths = np.array([len(q) for q in sequences], dtype=np.int32)
    tokens = np.concatenate([np.asarray(q, dtype=np.int32) for q in sequences]) if len(sequences) else np.zeros(0, np.int32)
    _check(lib().hs_shard_write(path.encode(), _ptr(lengths), len(sequences), _ptr(tokens) if tokens.size else None))


class Dataset:
    """Thin wrapper of the hs_dataset_* calls (argument marshalling only)."""

    def __init__(self, paths, cache_instances=0, prefetch_batches=2):
        arr = (C.c_char_p * len(paths))(*[p.encode() for p in paths])
        self.h = _P()
        _check(lib().hs_dataset_open(arr, len(paths), cache_instances, prefetch_batches, C.byref(self.h)))

    def close(self):
        if self.h:
            _check(lib().hs_dataset_close(self.h))
            self.h = None

    def __len__(self):
        return lib().hs_dataset_size(self.h)

    def lengths(self) -> np.ndarray:
        out = np.empty(len(self), dtype=np.int32)
        _check(lib().hs_dataset_lengths(self.h, _ptr(out)))
        return out

    def locate(self, instance: int):
        s, r = _I32(), _I64()
        _check(lib().hs_dataset_locate(self.h, instance, C.byref(s), C.byref(r)))
        return s.value, r.value

    def begin_epoch(self, seed, epoch, bucket_width, max_tokens, cap_mode=0, world=1, rank=0) -> int:
        n = _I64()
        _check(lib().hs_dataset_begin_epoch(self.h, seed & 0xFFFFFFFFFFFFFFFF, epoch, bucket_width, max_tokens, cap_mode, world, rank,
                                            C.byref(n)))
        return n.value

    def peek(self):
        b, l = _I32(), _I32()
        _check(lib().hs_dataset_peek(self.h, C.byref(b), C.byref(l)))
        return b.value, l.value

    def next(self, ids_out=None, lens_out=None):
        """Returns (ids [B, L], lens [B], instance indices [B]); ids_out / lens_out may be preallocated
        (for example pinned) int32 arrays or tensors of sufficient size."""
        B, L = self.peek()
        if B == 0:
            raise StopIteration
        ids = np.empty((B, L), dtype=np.int32) if ids_out is None else ids_out
        lens = np.empty(B, dtype=np.int32) if lens_out is None else lens_out
        inst = np.empty(B, dtype=np.int64)
        _check(lib().hs_dataset_next(self.h, _ptr(ids), _ptr(lens), _ptr(inst)))
        return ids, lens, inst

    def stats(self):
        a, b = _I64(), _I64()
        _check(lib().hs_dataset_stats(self.h, C.byref(a), C.byref(b)))
        return a.value, b.value


def hs_lr_linear(t, max_lr, warmup, total) -> float:
    lr = lib().hs_lr_linear(int(t), float(max_lr), int(warmup), int(total))
    if lr != lr:
        raise HsError(1, (lib().hs_last_error(None) or b"").decode())
    return lr


def hs_checkpoint_write(path: str, header: hs_ckpt_header, w: np.ndarray, m: np.ndarray, v: np.ndarray):
    """w, m, v: contiguous float32 HOST arrays of header.n_params elements."""
    for a in (w, m, v):
        assert isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags["C_CONTIGUOUS"] and a.size == header.n_params
    _check(lib().hs_checkpoint_write(path.encode(), C.byref(header), _ptr(w), _ptr(m), _ptr(v)))


def hs_checkpoint_read_header(path: str) -> hs_ckpt_header:
    h = hs_ckpt_header()
    _check(lib().hs_checkpoint_read_header(path.encode(), C.byref(h)))
    return h


def hs_checkpoint_read(path: str, w: np.ndarray, m: np.ndarray, v: np.ndarray) -> hs_ckpt_header:
    """Fills the contiguous float32 HOST arrays w, m, v (same size) and returns the header."""
    for a in (w, m, v):
        assert isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags["C_CONTIGUOUS"] and a.size == w.size
    h = hs_ckpt_header()
    _check(lib().hs_checkpoint_read(path.encode(), C.byref(h), _ptr(w), _ptr(m), _ptr(v), w.size))
    return h



def hs_ctx_create(cfg: hs_model_cfg):
    out = _P()
    _check(lib().hs_ctx_create(C.byref(cfg), C.byref(out)))
    return out


def hs_ctx_destroy(ctx):
    _check(lib().hs_ctx_destroy(ctx))


def hs_param_count(cfg) -> int:
    return int(lib().hs_param_count(C.byref(cfg)))


def hs_param_layout(cfg):
    """List of (name, offset, rows, cols)."""
    n = _I32(0)
    _check(lib().hs_param_layout(C.byref(cfg), None, C.byref(n)))
    arr = (hs_param_entry * n.value)()
    _check(lib().hs_param_layout(C.byref(cfg), arr, C.byref(n)))
    return [(e.name.decode(), int(e.offset), int(e.rows), int(e.cols)) for e in arr[:n.value]]


def hs_acts_bytes(cfg, B, L, M) -> int:
    return int(lib().hs_acts_bytes(C.byref(cfg), B, L, M))


def hs_workspace_bytes(cfg, B, L, M) -> int:
    return int(lib().hs_workspace_bytes(C.byref(cfg), B, L, M))


def hs_make_batches(lengths, bucket_width, max_tokens, cap_mode=0):
    """Returns (seq_index, batch_offsets, batch_pad_len) as numpy arrays trimmed to size."""
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    n = lengths.size
    seq = np.zeros(max(n, 1), dtype=np.int32)
    offs = np.zeros(n + 1, dtype=np.int64)
    pads = np.zeros(max(n, 1), dtype=np.int32)
    nb = _I64(0)
    _check(lib().hs_make_batches(lengths.ctypes.data, n, bucket_width, max_tokens, cap_mode, seq.ctypes.data,
                                 offs.ctypes.data, pads.ctypes.data, C.byref(nb)))
    return seq[:n], offs[:nb.value + 1], pads[:nb.value]


# ---- device calls --------------------------------------------------------------------------
def hs_key_mask(lens, B, L, mask_out, stream=None):
    _check(lib().hs_key_mask(_ptr(lens), B, L, _ptr(mask_out), _stream(stream)))


def hs_encoder_fwd(ctx, w, ids, lens, lens_host, B, L, acts, hidden_out, workspace, workspace_bytes, stream=None):
    _check(lib().hs_encoder_fwd(ctx, _ptr(w), _ptr(ids), _ptr(lens), _ptr(lens_host), B, L, _ptr(acts), _ptr(hidden_out),
                                _ptr(workspace), workspace_bytes, _stream(stream)), ctx)


def hs_mlm_loss(ctx, w, hidden, mlm_pos, mlm_label, M, B, L, loss_sum, d_hidden, g, accumulate, workspace,
                workspace_bytes, stream=None):
    _check(lib().hs_mlm_loss(ctx, _ptr(w), _ptr(hidden), _ptr(mlm_pos), _ptr(mlm_label), M, B, L, _ptr(loss_sum),
                             _ptr(d_hidden), _ptr(g), accumulate, _ptr(workspace), workspace_bytes, _stream(stream)), ctx)


def hs_encoder_bwd(ctx, w, acts, ids, lens, B, L, d_hidden, g, accumulate, workspace, workspace_bytes, stream=None):
    _check(lib().hs_encoder_bwd(ctx, _ptr(w), _ptr(acts), _ptr(ids), _ptr(lens), B, L, _ptr(d_hidden), _ptr(g), accumulate,
                                _ptr(workspace), workspace_bytes, _stream(stream)), ctx)


def hs_arm_update(ctx, w, m, v, G, w_lowp_out, denom, lr, beta1, beta2, eps, weight_decay, t):
    _check(lib().hs_arm_update(ctx, _ptr(w), _ptr(m), _ptr(v), _ptr(G), _ptr(w_lowp_out), float(denom), lr, beta1, beta2, eps,
                               weight_decay, t), ctx)


def hs_set_dropout(ctx, p, seed, stream_no):
    _check(lib().hs_set_dropout(ctx, float(p), int(seed) & 0xFFFFFFFFFFFFFFFF, int(stream_no) & 0xFFFFFFFF), ctx)


def hs_dropout_keep_mask(ctx, site, n, mask_out, stream=None):
    _check(lib().hs_dropout_keep_mask(ctx, int(site), int(n), _ptr(mask_out), _stream(stream)), ctx)


def hs_grad_accum_normalize(G, g, n, ignore, denom, stream=None):
    _check(lib().hs_grad_accum_normalize(_ptr(G), _ptr(g), n, ignore, float(denom), _stream(stream)))


def hs_adam_step(w, m, v, G, w_lowp_out, n, lr, beta1, beta2, eps, weight_decay, t, stream=None):
    _check(lib().hs_adam_step(_ptr(w), _ptr(m), _ptr(v), _ptr(G), _ptr(w_lowp_out), n, lr, beta1, beta2, eps, weight_decay,
                              t, _stream(stream)))


def hs_cast_params(src, dst, n, dst_dtype, stream=None):
    _check(lib().hs_cast_params(_ptr(src), _ptr(dst), n, dst_dtype, _stream(stream)))


def hs_profile_enable(ctx, on):
    _check(lib().hs_profile_enable(ctx, 1 if on else 0), ctx)


def hs_profile_read(ctx):
    """dict name -> dict(launches, ms, flops, bytes); synchronises the recorded events."""
    n = _I32(32)
    arr = (hs_profile_entry * 32)()
    _check(lib().hs_profile_read(ctx, arr, C.byref(n)), ctx)
    return {e.name.decode(): dict(launches=int(e.launches), ms=float(e.ms), flops=float(e.flops), bytes=float(e.bytes))
            for e in arr[:n.value]}


def hs_op_gemm(dtype, a_kmajor, b_kmajor, M, N, K, A, lda, B, ldb, Cm, ldc, c_f32=0, beta=0.0, bias=None, epi=0, aux=None,
               ldaux=0, C2=None, scratch=None, scratch_bytes=0, stream=None):
    _check(lib().hs_op_gemm(dtype, a_kmajor, b_kmajor, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(Cm), ldc, c_f32, beta,
                            _ptr(bias), epi, _ptr(aux), ldaux, _ptr(C2), _ptr(scratch), scratch_bytes, _stream(stream)))


def hs_tune_gemm_variant(variant: int):
    _check(lib().hs_tune_gemm_variant(int(variant)))


def hs_op_layernorm_fwd(dtype, x, gain, bias, y, stats, R, H, eps, stream=None):
    _check(lib().hs_op_layernorm_fwd(dtype, _ptr(x), _ptr(gain), _ptr(bias), _ptr(y), _ptr(stats), R, H, eps, _stream(stream)))


def hs_fill_zero(dst, nbytes, stream=None):
    _check(lib().hs_fill_zero(_ptr(dst), nbytes, _stream(stream)))


def hs_weighted_loss(loss_sums, n, denom, loss_out, stream=None):
    _check(lib().hs_weighted_loss(_ptr(loss_sums), n, float(denom), _ptr(loss_out), _stream(stream)))


def hs_op_layernorm_bwd_scratch(R, H) -> int:
    return int(lib().hs_op_layernorm_bwd_scratch(R, H))


def hs_op_layernorm_bwd(dtype, dy, x, stats, gain, dx, d_gain, d_bias, d_colsum, beta, R, H, partials, stream=None):
    _check(lib().hs_op_layernorm_bwd(dtype, _ptr(dy), _ptr(x), _ptr(stats), _ptr(gain), _ptr(dx), _ptr(d_gain), _ptr(d_bias),
                                     _ptr(d_colsum), beta, R, H, _ptr(partials), _stream(stream)))


def hs_op_layernorm_bwd_noalloc(dtype, dy, x, stats, gain, dx, d_gain, d_bias, d_colsum, beta, R, H, stream=None):
    _check(lib().hs_op_layernorm_bwd_noalloc(dtype, _ptr(dy), _ptr(x), _ptr(stats), _ptr(gain), _ptr(dx), _ptr(d_gain),
                                             _ptr(d_bias), _ptr(d_colsum), beta, R, H, _stream(stream)))


def hs_op_attention_fwd(dtype, qkv, lens, B, L, A, ctx_out, lse, stream=None):
    _check(lib().hs_op_attention_fwd(dtype, _ptr(qkv), _ptr(lens), B, L, A, _ptr(ctx_out), _ptr(lse), _stream(stream)))


def hs_op_attention_bwd(dtype, qkv, ctx_in, lse, d_ctx, lens, B, L, A, dqkv, dvec, stream=None):
    _check(lib().hs_op_attention_bwd(dtype, _ptr(qkv), _ptr(ctx_in), _ptr(lse), _ptr(d_ctx), _ptr(lens), B, L, A, _ptr(dqkv),
                                     _ptr(dvec), _stream(stream)))


# ---- translation workload -----------------------------------------------------------------
def make_s2s_cfg(n_enc, n_dec, hidden, n_heads, ffn, vocab, max_pos, ln_eps=1e-5, compute=HS_BF16) -> hs_s2s_cfg:
    return hs_s2s_cfg(n_enc, n_dec, hidden, n_heads, ffn, vocab, max_pos, ln_eps, compute)


def hs_s2s_ctx_create(cfg: hs_s2s_cfg):
    h = _P()
    _check(lib().hs_s2s_ctx_create(C.byref(cfg), C.byref(h)))
    return h


def hs_s2s_param_count(cfg) -> int:
    return int(lib().hs_s2s_param_count(C.byref(cfg)))


def hs_s2s_param_layout(cfg):
    """List of (name, offset, rows, cols)."""
    n = _I32(0)
    _check(lib().hs_s2s_param_layout(C.byref(cfg), None, C.byref(n)))
    arr = (hs_param_entry * n.value)()
    _check(lib().hs_s2s_param_layout(C.byref(cfg), arr, C.byref(n)))
    return [(e.name.decode(), int(e.offset), int(e.rows), int(e.cols)) for e in arr[:n.value]]


def hs_s2s_acts_bytes(cfg, B, Ls, Lt) -> int:
    return int(lib().hs_s2s_acts_bytes(C.byref(cfg), B, Ls, Lt))


def hs_s2s_workspace_bytes(cfg, B, Ls, Lt) -> int:
    return int(lib().hs_s2s_workspace_bytes(C.byref(cfg), B, Ls, Lt))


def hs_s2s_fwd(ctx, w, src, src_lens, tgt_in, tgt_lens, B, Ls, Lt, acts, dec_out, stream=None):
    _check(lib().hs_s2s_fwd(ctx, _ptr(w), _ptr(src), _ptr(src_lens), _ptr(tgt_in), _ptr(tgt_lens), B, Ls, Lt, _ptr(acts), _ptr(dec_out),
                            _stream(stream)), ctx)


def hs_s2s_loss(ctx, w, dec_out, tgt_out, tgt_lens, tgt_lens_host, B, Lt, eps, loss_sum, nll_sum, d_dec_out, g, accumulate, workspace,
                workspace_bytes, stream=None):
    _check(lib().hs_s2s_loss(ctx, _ptr(w), _ptr(dec_out), _ptr(tgt_out), _ptr(tgt_lens), _ptr(tgt_lens_host), B, Lt, float(eps), _ptr(loss_sum),
                             _ptr(nll_sum),
                             _ptr(d_dec_out), _ptr(g), accumulate, _ptr(workspace), workspace_bytes, _stream(stream)), ctx)


def hs_s2s_bwd(ctx, w, acts, src, src_lens, tgt_in, tgt_lens, B, Ls, Lt, d_dec_out, g, accumulate, workspace, workspace_bytes, stream=None):
    _check(lib().hs_s2s_bwd(ctx, _ptr(w), _ptr(acts), _ptr(src), _ptr(src_lens), _ptr(tgt_in), _ptr(tgt_lens), B, Ls, Lt, _ptr(d_dec_out),
                            _ptr(g), accumulate, _ptr(workspace), workspace_bytes, _stream(stream)), ctx)


def hs_op_attention_general_fwd(dtype, q, ldq, k, v, ldkv, qlens, klens, B, Lq, Lk, A, causal, ctx_out, lse, stream=None):
    _check(lib().hs_op_attention_general_fwd(dtype, _ptr(q), ldq, _ptr(k), _ptr(v), ldkv, _ptr(qlens), _ptr(klens), B, Lq, Lk, A, causal,
                                             _ptr(ctx_out), _ptr(lse), _stream(stream)))


def hs_op_attention_general_bwd(dtype, q, ldq, k, v, ldkv, qlens, klens, B, Lq, Lk, A, causal, ctx_in, lse, d_ctx, dq, lddq, dk, dv, lddkv,
                                dvec, stream=None):
    _check(lib().hs_op_attention_general_bwd(dtype, _ptr(q), ldq, _ptr(k), _ptr(v), ldkv, _ptr(qlens), _ptr(klens), B, Lq, Lk, A, causal,
                                             _ptr(ctx_in), _ptr(lse), _ptr(d_ctx), _ptr(dq), lddq, _ptr(dk), _ptr(dv), lddkv, _ptr(dvec),
                                             _stream(stream)))
