"""ctypes binding of libzo.so: argument marshalling only.

Every function here has the name and the argument order of the C entry point
in include/zo.h; tensors are torch tensors already resident on the device (or
plain integers holding device pointers) and are passed as raw pointers.  No
step of the path is computed here, and there is no fallback: if the shared
library is missing, loading fails with an error that says how to build it.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libzo.so")

ZO_F32, ZO_BF16 = 0, 1
ZO_OK = 0
ZO_LAYER_NORM, ZO_RMS_NORM = 0, 1
ZO_ERR_NULL, ZO_ERR_SHAPE, ZO_ERR_INDEX, ZO_ERR_BANK_FULL = -1, -2, -3, -4
ZO_ERR_WORKSPACE, ZO_ERR_UNSUPPORTED, ZO_ERR_HIP = -5, -6, -7

_c_i32p = C.POINTER(C.c_int32)
_c_f32p = C.POINTER(C.c_float)
_c_u64p = C.POINTER(C.c_uint64)


class zo_batch(C.Structure):
    _fields_ = [("n_tokens", C.c_int32), ("n_seqs", C.c_int32),
                ("cu_seqlens", C.c_void_p), ("seq_cand", C.c_void_p),
                ("n_cands", C.c_int32), ("cand_dir", C.c_void_p), ("cand_sign", C.c_void_p),
                ("n_dirs", C.c_int32), ("dir_seed", C.c_void_p),
                ("host_cu_seqlens", C.c_void_p), ("host_seq_cand", C.c_void_p),
                ("host_cand_dir", C.c_void_p), ("dir_seed_v", C.c_void_p)]


class zo_bank(C.Structure):
    _fields_ = [("R_cap", C.c_int32), ("R_used", C.c_int32), ("P", C.c_void_p), ("Vb", C.c_void_p)]


class zo_layer_bank(C.Structure):
    _fields_ = [("bank", zo_bank), ("m", C.c_int32), ("n", C.c_int32), ("tensor_id", C.c_uint32),
                ("reserved", C.c_int32)]


class zo_sched(C.Structure):
    """Layout of the device-resident schedule state (for host-side initialisation and read-back)."""
    _fields_ = [("next_step", C.c_int64), ("step", C.c_int64), ("interval", C.c_int32), ("block", C.c_int32),
                ("append", C.c_int32), ("reserved", C.c_int32)]


class ZoError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("zo status %d: %s" % (status, message))
        self.status = status


_lib = None

_PROTOS = {
    "zo_version": (C.c_int32, []),
    "zo_last_error": (C.c_size_t, [C.c_char_p, C.c_size_t]),
    "zo_philox_words": (C.c_int32, [C.c_uint64, C.c_uint32, C.c_uint64, C.c_int64, C.c_void_p, C.c_void_p]),
    "zo_factor_fill": (C.c_int32, [C.c_uint64, C.c_uint32, C.c_int64, C.c_int32, C.c_int, C.c_void_p, C.c_void_p]),
    "zo_batch_index": (C.c_int32, [C.POINTER(zo_batch), C.c_void_p, C.c_void_p, C.c_void_p]),
    "zo_probe_linear_workspace_bytes": (C.c_size_t, [C.c_int32] * 7 + [C.c_int]),
    "zo_probe_linear": (C.c_int32, [C.POINTER(zo_batch), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                    C.c_int32, C.c_int32, C.c_int, C.c_int32, C.c_float, C.c_uint32,
                                    C.POINTER(zo_bank), C.c_int32, C.c_void_p, C.c_int64, C.c_int,
                                    C.c_void_p, C.c_size_t, C.c_void_p]),
    "zo_score_workspace_bytes": (C.c_size_t, [C.c_int32] * 4 + [C.c_int]),
    "zo_score": (C.c_int32, [C.POINTER(zo_batch), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                             C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                             C.c_void_p, C.c_size_t, C.c_void_p]),
    "zo_score_static_capacity": (C.c_size_t, []),
    "zo_score_static": (C.c_int32, [C.POINTER(zo_batch), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32,
                                    C.c_int32, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p]),
    "zo_estimate": (C.c_int32, [C.POINTER(zo_batch), C.c_void_p, C.c_void_p, C.c_float, C.c_int32, C.c_void_p,
                                C.c_void_p, C.c_void_p]),
    "zo_bank_update": (C.c_int32, [C.POINTER(zo_bank), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                   C.c_void_p, C.c_uint32, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_int32,
                                   C.c_int, C.c_void_p]),
    "zo_schedule_step": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_uint64, C.c_uint64,
                                     C.c_void_p, C.c_void_p, C.c_void_p]),
    "zo_estimate_es": (C.c_int32, [C.POINTER(zo_batch), C.c_void_p, C.c_void_p, C.c_float, C.c_int32, C.c_void_p,
                                   C.c_void_p, C.c_void_p]),
    "zo_fold_bank": (C.c_int32, [C.POINTER(zo_bank), C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int, C.c_void_p]),
    "zo_bank_update_scheduled": (C.c_int32, [C.POINTER(zo_bank), C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_float, C.c_void_p,
                                             C.c_void_p, C.c_int32, C.c_int, C.c_void_p]),
    "zo_add_norm": (C.c_int32, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int32,
                                C.c_float, C.c_int32, C.c_int32, C.c_int, C.c_void_p, C.c_int64, C.c_void_p,
                                C.c_int64, C.c_void_p]),
    "zo_attention": (C.c_int32, [C.POINTER(zo_batch), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                 C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_int, C.c_void_p,
                                 C.c_int64, C.c_void_p]),
    "zo_qk_norm_rope": (C.c_int32, [C.POINTER(zo_batch), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32,
                                    C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_float, C.c_float, C.c_int,
                                    C.c_void_p]),
    "zo_bank_update_multi": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_float, C.c_void_p, C.c_void_p, C.c_int32, C.c_int, C.c_void_p]),
}
EXPORTS = tuple(_PROTOS)


def lib():
    """Loads libzo.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_2605_28760_amd.build` "
                               "(there is no fallback path)" % LIB_PATH)
        # The caller's device memory comes from torch, which ships its own HIP runtime;
        # load it first so that libzo.so binds to the same runtime instance (two runtimes
        # in one process do not see each other's device state).
        import torch  # noqa: F401
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in _PROTOS.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def last_error():
    buf = C.create_string_buffer(1024)
    lib().zo_last_error(buf, 1024)
    return buf.value.decode()


def _check(status):
    if status != ZO_OK:
        raise ZoError(status, last_error())


def _ptr(x):
    """Raw address of a torch tensor, a ctypes array / numpy array (host), an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    return C.addressof(x)


def _stream(stream):
    if stream is None:
        return None
    return getattr(stream, "cuda_stream", stream)


def make_batch(n_tokens, cu_seqlens, seq_cand, cand_dir, cand_sign, dir_seed,
               host_cu_seqlens=None, host_seq_cand=None, host_cand_dir=None,
               n_seqs=None, n_cands=None, n_dirs=None, dir_seed_v=None):
    """Fills a zo_batch from device tensors (and optional host numpy mirrors).
    The caller keeps the tensors alive for as long as the struct is used."""
    b = zo_batch()
    b.n_tokens = int(n_tokens)
    b.n_seqs = int(len(seq_cand) if n_seqs is None else n_seqs)
    b.n_cands = int(len(cand_dir) if n_cands is None else n_cands)
    b.n_dirs = int(len(dir_seed) if n_dirs is None else n_dirs)
    b.cu_seqlens, b.seq_cand = _ptr(cu_seqlens), _ptr(seq_cand)
    b.cand_dir, b.cand_sign, b.dir_seed = _ptr(cand_dir), _ptr(cand_sign), _ptr(dir_seed)
    b.host_cu_seqlens, b.host_seq_cand, b.host_cand_dir = _ptr(host_cu_seqlens), _ptr(host_seq_cand), _ptr(host_cand_dir)
    b.dir_seed_v = _ptr(dir_seed_v)
    b._keep = (cu_seqlens, seq_cand, cand_dir, cand_sign, dir_seed, host_cu_seqlens, host_seq_cand, host_cand_dir,
               dir_seed_v)
    return b


def make_bank(R_cap, R_used, P, Vb):
    k = zo_bank()
    k.R_cap, k.R_used, k.P, k.Vb = int(R_cap), int(R_used), _ptr(P), _ptr(Vb)
    k._keep = (P, Vb)
    return k


def zo_version():
    return lib().zo_version()


def zo_philox_words(seed, tensor_id, first_block, n_blocks, out_words, stream=None):
    _check(lib().zo_philox_words(seed, tensor_id, first_block, n_blocks, _ptr(out_words), _stream(stream)))


def zo_factor_fill(seed, tensor_id, rows, r, dtype, out, stream=None):
    _check(lib().zo_factor_fill(seed, tensor_id, rows, r, dtype, _ptr(out), _stream(stream)))


def zo_batch_index(batch, tok_seq, tok_cand, stream=None):
    _check(lib().zo_batch_index(C.byref(batch), _ptr(tok_seq), _ptr(tok_cand), _stream(stream)))


def zo_probe_linear_workspace_bytes(n_tokens, n_seqs, n_dirs, m, n, r, R_used, in_dtype):
    return lib().zo_probe_linear_workspace_bytes(n_tokens, n_seqs, n_dirs, m, n, r, R_used, in_dtype)


def zo_probe_linear(batch, X, ldx, W, ldw, bias, m, n, in_dtype, r, eps, tensor_id, bank, act,
                    Y, ldy, out_dtype, workspace, workspace_bytes, stream=None):
    _check(lib().zo_probe_linear(C.byref(batch), _ptr(X), ldx, _ptr(W), ldw, _ptr(bias), m, n, in_dtype, r, eps,
                                 tensor_id, C.byref(bank) if bank is not None else None, act, _ptr(Y), ldy,
                                 out_dtype, _ptr(workspace), workspace_bytes, _stream(stream)))


def zo_score_workspace_bytes(n_tokens, n_seqs, vocab, d, dtype):
    return lib().zo_score_workspace_bytes(n_tokens, n_seqs, vocab, d, dtype)


def zo_score(batch, H, ldh, W_head, ldw, vocab, d, dtype, targets, tok_nll, seq_nll, cand_sum, cand_cnt,
             workspace, workspace_bytes, stream=None):
    _check(lib().zo_score(C.byref(batch), _ptr(H), ldh, _ptr(W_head), ldw, vocab, d, dtype, _ptr(targets),
                          _ptr(tok_nll), _ptr(seq_nll), _ptr(cand_sum), _ptr(cand_cnt), _ptr(workspace),
                          workspace_bytes, _stream(stream)))


def zo_score_static_capacity():
    return lib().zo_score_static_capacity()


def zo_score_static(batch, H, ldh, W_head, ldw, vocab, d, dtype, targets, tok_nll, seq_nll, cand_sum, cand_cnt,
                    stream=None):
    _check(lib().zo_score_static(C.byref(batch), _ptr(H), ldh, _ptr(W_head), ldw, vocab, d, dtype, _ptr(targets),
                                 _ptr(tok_nll), _ptr(seq_nll), _ptr(cand_sum), _ptr(cand_cnt), _stream(stream)))


def zo_estimate(batch, cand_sum, cand_cnt, eps, reduction, cand_loss, proj_grad, stream=None):
    _check(lib().zo_estimate(C.byref(batch), _ptr(cand_sum), _ptr(cand_cnt), eps, reduction, _ptr(cand_loss),
                             _ptr(proj_grad), _stream(stream)))


def zo_bank_update(bank, m, n, r, n_dirs, dir_seed, tensor_id, proj_grad, lr, dir_weight, host_col0, append,
                   factor_dtype, stream=None, dir_seed_v=None):
    _check(lib().zo_bank_update(C.byref(bank), m, n, r, n_dirs, _ptr(dir_seed), _ptr(dir_seed_v), tensor_id,
                                _ptr(proj_grad), lr, _ptr(dir_weight), _ptr(host_col0), append, factor_dtype,
                                _stream(stream)))


def zo_schedule_step(sched, nu, n_blocks, n_dirs, base_u, base_v, dir_seed, dir_seed_v, stream=None):
    _check(lib().zo_schedule_step(_ptr(sched), nu, n_blocks, n_dirs, base_u, base_v, _ptr(dir_seed),
                                  _ptr(dir_seed_v), _stream(stream)))


def zo_bank_update_scheduled(bank, m, n, r, n_dirs, dir_seed, dir_seed_v, tensor_id, proj_grad, lr, dir_weight,
                             sched, n_blocks, factor_dtype, stream=None):
    _check(lib().zo_bank_update_scheduled(C.byref(bank), m, n, r, n_dirs, _ptr(dir_seed), _ptr(dir_seed_v), tensor_id,
                                          _ptr(proj_grad), lr, _ptr(dir_weight), _ptr(sched), n_blocks, factor_dtype,
                                          _stream(stream)))


def zo_fold_bank(bank, W, ldw, m, n, dtype, stream=None):
    _check(lib().zo_fold_bank(C.byref(bank), _ptr(W), ldw, m, n, dtype, _stream(stream)))


def zo_estimate_es(batch, cand_sum, cand_cnt, eps, reduction, cand_loss, proj_grad, stream=None):
    _check(lib().zo_estimate_es(C.byref(batch), _ptr(cand_sum), _ptr(cand_cnt), eps, reduction, _ptr(cand_loss),
                                _ptr(proj_grad), _stream(stream)))


def zo_add_norm(X, ldx, R, ldr, gamma, beta, kind, norm_eps, n_tokens, d, dtype, Hsum, ldh, Y, ldy, stream=None):
    _check(lib().zo_add_norm(_ptr(X), ldx, _ptr(R), ldr, _ptr(gamma), _ptr(beta), kind, norm_eps, n_tokens, d,
                             dtype, _ptr(Hsum), ldh, _ptr(Y), ldy, _stream(stream)))


def zo_attention(batch, Q, ldq, K, ldk, V, ldv, n_heads, n_kv_heads, head_dim, scale, dtype, O, ldo, stream=None):
    _check(lib().zo_attention(C.byref(batch), _ptr(Q), ldq, _ptr(K), ldk, _ptr(V), ldv, n_heads, n_kv_heads,
                              head_dim, scale, dtype, _ptr(O), ldo, _stream(stream)))


def zo_qk_norm_rope(batch, Q, ldq, K, ldk, n_heads, n_kv_heads, head_dim, gamma_q, gamma_k, norm_eps, rope_theta,
                    dtype, stream=None):
    _check(lib().zo_qk_norm_rope(C.byref(batch), _ptr(Q), ldq, _ptr(K), ldk, n_heads, n_kv_heads, head_dim,
                                 _ptr(gamma_q), _ptr(gamma_k), norm_eps, rope_theta, dtype, _stream(stream)))


def make_layer_banks(entries):
    """entries: sequence of (zo_bank, m, n, tensor_id).  Returns a ctypes array of zo_layer_bank that shares
    nothing with the given structs: R_used changes made by an append are read back from the array."""
    arr = (zo_layer_bank * len(entries))()
    for i, (bank, m, n, tid) in enumerate(entries):
        arr[i].bank.R_cap, arr[i].bank.R_used, arr[i].bank.P, arr[i].bank.Vb = bank.R_cap, bank.R_used, bank.P, bank.Vb
        arr[i].m, arr[i].n, arr[i].tensor_id = m, n, tid
    return arr


def zo_bank_update_multi(layers, r, n_dirs, dir_seed, dir_seed_v, proj_grad, lr, dir_weight, host_col0, append,
                         factor_dtype, stream=None):
    _check(lib().zo_bank_update_multi(C.addressof(layers) if len(layers) else None, len(layers), r, n_dirs,
                                      _ptr(dir_seed), _ptr(dir_seed_v), _ptr(proj_grad), lr, _ptr(dir_weight),
                                      _ptr(host_col0), append, factor_dtype, _stream(stream)))
