"""ctypes binding of include/ea.h and include/ea_profile.h -- same names, argument marshalling only.

Tensor arguments are torch CUDA tensors (or anything with .data_ptr()); `stream` is a
torch.cuda.Stream, a raw hipStream_t integer, or None for torch's current stream."""
import ctypes
import os

EA_F32, EA_BF16, EA_FP8_E4M3 = 0, 1, 2
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class EaError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s: %s (status %d)" % (where, status_string(code), code))


class EaParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("rope_layout", ctypes.c_int32),
                ("q_is_rotated", ctypes.c_int32), ("cov_ddof", ctypes.c_int32),
                ("horizon_T", ctypes.c_int32), ("epsilon", ctypes.c_float)]


class EaPaged(ctypes.Structure):
    _fields_ = [("block_table", ctypes.c_void_p), ("block_size", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("num_blocks", ctypes.c_int64)]


def lib_path():
    """In-tree libea.so; the environment variable EA_LIBRARY names another build of it."""
    return os.environ.get("EA_LIBRARY") or os.path.join(_HERE, "libea.so")


def load_library():
    """Loads libea.so (built in-tree by paper_2510_00636_amd.build).  Raises if it is absent:
    there is deliberately no fallback implementation."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError("libea.so not found at %s -- run `python -m paper_2510_00636_amd.build` "
                           "(or __graft_entry__.build()) first" % path)
    lib = ctypes.CDLL(path)
    P, VP, I64, SZ = ctypes.POINTER(EaParams), ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    lib.ea_workspace_bytes.restype = SZ
    lib.ea_workspace_bytes.argtypes = [P, I64, I64]
    lib.ea_query_stats.restype = ctypes.c_int
    lib.ea_query_stats.argtypes = [P, VP, I64, I64, VP, I64, VP, VP, VP, SZ, VP]
    lib.ea_query_stats_hidden.restype = ctypes.c_int
    lib.ea_query_stats_hidden.argtypes = [P, VP, VP, I64, I64, VP, I64, VP, VP, VP, SZ, VP]
    lib.ea_score.restype = ctypes.c_int
    lib.ea_score.argtypes = [P, VP, VP, I64, I64, VP, VP, VP, VP, SZ, VP]
    lib.ea_select.restype = ctypes.c_int
    lib.ea_select.argtypes = [P, VP, I64, I64, VP, VP, SZ, VP]
    lib.ea_wo_gram.restype = ctypes.c_int
    lib.ea_wo_gram.argtypes = [P, VP, I64, VP, VP]
    lib.ea_value_norms_wo.restype = ctypes.c_int
    lib.ea_value_norms_wo.argtypes = [P, VP, I64, I64, VP, VP, VP, SZ, VP]
    lib.ea_score_wo.restype = ctypes.c_int
    lib.ea_score_wo.argtypes = [P, VP, VP, I64, I64, VP, VP, VP, VP, VP, SZ, VP]
    lib.ea_select_static.restype = ctypes.c_int
    lib.ea_select_static.argtypes = [P, VP, I64, I64, VP, VP]
    lib.ea_compact.restype = ctypes.c_int
    lib.ea_compact.argtypes = [P, VP, VP, I64, I64, VP, I64, VP, VP, VP, SZ, VP]
    lib.ea_compress_layer.restype = ctypes.c_int
    lib.ea_compress_layer.argtypes = [P, VP, I64, I64, VP, I64, VP, VP, I64, I64, I64, VP, VP, VP, SZ, VP]
    lib.ea_select_adaptive.restype = ctypes.c_int
    lib.ea_select_adaptive.argtypes = [P, VP, I64, I64, I64, VP, VP, VP, SZ, VP]
    lib.ea_compress_layer_adaptive.restype = ctypes.c_int
    lib.ea_compress_layer_adaptive.argtypes = [P, VP, I64, I64, VP, I64, VP, VP, I64, I64, I64, I64, VP, VP, VP, VP,
                                               SZ, VP]
    lib.ea_compact_ragged.restype = ctypes.c_int
    lib.ea_compact_ragged.argtypes = [P, VP, VP, I64, I64, VP, VP, VP, SZ, VP]
    lib.ea_score_baseline.restype = ctypes.c_int
    lib.ea_score_baseline.argtypes = [P, ctypes.c_int32, VP, I64, I64, I64, VP, VP, SZ, VP]
    lib.ea_compact_unordered.restype = ctypes.c_int
    lib.ea_compact_unordered.argtypes = [P, VP, VP, I64, I64, VP, I64, VP, VP]
    lib.ea_compress_layer_unordered.restype = ctypes.c_int
    lib.ea_compress_layer_unordered.argtypes = [P, VP, I64, I64, VP, I64, VP, VP, I64, I64, I64, VP, VP, VP, VP, SZ, VP]
    PG = ctypes.POINTER(EaPaged)
    lib.ea_score_paged.restype = ctypes.c_int
    lib.ea_score_paged.argtypes = [P, VP, VP, PG, I64, VP, VP, VP, VP, SZ, VP]
    lib.ea_compact_paged.restype = ctypes.c_int
    lib.ea_compact_paged.argtypes = [P, VP, VP, PG, I64, VP, I64, ctypes.c_int32, VP, VP, SZ, VP]
    lib.ea_compress_layer_paged.restype = ctypes.c_int
    lib.ea_compress_layer_paged.argtypes = [P, VP, I64, I64, VP, I64, VP, VP, PG, I64, I64, ctypes.c_int32,
                                            VP, VP, VP, VP, SZ, VP]
    lib.ea_score_fp8.restype = ctypes.c_int
    lib.ea_score_fp8.argtypes = [P, VP, VP, VP, VP, I64, I64, VP, VP, VP, VP, SZ, VP]
    lib.ea_compress_layer_fp8.restype = ctypes.c_int
    lib.ea_compress_layer_fp8.argtypes = [P, VP, I64, I64, VP, I64, VP, VP, VP, VP, I64, I64, I64, ctypes.c_int32,
                                          VP, VP, VP, VP, SZ, VP]
    lib.ea_compress_layer_timed.restype = ctypes.c_int
    lib.ea_compress_layer_timed.argtypes = [P, VP, I64, I64, VP, I64, VP, VP, I64, I64, I64, VP, SZ, VP,
                                            ctypes.POINTER(ctypes.c_float)]
    lib.ea_debug_status.restype = ctypes.c_int
    lib.ea_debug_status.argtypes = [P, I64, I64, VP, SZ, VP, ctypes.POINTER(ctypes.c_uint32)]
    lib.ea_n_keep.restype = I64
    lib.ea_n_keep.argtypes = [I64, ctypes.c_double]
    lib.ea_status_string.restype = ctypes.c_char_p
    lib.ea_status_string.argtypes = [ctypes.c_int]
    _LIB = lib
    return lib


def make_params(batch, n_q_heads, n_kv_heads, head_dim, dtype, rope_layout=0, q_is_rotated=1,
                cov_ddof=0, horizon_T=512, epsilon=0.02):
    return EaParams(batch, n_q_heads, n_kv_heads, head_dim, dtype, rope_layout, q_is_rotated,
                    cov_ddof, horizon_T, epsilon)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _nbytes(t):
    return t.numel() * t.element_size()


def _stream(s):
    if s is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(s, int):
        return ctypes.c_void_p(s)
    return ctypes.c_void_p(s.cuda_stream)


def _check(code, where):
    if code != 0:
        raise EaError(code, where)


def status_string(code):
    return load_library().ea_status_string(int(code)).decode()


def n_keep(n, ratio):
    return int(load_library().ea_n_keep(int(n), float(ratio)))


def workspace_bytes(p, n, window):
    return int(load_library().ea_workspace_bytes(ctypes.byref(p), int(n), int(window)))


def query_stats(p, q_win, window, q_pos0, inv_freq, t_next, mu, sigma, ws, stream=None):
    _check(load_library().ea_query_stats(ctypes.byref(p), _ptr(q_win), int(window), int(q_pos0),
                                         _ptr(inv_freq), int(t_next), _ptr(mu), _ptr(sigma),
                                         _ptr(ws), _nbytes(ws), _stream(stream)), "ea_query_stats")


def query_stats_hidden(p, hidden, w_q, d_model, window, inv_freq, t_next, mu, sigma, ws, stream=None):
    _check(load_library().ea_query_stats_hidden(ctypes.byref(p), _ptr(hidden), _ptr(w_q), int(d_model),
                                                int(window), _ptr(inv_freq), int(t_next), _ptr(mu),
                                                _ptr(sigma), _ptr(ws), _nbytes(ws), _stream(stream)),
           "ea_query_stats_hidden")


def wo_gram(p, w_o, d_model, gram, stream=None):
    _check(load_library().ea_wo_gram(ctypes.byref(p), _ptr(w_o), int(d_model), _ptr(gram), _stream(stream)),
           "ea_wo_gram")


def value_norms_wo(p, v, n, n_cap, gram, wnorm, ws, stream=None):
    _check(load_library().ea_value_norms_wo(ctypes.byref(p), _ptr(v), int(n), int(n_cap), _ptr(gram),
                                            _ptr(wnorm), _ptr(ws), _nbytes(ws), _stream(stream)),
           "ea_value_norms_wo")


def score_wo(p, k, v, n, n_cap, mu, sigma, wnorm, scores, ws, stream=None):
    _check(load_library().ea_score_wo(ctypes.byref(p), _ptr(k), _ptr(v), int(n), int(n_cap), _ptr(mu),
                                      _ptr(sigma), _ptr(wnorm), _ptr(scores), _ptr(ws), _nbytes(ws),
                                      _stream(stream)), "ea_score_wo")


def score(p, k, v, n, n_cap, mu, sigma, scores, ws, stream=None):
    _check(load_library().ea_score(ctypes.byref(p), _ptr(k), _ptr(v), int(n), int(n_cap), _ptr(mu),
                                   _ptr(sigma), _ptr(scores), _ptr(ws), _nbytes(ws),
                                   _stream(stream)), "ea_score")


def select(p, scores, n, n_keep_, idx, ws, stream=None):
    _check(load_library().ea_select(ctypes.byref(p), _ptr(scores), int(n), int(n_keep_), _ptr(idx),
                                    _ptr(ws), _nbytes(ws), _stream(stream)), "ea_select")


def select_static(p, scores, n, n_keep_, idx, stream=None):
    _check(load_library().ea_select_static(ctypes.byref(p), _ptr(scores), int(n), int(n_keep_),
                                           _ptr(idx), _stream(stream)), "ea_select_static")


def compact(p, k, v, n, n_cap, idx, n_keep_, k_out, v_out, ws, stream=None):
    _check(load_library().ea_compact(ctypes.byref(p), _ptr(k), _ptr(v), int(n), int(n_cap),
                                     _ptr(idx), int(n_keep_), _ptr(k_out), _ptr(v_out), _ptr(ws),
                                     _nbytes(ws), _stream(stream)), "ea_compact")


def compress_layer(p, q_win, window, q_pos0, inv_freq, t_next, k, v, n, n_cap, n_keep_,
                   scores_out, idx_out, ws, stream=None):
    _check(load_library().ea_compress_layer(ctypes.byref(p), _ptr(q_win), int(window), int(q_pos0),
                                            _ptr(inv_freq), int(t_next), _ptr(k), _ptr(v), int(n),
                                            int(n_cap), int(n_keep_), _ptr(scores_out),
                                            _ptr(idx_out), _ptr(ws), _nbytes(ws), _stream(stream)),
           "ea_compress_layer")


def select_adaptive(p, scores, n, n_keep_, floor, idx, lengths, ws, stream=None):
    _check(load_library().ea_select_adaptive(ctypes.byref(p), _ptr(scores), int(n), int(n_keep_), int(floor),
                                             _ptr(idx), _ptr(lengths), _ptr(ws), _nbytes(ws),
                                             _stream(stream)), "ea_select_adaptive")


def compress_layer_adaptive(p, q_win, window, q_pos0, inv_freq, t_next, k, v, n, n_cap, n_keep_, floor,
                            scores_out, idx_out, lengths_out, ws, stream=None):
    _check(load_library().ea_compress_layer_adaptive(ctypes.byref(p), _ptr(q_win), int(window), int(q_pos0),
                                                     _ptr(inv_freq), int(t_next), _ptr(k), _ptr(v), int(n),
                                                     int(n_cap), int(n_keep_), int(floor), _ptr(scores_out),
                                                     _ptr(idx_out), _ptr(lengths_out), _ptr(ws), _nbytes(ws),
                                                     _stream(stream)), "ea_compress_layer_adaptive")


def compact_ragged(p, k, v, n, n_cap, idx, lengths, ws, stream=None):
    _check(load_library().ea_compact_ragged(ctypes.byref(p), _ptr(k), _ptr(v), int(n), int(n_cap), _ptr(idx),
                                            _ptr(lengths), _ptr(ws), _nbytes(ws), _stream(stream)),
           "ea_compact_ragged")


SCORER_KNORM, SCORER_STREAMING, SCORER_KEYDIFF = 0, 1, 2


def score_baseline(p, scorer, k, n, n_cap, n_sink, scores, ws, stream=None):
    _check(load_library().ea_score_baseline(ctypes.byref(p), int(scorer), _ptr(k), int(n), int(n_cap),
                                            int(n_sink), _ptr(scores), _ptr(ws), _nbytes(ws),
                                            _stream(stream)), "ea_score_baseline")


def compact_unordered(p, k, v, n, n_cap, idx, n_keep_, perm_out=None, stream=None):
    _check(load_library().ea_compact_unordered(ctypes.byref(p), _ptr(k), _ptr(v), int(n), int(n_cap),
                                               _ptr(idx), int(n_keep_), _ptr(perm_out), _stream(stream)),
           "ea_compact_unordered")


def compress_layer_unordered(p, q_win, window, q_pos0, inv_freq, t_next, k, v, n, n_cap, n_keep_,
                             scores_out, idx_out, perm_out, ws, stream=None):
    _check(load_library().ea_compress_layer_unordered(ctypes.byref(p), _ptr(q_win), int(window),
                                                      int(q_pos0), _ptr(inv_freq), int(t_next), _ptr(k),
                                                      _ptr(v), int(n), int(n_cap), int(n_keep_),
                                                      _ptr(scores_out), _ptr(idx_out), _ptr(perm_out),
                                                      _ptr(ws), _nbytes(ws), _stream(stream)),
           "ea_compress_layer_unordered")


def make_paged(block_table, block_size, num_blocks):
    """ea_paged for a block table tensor [B, max_blocks] int32 on the device."""
    return EaPaged(block_table.data_ptr(), int(block_size), int(block_table.shape[-1]), int(num_blocks))


def score_paged(p, k_pool, v_pool, pg, n, mu, sigma, scores, ws, stream=None):
    _check(load_library().ea_score_paged(ctypes.byref(p), _ptr(k_pool), _ptr(v_pool), ctypes.byref(pg), int(n),
                                         _ptr(mu), _ptr(sigma), _ptr(scores), _ptr(ws), _nbytes(ws),
                                         _stream(stream)), "ea_score_paged")


def compact_paged(p, k_pool, v_pool, pg, n, idx, n_keep_, order_free, perm_out, ws, stream=None):
    _check(load_library().ea_compact_paged(ctypes.byref(p), _ptr(k_pool), _ptr(v_pool), ctypes.byref(pg), int(n),
                                           _ptr(idx), int(n_keep_), int(order_free), _ptr(perm_out), _ptr(ws),
                                           _nbytes(ws), _stream(stream)), "ea_compact_paged")


def compress_layer_paged(p, q_win, window, q_pos0, inv_freq, t_next, k_pool, v_pool, pg, n, n_keep_, order_free,
                         scores_out, idx_out, perm_out, ws, stream=None):
    _check(load_library().ea_compress_layer_paged(ctypes.byref(p), _ptr(q_win), int(window), int(q_pos0),
                                                  _ptr(inv_freq), int(t_next), _ptr(k_pool), _ptr(v_pool),
                                                  ctypes.byref(pg), int(n), int(n_keep_), int(order_free),
                                                  _ptr(scores_out), _ptr(idx_out), _ptr(perm_out), _ptr(ws),
                                                  _nbytes(ws), _stream(stream)), "ea_compress_layer_paged")


def score_fp8(p, k8, v8, k_scale, v_scale, n, n_cap, mu, sigma, scores, ws, stream=None):
    _check(load_library().ea_score_fp8(ctypes.byref(p), _ptr(k8), _ptr(v8), _ptr(k_scale), _ptr(v_scale), int(n),
                                       int(n_cap), _ptr(mu), _ptr(sigma), _ptr(scores), _ptr(ws), _nbytes(ws),
                                       _stream(stream)), "ea_score_fp8")


def compress_layer_fp8(p, q_win, window, q_pos0, inv_freq, t_next, k8, v8, k_scale, v_scale, n, n_cap, n_keep_,
                       order_free, scores_out, idx_out, perm_out, ws, stream=None):
    _check(load_library().ea_compress_layer_fp8(ctypes.byref(p), _ptr(q_win), int(window), int(q_pos0),
                                                _ptr(inv_freq), int(t_next), _ptr(k8), _ptr(v8), _ptr(k_scale),
                                                _ptr(v_scale), int(n), int(n_cap), int(n_keep_), int(order_free),
                                                _ptr(scores_out), _ptr(idx_out), _ptr(perm_out), _ptr(ws),
                                                _nbytes(ws), _stream(stream)), "ea_compress_layer_fp8")


N_STAGES = 6
STAGE_NAMES = ("stats", "prep", "score_a", "score_b", "select", "compact")


def compress_layer_timed(p, q_win, window, q_pos0, inv_freq, t_next, k, v, n, n_cap, n_keep_, ws,
                         stream=None):
    """Profiling variant: returns the six stage times in milliseconds (host floats)."""
    ms = (ctypes.c_float * N_STAGES)()
    _check(load_library().ea_compress_layer_timed(ctypes.byref(p), _ptr(q_win), int(window),
                                                  int(q_pos0), _ptr(inv_freq), int(t_next), _ptr(k),
                                                  _ptr(v), int(n), int(n_cap), int(n_keep_), _ptr(ws),
                                                  _nbytes(ws), _stream(stream), ms),
           "ea_compress_layer_timed")
    return list(ms)


STATUS_BAD_SCORE, STATUS_COMPACT_WAIT, STATUS_BAD_INDEX = 1, 2, 4


def debug_status(p, n, window, ws, stream=None):
    """Debugging aid (blocks): the status bits the kernels left in the workspace."""
    word = ctypes.c_uint32(0)
    _check(load_library().ea_debug_status(ctypes.byref(p), int(n), int(window), _ptr(ws), _nbytes(ws),
                                          _stream(stream), ctypes.byref(word)), "ea_debug_status")
    return int(word.value)
