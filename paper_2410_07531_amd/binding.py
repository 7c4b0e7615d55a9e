"""Thin ctypes binding over librov.so: argument marshalling only.

Every function takes torch tensors (device memory) and streams as plumbing and
forwards raw pointers to the C ABI declared in include/rov.h.  There is no CPU
fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librov.so")

OK, ERR_INVALID, ERR_UNSUPPORTED, ERR_HIP, ERR_WORKSPACE = 0, -1, -2, -3, -4
F32, BF16, FP8_E4M3 = 0, 1, 2
SCHED_SEQUENTIAL, SCHED_FUSED, SCHED_OVERLAP, SCHED_HYBRID, SCHED_OVERLAP_DEFERRED = 0, 1, 2, 3, 4
MASK_NOT_READY, MASK_READY, MASK_IN_FLIGHT = 0, 1, 2

_ERR_NAMES = {ERR_INVALID: "ROV_ERR_INVALID", ERR_UNSUPPORTED: "ROV_ERR_UNSUPPORTED",
              ERR_HIP: "ROV_ERR_HIP", ERR_WORKSPACE: "ROV_ERR_WORKSPACE"}


class RovError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (what, _ERR_NAMES.get(code, "?"), code))


class GemmDesc(ctypes.Structure):
    _fields_ = [("A", ctypes.c_void_p), ("Bm", ctypes.c_void_p), ("C", ctypes.c_void_p),
                ("M", ctypes.c_int), ("N", ctypes.c_int), ("K", ctypes.c_int),
                ("dtype", ctypes.c_int), ("transB", ctypes.c_int),
                ("scaleA", ctypes.c_float), ("scaleB", ctypes.c_float)]


class AttnDesc(ctypes.Structure):
    _fields_ = [("Q", ctypes.c_void_p), ("K", ctypes.c_void_p), ("V", ctypes.c_void_p),
                ("O", ctypes.c_void_p),
                ("B", ctypes.c_int), ("H", ctypes.c_int), ("Hkv", ctypes.c_int),
                ("S", ctypes.c_int), ("d", ctypes.c_int),
                ("strides", ctypes.c_int64 * 12),
                ("dtype", ctypes.c_int), ("causal", ctypes.c_int), ("p", ctypes.c_float)]


class BlockCfg(ctypes.Structure):
    _fields_ = [("H", ctypes.c_int), ("Hkv", ctypes.c_int), ("d", ctypes.c_int),
                ("hidden", ctypes.c_int), ("ffn", ctypes.c_int), ("dtype", ctypes.c_int),
                ("causal", ctypes.c_int), ("p", ctypes.c_float), ("eps", ctypes.c_float),
                ("rope_theta", ctypes.c_float), ("act_scale", ctypes.c_float * 4)]


class BlockWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("norm1", "norm2", "wqkv", "wo", "wg", "wu", "wd")] + \
               [("w_scale", ctypes.c_float * 5)]


# name -> (restype, argtypes); also the list of symbols the header declares
_u64, _i, _f, _p = ctypes.c_uint64, ctypes.c_int, ctypes.c_float, ctypes.c_void_p
SIGNATURES = {
    "rov_last_hip_error": (_i, []),
    "rov_version": (ctypes.c_char_p, []),
    "rov_mask_words": (_u64, [_i, _i, _i]),
    "rov_mask_philox_calls": (_u64, [_i, _i, _i]),
    "rov_philox_raw": (_i, [_u64, _u64, _u64, _i, _p, _p]),
    "rov_dropout_mask_generate": (_i, [_u64, _u64, _i, _i, _i, _f, _p, _p]),
    "rov_dropout_mask_generate_rounds": (_i, [_u64, _u64, _i, _i, _i, _f, _i, _p, _p]),
    "rov_dropout_mask_generate_causal": (_i, [_u64, _u64, _i, _i, _i, _f, _p, _p]),
    "rov_dropout_mask_generate_bits": (_i, [_u64, _u64, _i, _i, _i, _f, _i, _p, _p]),
    "rov_mask_philox_calls_bits": (_u64, [_i, _i, _i, _i]),
    "rov_mask_words_rows": (_u64, [_i, _i, _i, _i, _i]),
    "rov_dropout_mask_generate_rows": (_i, [_u64, _u64, _i, _i, _i, _f, _i, _i, _p, _p]),
    "rov_attention_fwd_dropout_rows": (_i, [_p, _p, _p, _p, _i, _i, _i, _i, _i,
                                            ctypes.POINTER(ctypes.c_int64), _i, _i, _f, _p, _u64, _u64,
                                            _i, _i, _p]),
    "rov_layer_step_chunked": (_i, [ctypes.POINTER(GemmDesc), _i, ctypes.POINTER(AttnDesc), _u64, _u64, _i,
                                    _p, _p, _p]),
    "rov_set_rng_max_workgroups": (_i, [_i]),
    "rov_set_gemm_tile_cols": (_i, [_i]),
    "rov_gemm_tile_cols": (_i, [_i, _i]),
    "rov_set_rng_overlap_workgroups_per_cu": (_i, [_i]),
    "rov_trace_enable": (_i, [_i]),
    "rov_trace_read": (_i, [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float), _i,
                            ctypes.POINTER(ctypes.c_int)]),
    "rov_valu_probe": (_i, [_i, _i, _i, _p, _p]),
    "rov_gemm": (_i, [_p, _p, _p, _i, _i, _i, _i, _i, _f, _f, _p]),
    "rov_gemm_swiglu": (_i, [_p, _p, _p, _p, _i, _i, _i, _p]),
    "rov_gemm_swiglu_fp8": (_i, [_p, _p, _p, _p, _i, _i, _i, _f, _f, _f, _f, _p]),
    "rov_gemm_rng_fused": (_i, [_p, _p, _p, _i, _i, _i, _u64, _u64, _i, _i, _i, _f, _p, _p]),
    "rov_attention_fwd_dropout": (_i, [_p, _p, _p, _p, _i, _i, _i, _i, _i,
                                       ctypes.POINTER(ctypes.c_int64), _i, _i, _f, _p, _u64, _u64, _p]),
    "rov_layer_step": (_i, [_i, ctypes.POINTER(GemmDesc), _i, ctypes.POINTER(AttnDesc), _u64, _u64,
                            _p, _p, _p]),
    "rov_layer_step_rounds": (_i, [_i, ctypes.POINTER(GemmDesc), _i, ctypes.POINTER(AttnDesc), _u64, _u64,
                                   _i, _p, _p, _p]),
    "rov_layer_step_bits": (_i, [_i, ctypes.POINTER(GemmDesc), _i, ctypes.POINTER(AttnDesc), _u64, _u64,
                                 _i, _p, _p, _p]),
    "rov_attention_fwd_dropout_bits": (_i, [_p, _p, _p, _p, _i, _i, _i, _i, _i,
                                            ctypes.POINTER(ctypes.c_int64), _i, _i, _f, _p, _u64, _u64, _i, _p]),
    "rov_attention_fwd_dropout_rounds": (_i, [_p, _p, _p, _p, _i, _i, _i, _i, _i,
                                              ctypes.POINTER(ctypes.c_int64), _i, _i, _f, _p, _u64, _u64, _i,
                                              _p]),
    "rov_block_workspace_bytes": (ctypes.c_size_t, [ctypes.POINTER(BlockCfg), _i, _i, _i]),
    "rov_block_hybrid_mask_rows": (_i, [ctypes.POINTER(BlockCfg), _i, _i]),
    "rov_set_block_hybrid_mask_rows": (_i, [_i]),
    "rov_block_forward": (_i, [ctypes.POINTER(BlockWeights), _p, _p, _i, _i, ctypes.POINTER(BlockCfg),
                               _i, _u64, _u64, _i, _p, _p, _p, ctypes.c_size_t, _p, _p]),
    "rov_mask_finish": (_i, [_p, _p]),
    "rov_block_static_scratch_bytes": (ctypes.c_size_t, []),
    "rov_block_forward_static": (_i, [ctypes.POINTER(BlockWeights), _p, _p, _i, _i, ctypes.POINTER(BlockCfg),
                                      _i, _u64, _u64, _i, _p, _p, _p, _p]),
}

_lib = None


def load():
    """Load librov.so (after torch, so that both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("librov.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    try:
        import torch  # noqa: F401  (loads libamdhip64 first)
    except ImportError:
        pass
    L = ctypes.CDLL(LIB_PATH)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def _check(code, what):
    if code != OK:
        raise RovError(code, what)


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype in (torch.float8_e4m3fn, torch.uint8):
        return FP8_E4M3
    raise TypeError("unsupported dtype %s" % t.dtype)


def mask_words(B, H, S):
    return int(load().rov_mask_words(B, H, S))


def mask_philox_calls(B, H, S):
    return int(load().rov_mask_philox_calls(B, H, S))


def mask_philox_calls_bits(B, H, S, bits):
    return int(load().rov_mask_philox_calls_bits(B, H, S, int(bits)))


def set_rng_max_workgroups(n):
    return int(load().rov_set_rng_max_workgroups(int(n)))


def set_gemm_tile_cols(cols):
    r = int(load().rov_set_gemm_tile_cols(int(cols)))
    if r < 0:
        raise RovError(r, "rov_set_gemm_tile_cols")
    return r


def gemm_tile_cols(M, N):
    return int(load().rov_gemm_tile_cols(int(M), int(N)))


def set_rng_overlap_workgroups_per_cu(n):
    return int(load().rov_set_rng_overlap_workgroups_per_cu(int(n)))


def philox_raw(seed, first_counter, ncalls, rounds=10, out=None, stream=None):
    """int32-viewed uint32 [ncalls, 4] tensor of raw Philox words (test hook)."""
    import torch
    if out is None:
        out = torch.empty((int(ncalls), 4), dtype=torch.int32, device="cuda")
    _check(load().rov_philox_raw(seed & (2**64 - 1), first_counter & (2**64 - 1), int(ncalls), int(rounds),
                                 ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream)), "rov_philox_raw")
    return out


def mask_shape(B, H, S):
    """Shape of the keep-mask word array: [B, H, T, T, 16] with T = ceil(S/32)."""
    T = (S + 31) // 32
    return (B, H, T, T, 16)


def dropout_mask_generate_causal(seed, offset, B, H, S, p, out, stream=None):
    """Writes only the tiles causal attention reads (plus their chunk neighbours) into `out`."""
    _check(load().rov_dropout_mask_generate_causal(seed & (2**64 - 1), offset & (2**64 - 1), B, H, S, p,
                                                   ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream)),
           "rov_dropout_mask_generate_causal")
    return out


def dropout_mask_generate(seed, offset, B, H, S, p, out=None, rounds=None, stream=None):
    """Keep-mask words as an int64 tensor of shape mask_shape(B, H, S) (bit patterns of uint64)."""
    import torch
    if out is None:
        out = torch.empty(mask_shape(B, H, S), dtype=torch.int64, device="cuda")
    L = load()
    if rounds is None:
        rc = L.rov_dropout_mask_generate(seed & (2**64 - 1), offset & (2**64 - 1), B, H, S, p,
                                         ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream))
    else:
        rc = L.rov_dropout_mask_generate_rounds(seed & (2**64 - 1), offset & (2**64 - 1), B, H, S, p, int(rounds),
                                                ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream))
    _check(rc, "rov_dropout_mask_generate")
    return out


def dropout_mask_generate_bits(seed, offset, B, H, S, p, bits, out=None, stream=None):
    """Keep-mask drawn with `bits` (8, 16 or 32) random bits per element; same shape and layout."""
    import torch
    if out is None:
        out = torch.empty(mask_shape(B, H, S), dtype=torch.int64, device="cuda")
    _check(load().rov_dropout_mask_generate_bits(seed & (2**64 - 1), offset & (2**64 - 1), B, H, S, p, int(bits),
                                                 ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream)),
           "rov_dropout_mask_generate_bits")
    return out


def gemm(A, Bm, C=None, transB=True, scaleA=1.0, scaleB=1.0, stream=None):
    """C = scaleA*scaleB * A @ (Bm^T if transB else Bm)."""
    import torch
    M, K = A.shape
    N = Bm.shape[0] if transB else Bm.shape[1]
    code = _dtype_code(A)
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32 if code == F32 else torch.bfloat16, device=A.device)
    _check(load().rov_gemm(ctypes.c_void_p(A.data_ptr()), ctypes.c_void_p(Bm.data_ptr()),
                           ctypes.c_void_p(C.data_ptr()), M, N, K, code, int(bool(transB)),
                           float(scaleA), float(scaleB), _stream_ptr(stream)), "rov_gemm")
    return C


def gemm_swiglu(A, Wg, Wu, C=None, stream=None):
    """C = silu(A @ Wg^T) * (A @ Wu^T), bf16."""
    import torch
    M, K = A.shape
    N = Wg.shape[0]
    if C is None:
        C = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    _check(load().rov_gemm_swiglu(ctypes.c_void_p(A.data_ptr()), ctypes.c_void_p(Wg.data_ptr()),
                                  ctypes.c_void_p(Wu.data_ptr()), ctypes.c_void_p(C.data_ptr()), M, N, K,
                                  _stream_ptr(stream)), "rov_gemm_swiglu")
    return C


def gemm_swiglu_fp8(A, Wg, Wu, scaleA, scaleWg, scaleWu, scaleC, C=None, stream=None):
    """C (e4m3 bytes) = e4m3(silu(sA sWg A Wg^T) * (sA sWu A Wu^T) / scaleC); A, Wg, Wu e4m3 bytes."""
    import torch
    M, K = A.shape
    N = Wg.shape[0]
    if C is None:
        C = torch.empty((M, N), dtype=torch.uint8, device=A.device)
    _check(load().rov_gemm_swiglu_fp8(ctypes.c_void_p(A.data_ptr()), ctypes.c_void_p(Wg.data_ptr()),
                                      ctypes.c_void_p(Wu.data_ptr()), ctypes.c_void_p(C.data_ptr()), M, N, K,
                                      float(scaleA), float(scaleWg), float(scaleWu), float(scaleC),
                                      _stream_ptr(stream)), "rov_gemm_swiglu_fp8")
    return C


def gemm_rng_fused(A, Bm, seed, offset, B, H, S, p, C=None, mask=None, stream=None):
    """C = A @ Bm^T (bf16) and the keep-mask of (seed, offset, B, H, S, p) from one wave-specialised kernel."""
    import torch
    M, K = A.shape
    N = Bm.shape[0]
    if C is None:
        C = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    if mask is None:
        mask = torch.empty(mask_shape(B, H, S), dtype=torch.int64, device=A.device)
    _check(load().rov_gemm_rng_fused(ctypes.c_void_p(A.data_ptr()), ctypes.c_void_p(Bm.data_ptr()),
                                     ctypes.c_void_p(C.data_ptr()), M, N, K, ctypes.c_uint64(seed),
                                     ctypes.c_uint64(offset), B, H, S, float(p), ctypes.c_void_p(mask.data_ptr()),
                                     _stream_ptr(stream)), "rov_gemm_rng_fused")
    return C, mask


def _strides12(Q, K, V, O):
    arr = (ctypes.c_int64 * 12)()
    for x, t in enumerate((Q, K, V, O)):
        assert t.stride(3) == 1, "head dimension must be contiguous"
        arr[3 * x + 0], arr[3 * x + 1], arr[3 * x + 2] = t.stride(0), t.stride(1), t.stride(2)
    return arr


def attention_fwd_dropout(Q, K, V, p, mask=None, seed=0, offset=0, causal=False, O=None, stream=None,
                          rounds=None, bits=None):
    """Q [B,S,H,d], K/V [B,S,Hkv,d] -> O [B,S,H,d]; mask=None with p>0 selects the fused variant
    (rounds: its Philox round count, 3/5/7/10, or bits: its random bits per element, 8/16/32;
    None = the 10-round, 32-bit entry point)."""
    import torch
    B, S, H, d = Q.shape
    Hkv = K.shape[2]
    if O is None:
        O = torch.empty_like(Q)
    strides = _strides12(Q, K, V, O)
    mptr = ctypes.c_void_p(mask.data_ptr()) if mask is not None else ctypes.c_void_p(0)
    if bits is not None:
        _check(load().rov_attention_fwd_dropout_bits(
            ctypes.c_void_p(Q.data_ptr()), ctypes.c_void_p(K.data_ptr()), ctypes.c_void_p(V.data_ptr()),
            ctypes.c_void_p(O.data_ptr()), B, H, Hkv, S, d, strides, _dtype_code(Q), int(bool(causal)),
            float(p), mptr, seed & (2**64 - 1), offset & (2**64 - 1), int(bits), _stream_ptr(stream)),
            "rov_attention_fwd_dropout_bits")
        return O
    if rounds is not None:
        _check(load().rov_attention_fwd_dropout_rounds(
            ctypes.c_void_p(Q.data_ptr()), ctypes.c_void_p(K.data_ptr()), ctypes.c_void_p(V.data_ptr()),
            ctypes.c_void_p(O.data_ptr()), B, H, Hkv, S, d, strides, _dtype_code(Q), int(bool(causal)),
            float(p), mptr, seed & (2**64 - 1), offset & (2**64 - 1), int(rounds), _stream_ptr(stream)),
            "rov_attention_fwd_dropout_rounds")
        return O
    _check(load().rov_attention_fwd_dropout(
        ctypes.c_void_p(Q.data_ptr()), ctypes.c_void_p(K.data_ptr()), ctypes.c_void_p(V.data_ptr()),
        ctypes.c_void_p(O.data_ptr()), B, H, Hkv, S, d, strides, _dtype_code(Q), int(bool(causal)), float(p),
        mptr, seed & (2**64 - 1), offset & (2**64 - 1), _stream_ptr(stream)), "rov_attention_fwd_dropout")
    return O


def mask_words_rows(B, H, S, q_begin, q_rows):
    return int(load().rov_mask_words_rows(B, H, S, int(q_begin), int(q_rows)))


def dropout_mask_generate_rows(seed, offset, B, H, S, p, q_begin, q_rows, out=None, stream=None):
    """Tile rows of query rows [q_begin, q_begin + q_rows): int64 tensor [B, H, nqt, T, 16]."""
    import torch
    if out is None:
        T = (S + 31) // 32
        nqt = (min(q_begin + q_rows, S) - q_begin + 31) // 32
        out = torch.empty((B, H, nqt, T, 16), dtype=torch.int64, device="cuda")
    _check(load().rov_dropout_mask_generate_rows(seed & (2**64 - 1), offset & (2**64 - 1), B, H, S, p,
                                                 int(q_begin), int(q_rows), ctypes.c_void_p(out.data_ptr()),
                                                 _stream_ptr(stream)), "rov_dropout_mask_generate_rows")
    return out


def attention_fwd_dropout_rows(Q, K, V, p, q_begin, q_rows, O, mask_rows=None, seed=0, offset=0, causal=False,
                               stream=None):
    """Computes query rows [q_begin, q_begin + q_rows) of O in place; mask_rows holds those tile rows."""
    B, S, H, d = Q.shape
    Hkv = K.shape[2]
    strides = _strides12(Q, K, V, O)
    mptr = ctypes.c_void_p(mask_rows.data_ptr()) if mask_rows is not None else ctypes.c_void_p(0)
    _check(load().rov_attention_fwd_dropout_rows(
        ctypes.c_void_p(Q.data_ptr()), ctypes.c_void_p(K.data_ptr()), ctypes.c_void_p(V.data_ptr()),
        ctypes.c_void_p(O.data_ptr()), B, H, Hkv, S, d, strides, _dtype_code(Q), int(bool(causal)), float(p),
        mptr, seed & (2**64 - 1), offset & (2**64 - 1), int(q_begin), int(q_rows), _stream_ptr(stream)),
        "rov_attention_fwd_dropout_rows")
    return O


def layer_step_chunked(gemm_descs, attn_desc, seed, offset, q_chunk_rows, mask_ring, main_stream, side_stream):
    arr = (GemmDesc * len(gemm_descs))(*gemm_descs)
    _check(load().rov_layer_step_chunked(arr, len(gemm_descs), ctypes.byref(attn_desc), seed & (2**64 - 1),
                                         offset & (2**64 - 1), int(q_chunk_rows),
                                         ctypes.c_void_p(mask_ring.data_ptr()), _stream_ptr(main_stream),
                                         _stream_ptr(side_stream)), "rov_layer_step_chunked")


def make_gemm_desc(A, Bm, C, transB=True, scaleA=1.0, scaleB=1.0):
    M, K = A.shape
    N = Bm.shape[0] if transB else Bm.shape[1]
    return GemmDesc(A.data_ptr(), Bm.data_ptr(), C.data_ptr(), M, N, K, _dtype_code(A), int(bool(transB)),
                    float(scaleA), float(scaleB))


def gemm_desc(desc, stream=None):
    """Runs the GEMM a GemmDesc describes."""
    _check(load().rov_gemm(desc.A, desc.Bm, desc.C, desc.M, desc.N, desc.K, desc.dtype, desc.transB,
                           desc.scaleA, desc.scaleB, _stream_ptr(stream)), "rov_gemm")


def make_attn_desc(Q, K, V, O, p, causal=False):
    B, S, H, d = Q.shape
    desc = AttnDesc(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, K.shape[2], S, d,
                    _strides12(Q, K, V, O), _dtype_code(Q), int(bool(causal)), float(p))
    return desc


def layer_step(schedule, gemm_descs, attn_desc, seed, offset, mask, main_stream, side_stream, rounds=None,
               bits=None):
    arr = (GemmDesc * len(gemm_descs))(*gemm_descs)
    mptr = ctypes.c_void_p(mask.data_ptr()) if mask is not None else ctypes.c_void_p(0)
    if bits is not None:
        _check(load().rov_layer_step_bits(int(schedule), arr, len(gemm_descs), ctypes.byref(attn_desc),
                                          seed & (2**64 - 1), offset & (2**64 - 1), int(bits), mptr,
                                          _stream_ptr(main_stream), _stream_ptr(side_stream)),
               "rov_layer_step_bits")
        return
    if rounds is not None:
        _check(load().rov_layer_step_rounds(int(schedule), arr, len(gemm_descs), ctypes.byref(attn_desc),
                                            seed & (2**64 - 1), offset & (2**64 - 1), int(rounds), mptr,
                                            _stream_ptr(main_stream), _stream_ptr(side_stream)),
               "rov_layer_step_rounds")
        return
    _check(load().rov_layer_step(int(schedule), arr, len(gemm_descs), ctypes.byref(attn_desc),
                                 seed & (2**64 - 1), offset & (2**64 - 1), mptr,
                                 _stream_ptr(main_stream), _stream_ptr(side_stream)), "rov_layer_step")


def block_workspace_bytes(cfg, B, S, schedule):
    return int(load().rov_block_workspace_bytes(ctypes.byref(cfg), B, S, int(schedule)))


def block_hybrid_mask_rows(cfg, B, S):
    return int(load().rov_block_hybrid_mask_rows(ctypes.byref(cfg), B, S))


def set_block_hybrid_mask_rows(rows):
    return int(load().rov_set_block_hybrid_mask_rows(int(rows)))


def make_block_cfg(H, Hkv, d, hidden, ffn, p, causal=False, eps=1e-5, rope_theta=500000.0, dtype=BF16,
                   act_scale=None):
    """act_scale (fp8 only): dequantisation scales of the four quantised activations h1, a, h2, u."""
    sc = (ctypes.c_float * 4)(*([float(v) for v in act_scale] if act_scale is not None else [0.0] * 4))
    return BlockCfg(H, Hkv, d, hidden, ffn, dtype, int(bool(causal)), float(p), float(eps), float(rope_theta), sc)


def make_block_weights(w, w_scale=None):
    """w: dict of device tensors norm1, norm2, wqkv, wo, wg, wu, wd; w_scale (fp8 only): dict of the five
    weight matrices' dequantisation scales."""
    names = ("wqkv", "wo", "wg", "wu", "wd")
    sc = (ctypes.c_float * 5)(*([float(w_scale[n]) for n in names] if w_scale is not None else [0.0] * 5))
    return BlockWeights(*[w[n].data_ptr() for n in ("norm1", "norm2") + names], sc)


def block_forward(weights, x, y, cfg, schedule, seed, offset, mask, workspace, main_stream, side_stream,
                  mask_ready=False, next_mask=None):
    B, S, _ = x.shape
    mptr = ctypes.c_void_p(mask.data_ptr()) if mask is not None else ctypes.c_void_p(0)
    nptr = ctypes.c_void_p(next_mask.data_ptr()) if next_mask is not None else ctypes.c_void_p(0)
    _check(load().rov_block_forward(ctypes.byref(weights), ctypes.c_void_p(x.data_ptr()),
                                    ctypes.c_void_p(y.data_ptr()), B, S, ctypes.byref(cfg), int(schedule),
                                    seed & (2**64 - 1), offset & (2**64 - 1), int(mask_ready), mptr, nptr,
                                    ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                    _stream_ptr(main_stream), _stream_ptr(side_stream)), "rov_block_forward")
    return y


def mask_finish(mask, main_stream):
    """Completes and joins a mask that an OVERLAP_DEFERRED block_forward left in flight."""
    _check(load().rov_mask_finish(ctypes.c_void_p(mask.data_ptr()), _stream_ptr(main_stream)), "rov_mask_finish")


def block_static_scratch_bytes():
    return int(load().rov_block_static_scratch_bytes())


def block_forward_static(weights, x, y, cfg, schedule, seed, offset, mask, main_stream, side_stream,
                         mask_ready=False, next_mask=None):
    """block_forward on the library's own static scratch (no workspace, nothing allocated)."""
    B, S, _ = x.shape
    mptr = ctypes.c_void_p(mask.data_ptr()) if mask is not None else ctypes.c_void_p(0)
    nptr = ctypes.c_void_p(next_mask.data_ptr()) if next_mask is not None else ctypes.c_void_p(0)
    _check(load().rov_block_forward_static(ctypes.byref(weights), ctypes.c_void_p(x.data_ptr()),
                                           ctypes.c_void_p(y.data_ptr()), B, S, ctypes.byref(cfg), int(schedule),
                                           seed & (2**64 - 1), offset & (2**64 - 1), int(mask_ready), mptr,
                                           nptr, _stream_ptr(main_stream), _stream_ptr(side_stream)),
           "rov_block_forward_static")
    return y


TRACE_GEMM, TRACE_RNG, TRACE_ATTENTION, TRACE_GLUE, TRACE_RNG_HELPER = 0, 1, 2, 3, 4


def trace_enable(on, kinds=None):
    """on=False: off.  on=True: every kind, or only the kinds listed (e.g. [TRACE_GEMM])."""
    if not on:
        sel = 0
    elif kinds is None:
        sel = -1
    else:
        sel = 0
        for k in kinds:
            sel |= 1 << int(k)
    return int(load().rov_trace_enable(sel))


def trace_read(max_records=16384):
    """List of (kind, milliseconds) in launch order; waits for the traced kernels to finish."""
    kinds = (ctypes.c_int * max_records)()
    ms = (ctypes.c_float * max_records)()
    n = ctypes.c_int(0)
    _check(load().rov_trace_read(kinds, ms, max_records, ctypes.byref(n)), "rov_trace_read")
    return [(int(kinds[i]), float(ms[i])) for i in range(n.value)]
