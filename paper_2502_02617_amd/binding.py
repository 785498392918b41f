"""ctypes binding of libpolarquant (argument marshalling only).

Function names mirror the C ABI: ``Context`` wraps ``pq_init_preconditioner`` /
``pq_destroy`` and its methods call ``pq_encode_kv``, ``pq_append_kv``, ``pq_append_kv_pair``,
``pq_decode_kv``, ``pq_export_canonical``, ``pq_attn_decode_polar``, ``pq_attn_decode_hybrid`` and ``pq_decode_step_polar`` with
pointers of torch tensors (torch is used for device memory and streams only).
"""
import ctypes
import os

import numpy as np

from . import _build

PQ_F32, PQ_BF16 = 0, 1
PQ_KEY, PQ_VALUE = 0, 1
TILE_TOKENS = 64
TILE_CODE_BYTES = 2944
TILE_RADII = 512
RECORD_BYTES = 62
D = 128

_lib = None


class PolarQuantError(RuntimeError):
    pass


def library():
    """Loads the in-tree libpolarquant.so (building it first if it is absent)."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB_PATH
    if not os.path.exists(path):
        _build.build()
    L = ctypes.CDLL(path)
    vp, i64, i32, u64 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint64
    L.pq_status_string.restype = ctypes.c_char_p
    L.pq_status_string.argtypes = [i32]
    L.pq_init_preconditioner.restype = i32
    L.pq_init_preconditioner.argtypes = [ctypes.POINTER(vp), i32, u64, vp]
    L.pq_init_preconditioner_hadamard.restype = i32
    L.pq_init_preconditioner_hadamard.argtypes = [ctypes.POINTER(vp), i32, u64]
    L.pq_set_codebooks.restype = i32
    L.pq_set_codebooks.argtypes = [vp, vp]
    L.pq_fit_codebooks.restype = i32
    L.pq_fit_codebooks.argtypes = [vp, vp, i32, i64, i32, i64, i64, vp, i32, vp, vp, ctypes.c_size_t, vp]
    L.pq_fit_codebooks_deep.restype = i32
    L.pq_fit_codebooks_deep.argtypes = [vp, vp, i32, i64, i32, i64, i64, vp, vp, i32, vp, vp, vp, ctypes.c_size_t, vp]
    L.pq_fit_workspace_bytes.restype = ctypes.c_size_t
    L.pq_fit_workspace_bytes.argtypes = []
    L.pq_fit_count_angles.restype = i32
    L.pq_fit_count_angles.argtypes = [vp, vp, i32, i64, i32, i64, i64, vp, ctypes.c_size_t, vp]
    L.pq_fit_cluster.restype = i32
    L.pq_fit_cluster.argtypes = [vp, vp, vp, vp, i32, vp, vp]
    L.pq_set_recursion_depth.restype = i32
    L.pq_set_recursion_depth.argtypes = [vp, i32, vp]
    L.pq_set_upper_codebooks.restype = i32
    L.pq_set_upper_codebooks.argtypes = [vp, vp]
    L.pq_recursion_depth.restype = i32
    L.pq_recursion_depth.argtypes = [vp]
    L.pq_preconditioner_structure.restype = i32
    L.pq_preconditioner_structure.argtypes = [vp]
    L.pq_radii_halves_per_tile.restype = i32
    L.pq_radii_halves_per_tile.argtypes = [vp]
    L.pq_record_bytes.restype = i32
    L.pq_record_bytes.argtypes = [vp]
    L.pq_get_upper_codebook.restype = i32
    L.pq_get_upper_codebook.argtypes = [vp, i32, vp, vp, vp]
    L.pq_get_preconditioner.restype = i32
    L.pq_get_preconditioner.argtypes = [vp, vp]
    L.pq_get_codebook.restype = i32
    L.pq_get_codebook.argtypes = [vp, i32, vp, vp]
    L.pq_destroy.restype = None
    L.pq_destroy.argtypes = [vp]
    L.pq_encode_kv.restype = i32
    L.pq_encode_kv.argtypes = [vp, vp, i32, i32, i64, i32, i64, i64, vp, vp, i64, i64, vp]
    L.pq_encode_kv_pair.restype = i32
    L.pq_encode_kv_pair.argtypes = [vp, vp, vp, i32, i64, i32, i64, i64, vp, vp, vp, vp, i64, i64, vp]
    L.pq_append_kv.restype = i32
    L.pq_append_kv.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, i64, vp, vp]
    L.pq_append_kv_pair.restype = i32
    L.pq_append_kv_pair.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, i64, vp, vp]
    L.pq_decode_kv.restype = i32
    L.pq_decode_kv.argtypes = [vp, i32, vp, vp, i64, i64, i64, i32, vp, i32, i64, i64, i32, vp]
    L.pq_export_canonical.restype = i32
    L.pq_export_canonical.argtypes = [vp, i32, vp, vp, i64, i64, i64, i32, vp, vp]
    L.pq_attn_decode_polar.restype = i32
    L.pq_attn_decode_polar.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, i64, i64,
                                       ctypes.c_float, vp, ctypes.c_size_t, vp]
    L.pq_decode_step_polar.restype = i32
    L.pq_decode_step_polar.argtypes = [vp, vp, vp, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, i64, i64,
                                       ctypes.c_float, vp, ctypes.c_size_t, vp]
    L.pq_attn_decode_hybrid.restype = i32
    L.pq_attn_decode_hybrid.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i64, i64,
                                        ctypes.c_float, vp, ctypes.c_size_t, vp]
    L.pq_attn_hybrid_workspace_bytes.restype = ctypes.c_size_t
    L.pq_attn_hybrid_workspace_bytes.argtypes = [i32, i32, i32, i64, i64]
    L.pq_attn_decode_polar_mq.restype = i32
    L.pq_attn_decode_polar_mq.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i64, i64,
                                          ctypes.c_float, vp, ctypes.c_size_t, vp]
    L.pq_attn_mq_workspace_bytes.restype = ctypes.c_size_t
    L.pq_attn_mq_workspace_bytes.argtypes = [i32, i32, i32, i32, i64]
    L.pq_attn_workspace_bytes.restype = ctypes.c_size_t
    L.pq_attn_workspace_bytes.argtypes = [i32, i32, i32, i64]
    L.pq_static_scratch_bytes.restype = ctypes.c_size_t
    L.pq_static_scratch_bytes.argtypes = []
    L.pq_prepare_device.restype = i32
    L.pq_prepare_device.argtypes = [vp]
    L.pq_attn_decode_polar_static.restype = i32
    L.pq_attn_decode_polar_static.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, i64, i64,
                                              ctypes.c_float, vp]
    L.pq_general_record_bytes.restype = ctypes.c_size_t
    L.pq_general_record_bytes.argtypes = [vp]
    L.pq_general_codebook_entries.restype = i32
    L.pq_general_codebook_entries.argtypes = [vp]
    L.pq_general_codebooks.restype = i32
    L.pq_general_codebooks.argtypes = [vp, vp]
    L.pq_general_encode.restype = i32
    L.pq_general_encode.argtypes = [vp, vp, vp, vp, i32, i64, i64, vp, vp]
    L.pq_general_decode.restype = i32
    L.pq_general_decode.argtypes = [vp, vp, vp, vp, i64, i32, vp, vp]
    L.pq_general_attn_decode.restype = i32
    L.pq_general_attn_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i64, ctypes.c_float, vp]
    L.pq_profile_begin.restype = i32
    L.pq_profile_begin.argtypes = [i32]
    L.pq_profile_begin_sampled.restype = i32
    L.pq_profile_begin_sampled.argtypes = [i32, i32]
    L.pq_profile_end.restype = i32
    L.pq_profile_end.argtypes = [vp, vp, vp, vp]
    L.pq_kernel_name_attn.restype = ctypes.c_char_p
    L.pq_kernel_name_encode.restype = ctypes.c_char_p
    _lib = L
    return L


def pq_status_string(code):
    return library().pq_status_string(int(code)).decode()


def profile_begin(max_launches, every=1):
    """Time at most max_launches launches of each of the two dominant kernels, every `every`-th one."""
    _check(library().pq_profile_begin_sampled(int(max_launches), int(every)))


def profile_end():
    """-> dict(attn_ms, attn_launches, encode_ms, encode_launches) of the launches timed since profile_begin."""
    a, e = ctypes.c_double(), ctypes.c_double()
    na, ne = ctypes.c_int(), ctypes.c_int()
    _check(library().pq_profile_end(ctypes.byref(a), ctypes.byref(na), ctypes.byref(e), ctypes.byref(ne)))
    return {"attn_ms": a.value, "attn_launches": na.value, "encode_ms": e.value, "encode_launches": ne.value}


def _check(code):
    if code != 0:
        raise PolarQuantError(pq_status_string(code))


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    import torch

    if t.dtype == torch.bfloat16:
        return PQ_BF16
    if t.dtype == torch.float32:
        return PQ_F32
    raise PolarQuantError("only float32 and bfloat16 tensors are supported")


class Context:
    """pq_ctx: the preconditioner S, the codebooks and the device constant tables."""

    def __init__(self, seed=0, S=None, d=D, hadamard=False):
        """S: explicit d x d orthogonal matrix; hadamard=True: randomised Hadamard matrix from seed
        (pq_init_preconditioner_hadamard); otherwise the QR factor of a seeded Gaussian matrix."""
        L = library()
        h = ctypes.c_void_p()
        if hadamard:
            if S is not None:
                raise PolarQuantError("give either S or hadamard=True")
            _check(L.pq_init_preconditioner_hadamard(ctypes.byref(h), int(d), int(seed)))
            self._h = h
            self.d = d
            return
        if S is not None:
            S = np.ascontiguousarray(S, dtype=np.float64)
            if S.shape != (d, d):
                raise PolarQuantError("S must be d x d")
            sp = S.ctypes.data_as(ctypes.c_void_p)
        else:
            sp = None
        _check(L.pq_init_preconditioner(ctypes.byref(h), int(d), int(seed), sp))
        self._h = h
        self.d = d

    def close(self):
        if getattr(self, "_h", None):
            library().pq_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_codebooks(self, cb):
        """cb: 28 centroids (16 of level 1, then 4 each of levels 2-4); only before the first launch."""
        cb = np.ascontiguousarray(cb, dtype=np.float64).reshape(-1)
        if cb.size != 28:
            raise PolarQuantError("cb must hold 28 centroids")
        _check(library().pq_set_codebooks(self._h, cb.ctypes.data_as(ctypes.c_void_p)))

    def set_recursion_depth(self, depth, upper_bits=None):
        """depth 4 (default) or 7 (full recursion: upper_bits = bits of levels 5, 6, 7); only before the first launch."""
        bits = None
        if upper_bits is not None:
            bits = np.ascontiguousarray(upper_bits, dtype=np.int32).reshape(-1)
            if bits.size != 3:
                raise PolarQuantError("upper_bits must hold 3 widths")
        _check(library().pq_set_recursion_depth(self._h, int(depth), bits.ctypes.data_as(ctypes.c_void_p) if bits is not None else None))

    def set_upper_codebooks(self, cbt):
        """Centroids of levels 5, 6, 7 of a depth-7 context, array [3, 8] (2^bits used per row); before the first launch."""
        c = np.ascontiguousarray(cbt, dtype=np.float64)
        if c.shape != (3, 8):
            raise PolarQuantError("cbt must have shape [3, 8]")
        _check(library().pq_set_upper_codebooks(self._h, c.ctypes.data_as(ctypes.c_void_p)))

    def recursion_depth(self):
        return int(library().pq_recursion_depth(self._h))

    def preconditioner_structure(self):
        """0 general S, 1 all entries +-1/sqrt(d), 2 sign diagonal times the Sylvester Hadamard matrix."""
        return int(library().pq_preconditioner_structure(self._h))

    def radii_halves_per_tile(self):
        return int(library().pq_radii_halves_per_tile(self._h))

    def record_bytes(self):
        return int(library().pq_record_bytes(self._h))

    def upper_codebook(self, level):
        """Level 5..7 of a depth-7 context: (bits, centroids, boundaries)."""
        bits = ctypes.c_int(0)
        c = np.zeros(8, dtype=np.float64)
        b = np.zeros(9, dtype=np.float64)
        _check(library().pq_get_upper_codebook(self._h, int(level), ctypes.byref(bits), c.ctypes.data_as(ctypes.c_void_p),
                                               b.ctypes.data_as(ctypes.c_void_p)))
        K = 1 << bits.value
        return bits.value, c[:K].copy(), b[: K + 1].copy()

    def alloc_cache_for(self, n_heads, pool_tokens, device="cuda"):
        """Cache buffers in this context's format (the radius plane depends on the recursion depth)."""
        return Context.alloc_cache(n_heads, pool_tokens, device, self.radii_halves_per_tile())

    def fit_codebooks(self, x, iterations, cb_init=None, workspace=None):
        """Online codebooks from x [n_tokens, n_heads, 128] (strides taken from the tensor, innermost contiguous):
        `iterations` k-means rounds on its angles -> 28 centroids (numpy).  Waits for the stream."""
        import torch

        if x.stride(2) != 1:
            raise PolarQuantError("innermost dimension must be contiguous")
        nbytes = int(library().pq_fit_workspace_bytes())
        if workspace is None:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=x.device)
        init = None
        if cb_init is not None:
            init = np.ascontiguousarray(cb_init, dtype=np.float64).reshape(-1)
            if init.size != 28:
                raise PolarQuantError("cb_init must hold 28 centroids")
        out = np.empty(28, dtype=np.float64)
        _check(library().pq_fit_codebooks(
            self._h, x.data_ptr(), _dtype_code(x), int(x.shape[0]), int(x.shape[1]), int(x.stride(0)), int(x.stride(1)),
            init.ctypes.data_as(ctypes.c_void_p) if init is not None else None, int(iterations),
            out.ctypes.data_as(ctypes.c_void_p), workspace.data_ptr(),
            int(workspace.numel() * workspace.element_size()), _stream()))
        return out

    def fit_count_angles(self, x, workspace):
        """First half of fit_codebooks: counts the angles of x into the histograms in workspace (uint8 device tensor of
        fit_workspace_bytes()); enqueued on the current stream, does not wait."""
        if x.stride(2) != 1:
            raise PolarQuantError("innermost dimension must be contiguous")
        _check(library().pq_fit_count_angles(
            self._h, x.data_ptr(), _dtype_code(x), int(x.shape[0]), int(x.shape[1]), int(x.stride(0)), int(x.stride(1)),
            workspace.data_ptr(), int(workspace.numel() * workspace.element_size()), _stream()))

    def fit_cluster(self, hist, iterations, cb_init=None, cbt_init=None):
        """Second half: hist = host copy (numpy uint32) of the workspace -> 28 centroids, and [3, 8] upper centroids for a
        depth-7 context (None otherwise)."""
        hist = np.ascontiguousarray(hist, dtype=np.uint32)
        if hist.size * 4 != self.fit_workspace_bytes():
            raise PolarQuantError("hist must be a copy of the whole fit workspace")
        init = None if cb_init is None else np.ascontiguousarray(cb_init, dtype=np.float64).reshape(-1)
        init_t = None if cbt_init is None else np.ascontiguousarray(cbt_init, dtype=np.float64)
        out, out_t = np.empty(28, dtype=np.float64), np.empty((3, 8), dtype=np.float64)
        _check(library().pq_fit_cluster(
            self._h, hist.ctypes.data_as(ctypes.c_void_p),
            init.ctypes.data_as(ctypes.c_void_p) if init is not None else None,
            init_t.ctypes.data_as(ctypes.c_void_p) if init_t is not None else None, int(iterations),
            out.ctypes.data_as(ctypes.c_void_p), out_t.ctypes.data_as(ctypes.c_void_p)))
        return out, (out_t if self.recursion_depth() == 7 else None)

    @staticmethod
    def fit_workspace_bytes():
        return int(library().pq_fit_workspace_bytes())

    def fit_codebooks_deep(self, x, iterations, cb_init=None, cbt_init=None, workspace=None):
        """fit_codebooks for a depth-7 context: also the codebooks of levels 5-7 -> (28 centroids, [3, 8] centroids)."""
        import torch

        if x.stride(2) != 1:
            raise PolarQuantError("innermost dimension must be contiguous")
        nbytes = int(library().pq_fit_workspace_bytes())
        if workspace is None:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=x.device)
        init = init_t = None
        if cb_init is not None:
            init = np.ascontiguousarray(cb_init, dtype=np.float64).reshape(-1)
            if init.size != 28:
                raise PolarQuantError("cb_init must hold 28 centroids")
        if cbt_init is not None:
            init_t = np.ascontiguousarray(cbt_init, dtype=np.float64)
            if init_t.shape != (3, 8):
                raise PolarQuantError("cbt_init must have shape [3, 8]")
        out = np.empty(28, dtype=np.float64)
        out_t = np.empty((3, 8), dtype=np.float64)
        _check(library().pq_fit_codebooks_deep(
            self._h, x.data_ptr(), _dtype_code(x), int(x.shape[0]), int(x.shape[1]), int(x.stride(0)), int(x.stride(1)),
            init.ctypes.data_as(ctypes.c_void_p) if init is not None else None,
            init_t.ctypes.data_as(ctypes.c_void_p) if init_t is not None else None, int(iterations),
            out.ctypes.data_as(ctypes.c_void_p), out_t.ctypes.data_as(ctypes.c_void_p), workspace.data_ptr(),
            int(workspace.numel() * workspace.element_size()), _stream()))
        return out, out_t

    # ---- host-side getters -------------------------------------------------
    def preconditioner(self):
        S = np.empty((self.d, self.d), dtype=np.float64)
        _check(library().pq_get_preconditioner(self._h, S.ctypes.data_as(ctypes.c_void_p)))
        return S

    def codebook(self, level):
        K = 16 if level == 1 else 4
        c = np.empty(K, dtype=np.float64)
        b = np.empty(K + 1, dtype=np.float64)
        _check(library().pq_get_codebook(self._h, int(level), c.ctypes.data_as(ctypes.c_void_p),
                                         b.ctypes.data_as(ctypes.c_void_p)))
        return c, b

    # ---- cache allocation helper (torch owns the memory) --------------------
    @staticmethod
    def alloc_cache(n_heads, pool_tokens, device="cuda", radii_halves=TILE_RADII):
        import torch

        if pool_tokens % TILE_TOKENS:
            raise PolarQuantError("pool_tokens must be a multiple of 64")
        tiles = pool_tokens // TILE_TOKENS
        codes = torch.empty((n_heads, tiles, TILE_CODE_BYTES), dtype=torch.uint8, device=device)
        radii = torch.empty((n_heads, tiles, radii_halves), dtype=torch.int16, device=device)
        return codes, radii

    # ---- kernels -------------------------------------------------------------
    def encode_kv(self, x, kind, codes, radii, dst_token0=0, ld_token=None, ld_head=None, n_tokens=None, n_heads=None):
        """x: [n_tokens, n_heads, 128] (token-major) or any strided view given ld_token / ld_head (elements)."""
        if ld_token is None:
            n_tokens, n_heads = x.shape[0], x.shape[1]
            ld_token, ld_head = x.stride(0), x.stride(1)
            if x.stride(2) != 1:
                raise PolarQuantError("innermost dimension must be contiguous")
        pool_tokens = codes.shape[1] * TILE_TOKENS
        _check(library().pq_encode_kv(self._h, x.data_ptr(), _dtype_code(x), int(kind), int(n_tokens), int(n_heads),
                                      int(ld_token), int(ld_head), codes.data_ptr(), radii.data_ptr(),
                                      int(pool_tokens), int(dst_token0), _stream()))

    def encode_kv_pair(self, xk, xv, k_codes, k_radii, v_codes, v_radii, dst_token0=0, ld_token=None, ld_head=None,
                       n_tokens=None, n_heads=None):
        """Keys and values of the same tokens in one launch; xk, xv as x of encode_kv, same shape, strides, dtype."""
        if ld_token is None:
            n_tokens, n_heads = xk.shape[0], xk.shape[1]
            ld_token, ld_head = xk.stride(0), xk.stride(1)
            if xk.stride(2) != 1 or xv.stride(2) != 1:
                raise PolarQuantError("innermost dimension must be contiguous")
            if xv.shape != xk.shape or xv.stride() != xk.stride():
                raise PolarQuantError("xk and xv must have the same shape and strides")
        if xk.dtype != xv.dtype:
            raise PolarQuantError("xk and xv must have the same dtype")
        if k_codes.shape != v_codes.shape:
            raise PolarQuantError("key and value caches must have the same pool size")
        pool_tokens = k_codes.shape[1] * TILE_TOKENS
        _check(library().pq_encode_kv_pair(self._h, xk.data_ptr(), xv.data_ptr(), _dtype_code(xk), int(n_tokens),
                                           int(n_heads), int(ld_token), int(ld_head), k_codes.data_ptr(),
                                           k_radii.data_ptr(), v_codes.data_ptr(), v_radii.data_ptr(),
                                           int(pool_tokens), int(dst_token0), _stream()))

    def append_kv(self, x, kind, codes, radii, dst_token):
        """x: [n_seq, n_heads, 128] contiguous; dst_token: int64 device tensor [n_seq]."""
        if not x.is_contiguous():
            raise PolarQuantError("x must be contiguous")
        pool_tokens = codes.shape[1] * TILE_TOKENS
        _check(library().pq_append_kv(self._h, x.data_ptr(), _dtype_code(x), int(kind), int(x.shape[0]), int(x.shape[1]),
                                      codes.data_ptr(), radii.data_ptr(), int(pool_tokens), dst_token.data_ptr(),
                                      _stream()))

    def append_kv_pair(self, xk, xv, k_codes, k_radii, v_codes, v_radii, dst_token):
        """xk, xv: [n_seq, n_heads, 128] contiguous, same dtype; dst_token: int64 device tensor [n_seq]."""
        if not (xk.is_contiguous() and xv.is_contiguous()):
            raise PolarQuantError("xk and xv must be contiguous")
        if xk.shape != xv.shape or xk.dtype != xv.dtype:
            raise PolarQuantError("xk and xv must have the same shape and dtype")
        if k_codes.shape != v_codes.shape:
            raise PolarQuantError("key and value caches must have the same pool size")
        pool_tokens = k_codes.shape[1] * TILE_TOKENS
        _check(library().pq_append_kv_pair(self._h, xk.data_ptr(), xv.data_ptr(), _dtype_code(xk), int(xk.shape[0]),
                                           int(xk.shape[1]), k_codes.data_ptr(), k_radii.data_ptr(),
                                           v_codes.data_ptr(), v_radii.data_ptr(), int(pool_tokens),
                                           dst_token.data_ptr(), _stream()))

    def decode_kv(self, kind, codes, radii, token0, n_tokens, out, rotated=False):
        """out: [n_tokens, n_heads, 128] float32 or bfloat16 (strides taken from the tensor)."""
        pool_tokens = codes.shape[1] * TILE_TOKENS
        _check(library().pq_decode_kv(self._h, int(kind), codes.data_ptr(), radii.data_ptr(), int(pool_tokens),
                                      int(token0), int(n_tokens), int(out.shape[1]), out.data_ptr(), _dtype_code(out),
                                      int(out.stride(0)), int(out.stride(1)), 1 if rotated else 0, _stream()))

    def export_canonical(self, kind, codes, radii, token0, n_tokens, rec):
        """rec: uint8 [n_heads, n_tokens, record_bytes()] contiguous (62, or 50 at depth 7)."""
        pool_tokens = codes.shape[1] * TILE_TOKENS
        _check(library().pq_export_canonical(self._h, int(kind), codes.data_ptr(), radii.data_ptr(), int(pool_tokens),
                                             int(token0), int(n_tokens), int(codes.shape[0]), rec.data_ptr(), _stream()))

    @staticmethod
    def attn_workspace_bytes(B, Hq, Hkv, max_ctx):
        return int(library().pq_attn_workspace_bytes(int(B), int(Hq), int(Hkv), int(max_ctx)))

    def attn_decode_polar_mq(self, q, out, k_codes, k_radii, v_codes, v_radii, seq_start, ctx_len, max_ctx,
                             softmax_scale, workspace):
        """M query tokens per sequence: q, out [B, M, Hq, 128]; token m sees ctx_len - (M-1-m) cached tokens."""
        B, M, Hq = q.shape[0], q.shape[1], q.shape[2]
        Hkv = k_codes.shape[0]
        if not (q.is_contiguous() and out.is_contiguous()):
            raise PolarQuantError("q and out must be contiguous")
        pool_tokens = k_codes.shape[1] * TILE_TOKENS
        _check(library().pq_attn_decode_polar_mq(
            self._h, q.data_ptr(), out.data_ptr(), _dtype_code(out), k_codes.data_ptr(), k_radii.data_ptr(),
            v_codes.data_ptr(), v_radii.data_ptr(), seq_start.data_ptr(), ctx_len.data_ptr(), int(B), int(M), int(Hq),
            int(Hkv), int(pool_tokens), int(max_ctx), float(softmax_scale), workspace.data_ptr(),
            int(workspace.numel() * workspace.element_size()), _stream()))

    @staticmethod
    def attn_mq_workspace_bytes(B, M, Hq, Hkv, max_ctx):
        return int(library().pq_attn_mq_workspace_bytes(int(B), int(M), int(Hq), int(Hkv), int(max_ctx)))

    def attn_decode_hybrid(self, q, out, k_codes, k_radii, v_codes, v_radii, seq_start, ctx_len, win_k, win_v, win_len,
                           max_ctx, softmax_scale, workspace):
        """Quantised prefix + bf16 window: win_k, win_v [B, Hkv, win_cap, 128] bf16 contiguous, win_len int32 [B]."""
        if not (win_k.is_contiguous() and win_v.is_contiguous()):
            raise PolarQuantError("win_k and win_v must be contiguous")
        B, Hq = q.shape[0], q.shape[1]
        Hkv = k_codes.shape[0]
        if win_k.shape != win_v.shape or tuple(win_k.shape[:2]) != (B, Hkv) or win_k.shape[3] != 128:
            raise PolarQuantError("win_k and win_v must both be [B, Hkv, win_cap, 128]")
        if _dtype_code(win_k) != PQ_BF16 or _dtype_code(win_v) != PQ_BF16:
            raise PolarQuantError("the window is bfloat16")
        pool_tokens = k_codes.shape[1] * TILE_TOKENS
        _check(library().pq_attn_decode_hybrid(
            self._h, q.data_ptr(), out.data_ptr(), _dtype_code(out), k_codes.data_ptr(), k_radii.data_ptr(),
            v_codes.data_ptr(), v_radii.data_ptr(), seq_start.data_ptr(), ctx_len.data_ptr(), win_k.data_ptr(),
            win_v.data_ptr(), win_len.data_ptr(), int(win_k.shape[2]), int(B), int(Hq), int(Hkv), int(pool_tokens),
            int(max_ctx), float(softmax_scale), workspace.data_ptr(),
            int(workspace.numel() * workspace.element_size()), _stream()))

    @staticmethod
    def attn_hybrid_workspace_bytes(B, Hq, Hkv, max_ctx, win_cap):
        return int(library().pq_attn_hybrid_workspace_bytes(int(B), int(Hq), int(Hkv), int(max_ctx), int(win_cap)))

    def decode_step_polar(self, xk, xv, dst_token, q, out, k_codes, k_radii, v_codes, v_radii, seq_start, ctx_len,
                          max_ctx, softmax_scale, workspace):
        """append_kv_pair(xk, xv -> dst_token) + attn_decode_polar in one call; xk, xv: [B, Hkv, 128] contiguous."""
        if not (xk.is_contiguous() and xv.is_contiguous()):
            raise PolarQuantError("xk and xv must be contiguous")
        B, Hq = q.shape[0], q.shape[1]
        Hkv = k_codes.shape[0]
        if tuple(xk.shape) != (B, Hkv, 128) or xk.shape != xv.shape or xk.dtype != xv.dtype:
            raise PolarQuantError("xk and xv must both be [B, Hkv, 128] of one dtype")
        pool_tokens = k_codes.shape[1] * TILE_TOKENS
        _check(library().pq_decode_step_polar(
            self._h, xk.data_ptr(), xv.data_ptr(), _dtype_code(xk), dst_token.data_ptr(), q.data_ptr(), out.data_ptr(),
            _dtype_code(out), k_codes.data_ptr(), k_radii.data_ptr(), v_codes.data_ptr(), v_radii.data_ptr(),
            seq_start.data_ptr(), ctx_len.data_ptr(), int(B), int(Hq), int(Hkv), int(pool_tokens), int(max_ctx),
            float(softmax_scale), workspace.data_ptr(), int(workspace.numel() * workspace.element_size()), _stream()))

    @staticmethod
    def static_scratch_bytes():
        return int(library().pq_static_scratch_bytes())

    def prepare_device(self):
        """Uploads the context's constants to the current device (the one call of the static path that allocates)."""
        _check(library().pq_prepare_device(self._h))

    def attn_decode_polar_static(self, q, out, k_codes, k_radii, v_codes, v_radii, seq_start, ctx_len, max_ctx,
                                 softmax_scale):
        """attn_decode_polar with the workspace in the library's static device array; allocates nothing."""
        B, Hq = q.shape[0], q.shape[1]
        Hkv = k_codes.shape[0]
        pool_tokens = k_codes.shape[1] * TILE_TOKENS
        _check(library().pq_attn_decode_polar_static(
            self._h, q.data_ptr(), out.data_ptr(), _dtype_code(out), k_codes.data_ptr(), k_radii.data_ptr(), v_codes.data_ptr(),
            v_radii.data_ptr(), seq_start.data_ptr(), ctx_len.data_ptr(), int(B), int(Hq), int(Hkv), int(pool_tokens),
            int(max_ctx), float(softmax_scale), _stream()))

    def attn_decode_polar(self, q, out, k_codes, k_radii, v_codes, v_radii, seq_start, ctx_len, max_ctx,
                          softmax_scale, workspace):
        """q: [B, Hq, 128] bf16; out: same shape, bf16 or float32; seq_start int64 [B], ctx_len int32 [B] (device)."""
        B, Hq = q.shape[0], q.shape[1]
        Hkv = k_codes.shape[0]
        pool_tokens = k_codes.shape[1] * TILE_TOKENS
        _check(library().pq_attn_decode_polar(
            self._h, q.data_ptr(), out.data_ptr(), _dtype_code(out), k_codes.data_ptr(), k_radii.data_ptr(), v_codes.data_ptr(),
            v_radii.data_ptr(), seq_start.data_ptr(), ctx_len.data_ptr(), int(B), int(Hq), int(Hkv), int(pool_tokens),
            int(max_ctx), float(softmax_scale), workspace.data_ptr(), int(workspace.numel() * workspace.element_size()),
            _stream()))


class GeneralFormat(ctypes.Structure):
    """pq_general_format: recursion depth 4..7 and bits per level (level 1: 3 or 4; 2-4: 2 or 3; 5-7: 1..3)."""
    _fields_ = [("depth", ctypes.c_int), ("bits", ctypes.c_int * 7)]

    def __init__(self, depth, bits):
        super().__init__()
        self.depth = int(depth)
        for l in range(7):
            self.bits[l] = int(bits[l]) if l < len(bits) else 0

    def record_bytes(self):
        n = int(library().pq_general_record_bytes(ctypes.byref(self)))
        if n == 0:
            raise PolarQuantError("general format refused (depth 4..7; bits: level 1 in {3,4}, 2-4 in {2,3}, 5-7 in {1,2,3})")
        return n

    def codebooks(self):
        """Lloyd-Max centroids of levels 1..depth, concatenated (numpy float64)."""
        n = int(library().pq_general_codebook_entries(ctypes.byref(self)))
        if n == 0:
            raise PolarQuantError("general format refused")
        out = np.empty(n, dtype=np.float64)
        _check(library().pq_general_codebooks(ctypes.byref(self), out.ctypes.data_as(ctypes.c_void_p)))
        return out


def _cbg(cbg):
    return np.ascontiguousarray(cbg, dtype=np.float64)


def general_encode(ctx, fmt, cbg, x, records):
    """x [n, 128] (bf16 or fp32 device tensor, rows contiguous) -> records (uint8 device tensor [n, record bytes])."""
    cb = _cbg(cbg)
    _check(library().pq_general_encode(ctx._h, ctypes.byref(fmt), cb.ctypes.data_as(ctypes.c_void_p), x.data_ptr(),
                                       _dtype_code(x), int(x.shape[0]), int(x.stride(0)), records.data_ptr(), _stream()))


def general_decode(ctx, fmt, cbg, records, n, out, rotated=False):
    cb = _cbg(cbg)
    _check(library().pq_general_decode(ctx._h, ctypes.byref(fmt), cb.ctypes.data_as(ctypes.c_void_p), records.data_ptr(),
                                       int(n), 1 if rotated else 0, out.data_ptr(), _stream()))


def general_attn_decode(ctx, fmt, cbg, q, out, k_records, v_records, seq_start, ctx_len, scale):
    """q bf16 [B, Hq, 128]; records uint8 [Hkv, pool_tokens, record bytes]; out fp32 [B, Hq, 128]."""
    cb = _cbg(cbg)
    B, Hq, _ = q.shape
    _check(library().pq_general_attn_decode(ctx._h, ctypes.byref(fmt), cb.ctypes.data_as(ctypes.c_void_p), q.data_ptr(),
                                            out.data_ptr(), k_records.data_ptr(), v_records.data_ptr(),
                                            seq_start.data_ptr(), ctx_len.data_ptr(), int(B), int(Hq),
                                            int(k_records.shape[0]), int(k_records.shape[1]), float(scale), _stream()))
