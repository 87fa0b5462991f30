"""ctypes binding of libwt.so: same names as include/wt.h, argument marshalling only.

Device buffers are torch tensors (used for memory and streams only); every step of the path
runs inside the library.  The library must have been built (python -m paper_2604_10187_amd.build);
loading fails loudly otherwise -- there is no fallback implementation.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwt.so")

WT_OK = 0
WT_ERR_INVALID_ARG, WT_ERR_UNSUPPORTED_CFG, WT_ERR_INFEASIBLE, WT_ERR_NOT_FITTED = -1, -2, -3, -4
WT_ERR_HIP, WT_ERR_BUFFER_TOO_SMALL, WT_ERR_IO, WT_ERR_NO_DEVICE, WT_ERR_NO_MEMORY = -5, -6, -7, -8, -9
WT_BF16, WT_FP8_E4M3, WT_ATTN_BF16 = 0, 1, 2
WT_OUT_F32, WT_OUT_BF16 = 0, 1
WT_MODEL_WAVE_BILINEAR, WT_MODEL_LINEAR, WT_MODEL_STEP = 0, 1, 2
WT_FIT_ABSOLUTE, WT_FIT_RELATIVE = 0, 1
WT_ROWS_TILES, WT_ROWS_BAND = 0, 1
WT_CAP_CU_TIMES_OCC, WT_CAP_CU_ONLY = 0, 1
WT_SPLITK_WS_FLOATS, WT_SPLITK_MAX_TILES, WT_MAX_ANCHORS = 1 << 26, 1 << 16, 8   # as #defined in wt.h
WT_NOALLOC_WS_FLOATS, WT_NOALLOC_MAX_TILES = 1 << 24, 1 << 15


class wt_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("bm", "bn", "bk", "nwave", "stages", "swizzle", "split", "id")]

    def astuple(self):
        return (self.bm, self.bn, self.bk, self.nwave, self.stages, self.swizzle, self.split)

    def __repr__(self):
        return (f"wt_cfg(bm={self.bm}, bn={self.bn}, bk={self.bk}, nwave={self.nwave}, stages={self.stages}, "
                f"swizzle={self.swizzle}, split={self.split}, id={self.id})")


class wt_cfg_res(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("lds_bytes", "vgprs", "nwave", "occ", "key_id", "micro_id")]


class wt_sample(C.Structure):
    _fields_ = [("key_id", C.c_int32), ("micro_id", C.c_int32), ("G", C.c_int64), ("L", C.c_int64),
                ("w", C.c_int32), ("family", C.c_int32), ("mean_us", C.c_double)]


SAMPLE_DTYPE = np.dtype([("key_id", "<i4"), ("micro_id", "<i4"), ("G", "<i8"), ("L", "<i8"),
                         ("w", "<i4"), ("family", "<i4"), ("mean_us", "<f8")])
assert SAMPLE_DTYPE.itemsize == C.sizeof(wt_sample)


class wt_grid(C.Structure):
    _fields_ = [("W", C.c_int32), ("I", C.c_int32), ("tau_num", C.c_int32), ("tau_den", C.c_int32),
                ("p", C.c_int32), ("n_k_anchors", C.c_int32), ("k_anchors", C.POINTER(C.c_int32)),
                ("warmup", C.c_int32), ("iters", C.c_int32), ("key_first", C.c_int32),
                ("key_count", C.c_int32), ("max_out_elems", C.c_int64), ("model", C.c_int32),
                ("W_split", C.c_int32), ("W_row", C.c_int32), ("row_fams", C.c_int32), ("skip_near", C.c_int32),
                ("n_heads", C.c_int32), ("weighting", C.c_int32), ("row_mode", C.c_int32)]


class WtError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_10187_amd.build` "
                               "(there is no fallback path)")
        # PyTorch ships its own HIP runtime; load it first so that libwt binds to the same copy
        # (two HIP runtimes in one process do not see each other's devices, streams or memory).
        import torch  # noqa: F401

        L = C.CDLL(LIB_PATH)
        vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int32, C.c_size_t
        sig = {
            "wt_create": [C.POINTER(vp), C.c_int, C.c_int, C.c_int],
            "wt_destroy": [vp],
            "wt_last_hip_error": [vp],
            "wt_config_count": [vp, C.POINTER(C.c_int)],
            "wt_config_get": [vp, C.c_int, C.POINTER(wt_cfg), C.POINTER(wt_cfg_res)],
            "wt_config_find": [vp, C.POINTER(wt_cfg), C.POINTER(C.c_int)],
            "wt_key_count": [vp, C.POINTER(C.c_int)],
            "wt_key_set_occ": [vp, C.c_int, C.c_int],
            "wt_set_capacity_mode": [vp, C.c_int],
            "wt_set_persistent": [vp, C.c_int],
            "wt_tile_coords": [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)],
            "wt_gemm": [vp, i64, i64, i64, vp, vp, vp, vp, vp, wt_cfg, vp],
            "wt_gemm_noalloc": [vp, i64, i64, i64, vp, vp, vp, vp, vp, wt_cfg, vp],
            "wt_gemm_grouped": [vp, i32, vp, i64, i64, i64, vp, vp, vp, vp, vp, wt_cfg, vp],
            "wt_time_gemm_grouped": [vp, i32, vp, i64, i64, i64, vp, vp, vp, vp, vp, wt_cfg, C.c_int, C.c_int, vp,
                                     C.POINTER(C.c_double)],
            "wt_wave_count_grouped": [vp, i32, vp, i64, i64, wt_cfg, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32)],
            "wt_select_grouped": [vp, i32, i64, i64, i64, C.POINTER(wt_cfg)],
            "wt_select_grouped_rows": [vp, i32, vp, i64, i64, C.POINTER(wt_cfg)],
            "wt_select_attn_varlen": [vp, i32, vp, vp, i64, C.POINTER(wt_cfg)],
            "wt_attn": [vp, i64, i64, i64, i64, vp, vp, vp, vp, C.c_float, C.c_int, wt_cfg, vp],
            "wt_attn_batched": [vp, i64, i64, i64, i64, i64, vp, vp, vp, vp, C.c_float, C.c_int, wt_cfg, vp],
            "wt_attn_varlen": [vp, i64, i64, i64, i64, i64, vp, vp, vp, vp, vp, vp, C.c_float, C.c_int, wt_cfg, vp],
            "wt_time_attn": [vp, i64, i64, i64, i64, vp, vp, vp, vp, C.c_float, C.c_int, wt_cfg, C.c_int, C.c_int, vp,
                             C.POINTER(C.c_double)],
            "wt_attn_block_coords": [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)],
            "wt_sample_grid_heads": [i64, i32, i32, i32, vp, vp, sz, C.POINTER(sz)],
            "wt_wave_count": [vp, i64, i64, i64, wt_cfg, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32)],
            "wt_sample_grid": [i64, i32, i32, i32, i32, i32, vp, vp, vp, sz, C.POINTER(sz)],
            "wt_sample_plan": [vp, C.POINTER(wt_grid), C.POINTER(sz), C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)],
            "wt_profile_sparse": [vp, C.POINTER(wt_grid), vp, vp, vp, sz, sz, sz, vp, vp, sz, C.POINTER(sz)],
            "wt_time_gemm": [vp, i64, i64, i64, vp, vp, vp, vp, vp, wt_cfg, C.c_int, C.c_int, vp, C.POINTER(C.c_double)],
            "wt_mfma_ceiling": [vp, C.c_int, C.c_int, vp, vp, C.POINTER(C.c_double)],
            "wt_fit": [vp, C.POINTER(wt_grid), vp, sz],
            "wt_select": [vp, i64, i64, i64, C.POINTER(wt_cfg)],
            "wt_predict_us": [vp, i64, i64, i64, wt_cfg, C.POINTER(C.c_double)],
            "wt_select_bench": [vp, vp, sz, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)],
            "wt_save": [vp, C.c_char_p],
            "wt_load": [vp, C.c_char_p],
        }
        for name, args in sig.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = C.c_int
        L.wt_status_string.argtypes = [C.c_int]
        L.wt_status_string.restype = C.c_char_p
        _lib = L
    return _lib


EXPORTS = ("wt_create", "wt_destroy", "wt_last_hip_error", "wt_status_string", "wt_config_count", "wt_config_get",
           "wt_config_find", "wt_key_count", "wt_key_set_occ", "wt_set_capacity_mode", "wt_set_persistent", "wt_tile_coords", "wt_gemm", "wt_gemm_noalloc", "wt_gemm_grouped",
           "wt_time_gemm_grouped", "wt_wave_count_grouped", "wt_select_grouped", "wt_select_grouped_rows", "wt_select_attn_varlen", "wt_wave_count", "wt_sample_grid",
           "wt_sample_plan", "wt_profile_sparse", "wt_time_gemm", "wt_mfma_ceiling", "wt_fit", "wt_select", "wt_predict_us",
           "wt_select_bench", "wt_save", "wt_load", "wt_attn", "wt_attn_batched", "wt_attn_varlen", "wt_time_attn", "wt_attn_block_coords",
           "wt_sample_grid_heads")


def status_string(status: int) -> str:
    return lib().wt_status_string(int(status)).decode()


def _check(rc, what):
    if rc != WT_OK:
        raise WtError(rc, what)


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / None."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return None
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


def make_grid(W=40, I=4, tau=(11, 10), p=10, k_anchors=(1024, 2048, 3072, 4096, 5120), warmup=3, iters=5,
              key_first=0, key_count=0, max_out_elems=0, model=0, W_row=0, W_split=0, row_fams=0, skip_near=0,
              n_heads=0, weighting=0, row_mode=0):
    arr = (C.c_int32 * len(k_anchors))(*k_anchors)
    g = wt_grid(W, I, tau[0], tau[1], p, len(k_anchors), C.cast(arr, C.POINTER(C.c_int32)), warmup, iters,
                key_first, key_count, max_out_elems, model, W_split, W_row, row_fams, skip_near, n_heads, weighting, row_mode)
    g._keep = arr  # keep the anchor array alive with the struct
    return g


# ---- functions named as in wt.h ---------------------------------------------------------------
def wt_create(device: int, in_type: int = WT_BF16, out_type: int = WT_OUT_F32):
    h = C.c_void_p()
    _check(lib().wt_create(C.byref(h), device, in_type, out_type), "wt_create")
    return h


def wt_destroy(ctx):
    _check(lib().wt_destroy(ctx), "wt_destroy")


def wt_last_hip_error(ctx) -> int:
    return lib().wt_last_hip_error(ctx)


def wt_config_count(ctx) -> int:
    n = C.c_int()
    _check(lib().wt_config_count(ctx, C.byref(n)), "wt_config_count")
    return n.value


def wt_key_count(ctx) -> int:
    n = C.c_int()
    _check(lib().wt_key_count(ctx, C.byref(n)), "wt_key_count")
    return n.value


def wt_config_get(ctx, i: int):
    c, r = wt_cfg(), wt_cfg_res()
    _check(lib().wt_config_get(ctx, i, C.byref(c), C.byref(r)), "wt_config_get")
    return c, r


def wt_config_find(ctx, bm, bn, bk, nwave, stages, swizzle, split=1) -> int:
    c = wt_cfg(bm, bn, bk, nwave, stages, swizzle, split, -1)
    i = C.c_int()
    _check(lib().wt_config_find(ctx, C.byref(c), C.byref(i)), "wt_config_find")
    return i.value


def wt_key_set_occ(ctx, key_id: int, occ: int):
    _check(lib().wt_key_set_occ(ctx, key_id, occ), "wt_key_set_occ")


def wt_set_capacity_mode(ctx, mode: int):
    _check(lib().wt_set_capacity_mode(ctx, mode), "wt_set_capacity_mode")


def wt_set_persistent(ctx, on):
    """0 / False: one block per task; 1 / True: resident blocks walk the task list with a fixed stride; 2: they draw
    their tasks from a device-side queue."""
    _check(lib().wt_set_persistent(ctx, int(on)), "wt_set_persistent")


def wt_tile_coords(tiles_m, tiles_n, swizzle, block):
    tm, tn = C.c_int(), C.c_int()
    _check(lib().wt_tile_coords(tiles_m, tiles_n, swizzle, block, C.byref(tm), C.byref(tn)), "wt_tile_coords")
    return tm.value, tn.value


def wt_gemm(ctx, M, N, K, A, B, Cout, cfg, scaleA=None, scaleB=None, stream=None):
    _check(lib().wt_gemm(ctx, M, N, K, _ptr(A), _ptr(B), _ptr(Cout), _ptr(scaleA), _ptr(scaleB), cfg,
                         _stream(stream)), "wt_gemm")


def wt_gemm_noalloc(ctx, M, N, K, A, B, Cout, cfg, scaleA=None, scaleB=None, stream=None):
    _check(lib().wt_gemm_noalloc(ctx, M, N, K, _ptr(A), _ptr(B), _ptr(Cout), _ptr(scaleA), _ptr(scaleB), cfg,
                                 _stream(stream)), "wt_gemm_noalloc")


def wt_gemm_grouped(ctx, groups, offsets, M_total, N, K, A, B, Cout, cfg, scaleA=None, scaleB=None, stream=None):
    """offsets: device int32 tensor of groups+1 row offsets."""
    _check(lib().wt_gemm_grouped(ctx, groups, _ptr(offsets), M_total, N, K, _ptr(A), _ptr(B), _ptr(Cout),
                                 _ptr(scaleA), _ptr(scaleB), cfg, _stream(stream)), "wt_gemm_grouped")


def wt_time_gemm_grouped(ctx, groups, offsets, M_total, N, K, A, B, Cout, cfg, warmup=3, iters=5, scaleA=None,
                         scaleB=None, stream=None) -> float:
    us = C.c_double()
    _check(lib().wt_time_gemm_grouped(ctx, groups, _ptr(offsets), M_total, N, K, _ptr(A), _ptr(B), _ptr(Cout),
                                      _ptr(scaleA), _ptr(scaleB), cfg, warmup, iters, _stream(stream),
                                      C.byref(us)), "wt_time_gemm_grouped")
    return us.value


def wt_attn_batched(ctx, batch, n_heads, n_kv_heads, S_q, S_kv, Q, K, V, O, scale, causal, cfg, stream=None):
    """Q, O: [batch, S_q, n_heads, 128]; K, V: [batch, S_kv, n_kv_heads, 128]; device bf16."""
    _check(lib().wt_attn_batched(ctx, batch, n_heads, n_kv_heads, S_q, S_kv, _ptr(Q), _ptr(K), _ptr(V), _ptr(O),
                                 float(scale), int(bool(causal)), cfg, _stream(stream)), "wt_attn_batched")


def wt_attn_varlen(ctx, batch, n_heads, n_kv_heads, total_q, total_kv, cu_q, cu_kv, Q, K, V, O, scale, causal, cfg,
                   stream=None):
    """cu_q, cu_kv: device int32 tensors of batch + 1 token offsets; Q, O: [total_q, n_heads, 128]; K, V: [total_kv, n_kv_heads, 128]."""
    _check(lib().wt_attn_varlen(ctx, batch, n_heads, n_kv_heads, total_q, total_kv, _ptr(cu_q), _ptr(cu_kv), _ptr(Q),
                                _ptr(K), _ptr(V), _ptr(O), float(scale), int(bool(causal)), cfg, _stream(stream)),
           "wt_attn_varlen")


def wt_attn(ctx, n_heads, n_kv_heads, S_q, S_kv, Q, K, V, O, scale, causal, cfg, stream=None):
    """Q, O: [S_q, n_heads, 128]; K, V: [S_kv, n_kv_heads, 128]; bf16 device tensors."""
    _check(lib().wt_attn(ctx, n_heads, n_kv_heads, S_q, S_kv, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), float(scale),
                         int(bool(causal)), cfg, _stream(stream)), "wt_attn")


def wt_time_attn(ctx, n_heads, n_kv_heads, S_q, S_kv, Q, K, V, O, scale, causal, cfg, warmup=3, iters=5,
                 stream=None) -> float:
    us = C.c_double()
    _check(lib().wt_time_attn(ctx, n_heads, n_kv_heads, S_q, S_kv, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), float(scale),
                              int(bool(causal)), cfg, warmup, iters, _stream(stream), C.byref(us)), "wt_time_attn")
    return us.value


def wt_attn_block_coords(n_heads, q_tiles, order, block):
    h, q = C.c_int(), C.c_int()
    _check(lib().wt_attn_block_coords(n_heads, q_tiles, order, block, C.byref(h), C.byref(q)), "wt_attn_block_coords")
    return h.value, q.value


def wt_sample_grid_heads(capacity, W, I, n_heads):
    n = W * I
    g, q = np.zeros(n, dtype=np.int64), np.zeros(n, dtype=np.int64)
    got = C.c_size_t()
    _check(lib().wt_sample_grid_heads(capacity, W, I, n_heads, g.ctypes.data, q.ctypes.data, n, C.byref(got)),
           "wt_sample_grid_heads")
    return g[:got.value], q[:got.value]


def wt_wave_count_grouped(ctx, group_rows, N, K, cfg):
    rows = np.ascontiguousarray(np.asarray(group_rows, dtype=np.int64))
    G, L, w = C.c_int64(), C.c_int64(), C.c_int32()
    _check(lib().wt_wave_count_grouped(ctx, len(rows), rows.ctypes.data, N, K, cfg, C.byref(G), C.byref(L),
                                       C.byref(w)), "wt_wave_count_grouped")
    return G.value, L.value, w.value


def wt_select_grouped(ctx, groups, M_total, N, K) -> wt_cfg:
    c = wt_cfg()
    _check(lib().wt_select_grouped(ctx, groups, M_total, N, K, C.byref(c)), "wt_select_grouped")
    return c


def wt_select_grouped_rows(ctx, group_rows, N, K) -> wt_cfg:
    rows = np.ascontiguousarray(np.asarray(group_rows, dtype=np.int64))
    c = wt_cfg()
    _check(lib().wt_select_grouped_rows(ctx, len(rows), rows.ctypes.data, N, K, C.byref(c)), "wt_select_grouped_rows")
    return c


def wt_select_attn_varlen(ctx, len_q, len_kv, n_heads) -> wt_cfg:
    lq = np.ascontiguousarray(np.asarray(len_q, dtype=np.int64))
    lkv = np.ascontiguousarray(np.asarray(len_kv, dtype=np.int64))
    if len(lq) != len(lkv):
        raise ValueError("one kv length per query length")
    c = wt_cfg()
    _check(lib().wt_select_attn_varlen(ctx, len(lq), lq.ctypes.data, lkv.ctypes.data, n_heads, C.byref(c)),
           "wt_select_attn_varlen")
    return c


def wt_time_gemm(ctx, M, N, K, A, B, Cout, cfg, warmup=3, iters=5, scaleA=None, scaleB=None, stream=None) -> float:
    us = C.c_double()
    _check(lib().wt_time_gemm(ctx, M, N, K, _ptr(A), _ptr(B), _ptr(Cout), _ptr(scaleA), _ptr(scaleB), cfg,
                              warmup, iters, _stream(stream), C.byref(us)), "wt_time_gemm")
    return us.value


def wt_mfma_ceiling(ctx, in_type=WT_BF16, iters=20000, stream=None) -> float:
    import torch

    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    tf = C.c_double()
    _check(lib().wt_mfma_ceiling(ctx, in_type, iters, _stream(stream), _ptr(sink), C.byref(tf)), "wt_mfma_ceiling")
    return tf.value


def wt_wave_count(ctx, M, N, K, cfg):
    G, L, w = C.c_int64(), C.c_int64(), C.c_int32()
    _check(lib().wt_wave_count(ctx, M, N, K, cfg, C.byref(G), C.byref(L), C.byref(w)), "wt_wave_count")
    return G.value, L.value, w.value


def wt_sample_grid(capacity, W, I, tau_num=11, tau_den=10, split=1):
    n = W * I
    g, m, nn = (np.zeros(n, dtype=np.int64) for _ in range(3))
    got = C.c_size_t()
    _check(lib().wt_sample_grid(capacity, W, I, tau_num, tau_den, split, g.ctypes.data, m.ctypes.data, nn.ctypes.data,
                                n, C.byref(got)), "wt_sample_grid")
    return g[:got.value], m[:got.value], nn[:got.value]


def wt_sample_plan(ctx, grid):
    n, a, b, c = (C.c_size_t() for _ in range(4))
    _check(lib().wt_sample_plan(ctx, C.byref(grid), C.byref(n), C.byref(a), C.byref(b), C.byref(c)), "wt_sample_plan")
    return n.value, a.value, b.value, c.value


def wt_profile_sparse(ctx, grid, scrA, scrB, scrC, stream=None) -> np.ndarray:
    n, _, _, _ = wt_sample_plan(ctx, grid)
    out = np.zeros(max(n, 1), dtype=SAMPLE_DTYPE)
    got = C.c_size_t()
    nbytes = lambda t: t.numel() * t.element_size()
    _check(lib().wt_profile_sparse(ctx, C.byref(grid), _ptr(scrA), _ptr(scrB), _ptr(scrC), nbytes(scrA),
                                   nbytes(scrB), nbytes(scrC), _stream(stream), out.ctypes.data, n,
                                   C.byref(got)), "wt_profile_sparse")
    return out[:got.value]


def wt_fit(ctx, grid, samples: np.ndarray):
    s = np.ascontiguousarray(samples, dtype=SAMPLE_DTYPE)
    _check(lib().wt_fit(ctx, C.byref(grid), s.ctypes.data, len(s)), "wt_fit")


def wt_select(ctx, M, N, K) -> wt_cfg:
    c = wt_cfg()
    _check(lib().wt_select(ctx, M, N, K, C.byref(c)), "wt_select")
    return c


def wt_predict_us(ctx, M, N, K, cfg) -> float:
    us = C.c_double()
    _check(lib().wt_predict_us(ctx, M, N, K, cfg, C.byref(us)), "wt_predict_us")
    return us.value


def wt_select_bench(ctx, shapes, repeats=3):
    s = np.ascontiguousarray(np.asarray(shapes, dtype=np.int64).reshape(-1, 3))
    mean, p99 = C.c_double(), C.c_double()
    _check(lib().wt_select_bench(ctx, s.ctypes.data, len(s), repeats, C.byref(mean), C.byref(p99)), "wt_select_bench")
    return mean.value, p99.value


def wt_save(ctx, path: str):
    _check(lib().wt_save(ctx, path.encode()), "wt_save")


def wt_load(ctx, path: str):
    _check(lib().wt_load(ctx, path.encode()), "wt_load")
