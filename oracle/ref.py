"""numpy-facing wrapper around liboracle.so (see oracle.c for what each routine computes).

bf16 tensors travel as uint16 bit patterns; results come back as float64 arrays.
"""
import ctypes as C
import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.oracle_bf16_to_f64.restype = C.c_double
        _lib.oracle_bf16_to_f64.argtypes = [C.c_uint16]
        _lib.oracle_f64_to_bf16.restype = C.c_uint16
        _lib.oracle_f64_to_bf16.argtypes = [C.c_double]
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def bf16_to_f64(bits):
    """uint16 bit patterns -> float64 (vectorised through the C helper)."""
    bits = _u16(bits)
    out = np.empty(bits.shape, dtype=np.float64)
    lib().oracle_widen_bf16(_p(bits, C.c_uint16), _p(out, C.c_double), C.c_int64(bits.size))
    return out


def round_to_bf16(y):
    """float64 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    y = np.ascontiguousarray(y, dtype=np.float64)
    out = np.empty(y.shape, dtype=np.uint16)
    lib().oracle_round_to_bf16(_p(y, C.c_double), _p(out, C.c_uint16), C.c_int64(y.size))
    return out


def apply_decode(x, y, A_tab, B_tab, rank, alpha, token_slot):
    """x [T,d_in], y [T,d_out], A_tab [S,r_max,d_in], B_tab [S,d_out,r_max] as uint16 bf16 bits;
    rank [S] int, alpha [S] float, token_slot [T] int.  Returns float64 [T,d_out]."""
    x, y, A_tab, B_tab = _u16(x), _u16(y), _u16(A_tab), _u16(B_tab)
    T, d_in = x.shape
    d_out = y.shape[1]
    S, r_max, _ = A_tab.shape
    assert A_tab.shape == (S, r_max, d_in) and B_tab.shape == (S, d_out, r_max) and y.shape[0] == T
    rank = _i32(rank)
    alpha = np.ascontiguousarray(np.asarray(alpha, dtype=np.float64))
    token_slot = _i32(token_slot)
    assert rank.shape == (S,) and alpha.shape == (S,) and token_slot.shape == (T,)
    out = np.empty((T, d_out), dtype=np.float64)
    rc = lib().oracle_apply_decode(
        _p(x, C.c_uint16), _p(y, C.c_uint16), _p(out, C.c_double),
        _p(A_tab, C.c_uint16), _p(B_tab, C.c_uint16), _p(rank, C.c_int32), _p(alpha, C.c_double),
        _p(token_slot, C.c_int32),
        C.c_int64(T), C.c_int64(d_in), C.c_int64(d_out), C.c_int64(S), C.c_int64(r_max))
    if rc != 0:
        raise ValueError(f"oracle_apply_decode rc={rc}")
    return out


def apply_segmented(x, y, A_tab, B_tab, rank, alpha, seg_off, seg_slot):
    x, y, A_tab, B_tab = _u16(x), _u16(y), _u16(A_tab), _u16(B_tab)
    T, d_in = x.shape
    d_out = y.shape[1]
    S, r_max, _ = A_tab.shape
    assert A_tab.shape == (S, r_max, d_in) and B_tab.shape == (S, d_out, r_max) and y.shape[0] == T
    rank = _i32(rank)
    alpha = np.ascontiguousarray(np.asarray(alpha, dtype=np.float64))
    seg_off, seg_slot = _i32(seg_off), _i32(seg_slot)
    nseg = seg_slot.shape[0]
    assert seg_off.shape == (nseg + 1,)
    out = np.empty((T, d_out), dtype=np.float64)
    rc = lib().oracle_apply_segmented(
        _p(x, C.c_uint16), _p(y, C.c_uint16), _p(out, C.c_double),
        _p(A_tab, C.c_uint16), _p(B_tab, C.c_uint16), _p(rank, C.c_int32), _p(alpha, C.c_double),
        _p(seg_off, C.c_int32), _p(seg_slot, C.c_int32), C.c_int64(nseg),
        C.c_int64(T), C.c_int64(d_in), C.c_int64(d_out), C.c_int64(S), C.c_int64(r_max))
    if rc != 0:
        raise ValueError(f"oracle_apply_segmented rc={rc}")
    return out


def apply_moe(x, y, A_tab, B_tab, rank, alpha, topk, token_slot):
    """x [T,d_in]; y [T*K,d_out]; A_tab [S,E,r_max,d_in]; B_tab [S,E,d_out,r_max]; topk [T,K]."""
    x, y, A_tab, B_tab = _u16(x), _u16(y), _u16(A_tab), _u16(B_tab)
    T, d_in = x.shape
    topk = _i32(topk)
    K = topk.shape[1]
    d_out = y.shape[1]
    S, E, r_max, _ = A_tab.shape
    assert A_tab.shape == (S, E, r_max, d_in) and B_tab.shape == (S, E, d_out, r_max)
    assert y.shape[0] == T * K and topk.shape == (T, K)
    rank = _i32(rank)
    alpha = np.ascontiguousarray(np.asarray(alpha, dtype=np.float64))
    token_slot = _i32(token_slot)
    out = np.empty((T * K, d_out), dtype=np.float64)
    rc = lib().oracle_apply_moe(
        _p(x, C.c_uint16), _p(y, C.c_uint16), _p(out, C.c_double),
        _p(A_tab, C.c_uint16), _p(B_tab, C.c_uint16), _p(rank, C.c_int32), _p(alpha, C.c_double),
        _p(topk, C.c_int32), _p(token_slot, C.c_int32),
        C.c_int64(T), C.c_int64(K), C.c_int64(E),
        C.c_int64(d_in), C.c_int64(d_out), C.c_int64(S), C.c_int64(r_max))
    if rc != 0:
        raise ValueError(f"oracle_apply_moe rc={rc}")
    return out


def apply_moe_down(x, y, A_tab, B_tab, rank, alpha, topk, w, token_slot):
    """Down projection with the routing-weight combine.  x [T*K,d_in] (one input row per pair);
    y [T,d_out]; w [T,K] routing weights; A_tab [S,E,r_max,d_in]; B_tab [S,E,d_out,r_max]."""
    x, y, A_tab, B_tab = _u16(x), _u16(y), _u16(A_tab), _u16(B_tab)
    topk = _i32(topk)
    T, K = topk.shape
    d_in, d_out = x.shape[1], y.shape[1]
    S, E, r_max, _ = A_tab.shape
    assert A_tab.shape == (S, E, r_max, d_in) and B_tab.shape == (S, E, d_out, r_max)
    assert x.shape[0] == T * K and y.shape[0] == T
    w = np.ascontiguousarray(np.asarray(w, dtype=np.float64))
    assert w.shape == (T, K)
    rank = _i32(rank)
    alpha = np.ascontiguousarray(np.asarray(alpha, dtype=np.float64))
    token_slot = _i32(token_slot)
    out = np.empty((T, d_out), dtype=np.float64)
    rc = lib().oracle_apply_moe_down(
        _p(x, C.c_uint16), _p(y, C.c_uint16), _p(out, C.c_double),
        _p(A_tab, C.c_uint16), _p(B_tab, C.c_uint16), _p(rank, C.c_int32), _p(alpha, C.c_double),
        _p(topk, C.c_int32), _p(w, C.c_double), _p(token_slot, C.c_int32),
        C.c_int64(T), C.c_int64(K), C.c_int64(E),
        C.c_int64(d_in), C.c_int64(d_out), C.c_int64(S), C.c_int64(r_max))
    if rc != 0:
        raise ValueError(f"oracle_apply_moe_down rc={rc}")
    return out


def route_sort(topk, token_slot, rank, n_experts):
    """Returns (sorted_pair [T*K] int32 with -1 tail, group_off [S*E+1] int32)."""
    topk = _i32(topk)
    T, K = topk.shape
    token_slot, rank = _i32(token_slot), _i32(rank)
    S = rank.shape[0]
    sorted_pair = np.empty(T * K, dtype=np.int32)
    group_off = np.empty(S * n_experts + 1, dtype=np.int32)
    rc = lib().oracle_route_sort(
        _p(topk, C.c_int32), _p(token_slot, C.c_int32), _p(rank, C.c_int32),
        C.c_int64(T), C.c_int64(K), C.c_int64(n_experts), C.c_int64(S),
        _p(sorted_pair, C.c_int32), _p(group_off, C.c_int32))
    if rc != 0:
        raise ValueError(f"oracle_route_sort rc={rc}")
    return sorted_pair, group_off
