"""ctypes binding with the same names as the C ABI in include/mlora.h (argument marshalling only)."""
import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MLORA_LIB") or os.path.join(HERE, "libmlora.so")   # MLORA_LIB: a variant build of the same library

STATUS = {0: "MLORA_OK", -1: "MLORA_E_INVALID", -2: "MLORA_E_SHAPE", -3: "MLORA_E_SLOT",
          -4: "MLORA_E_SEGMENTS", -5: "MLORA_E_HIP", -6: "MLORA_E_UNSUPPORTED"}


class MLoraError(RuntimeError):
    def __init__(self, fn, status, text):
        super().__init__(f"{fn}: {STATUS.get(status, status)} ({text})")
        self.status = status


class SiteDesc(C.Structure):
    _fields_ = [("d_in", C.c_int32), ("d_out", C.c_int32), ("r_max", C.c_int32),
                ("n_slots", C.c_int32), ("n_experts", C.c_int32), ("device", C.c_int32)]


_lib = None
_vp, _i32, _i64, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t

SIGNATURES = {
    "mlora_status_str": (C.c_char_p, [_i32]),
    "mlora_set_tuning": (_i32, [C.c_char_p, _i32]),
    "mlora_site_bytes": (_i32, [C.POINTER(SiteDesc)] + [C.POINTER(_sz)] * 4),
    "mlora_site_create": (_i32, [C.POINTER(SiteDesc), _vp, _vp, _vp, _vp, C.POINTER(_vp)]),
    "mlora_site_destroy": (None, [_vp]),
    "mlora_site_check": (_i32, [_vp, _vp]),
    "lora_slots_upload": (_i32, [_vp, _i32, _i64, _vp, _vp, _i32, C.c_float, _i32, _vp]),
    "lora_slots_evict": (_i32, [_vp, _i32, _vp]),
    "lora_slot_lookup": (_i32, [_vp, _vp, _i32, _vp, _vp]),
    "mlora_slot_image_bytes": (_i32, [C.POINTER(SiteDesc)] + [C.POINTER(_sz)] * 2),
    "mlora_pack_experts": (_i32, [C.POINTER(SiteDesc), C.POINTER(_vp), C.POINTER(_vp), _i32, _vp, _vp]),
    "lora_slots_upload_experts": (_i32, [_vp, _i32, _i64, C.POINTER(_vp), C.POINTER(_vp), _i32, C.c_float, _vp]),
    "mlora_plan_bytes": (_i32, [_i32, _i32, C.POINTER(_sz)]),
    "mlora_plan_create": (_i32, [_i32, _i32, _i32, _vp, C.POINTER(_vp)]),
    "mlora_plan_destroy": (None, [_vp]),
    "lora_plan_decode": (_i32, [_vp, _vp, _i32, _i32, _vp, _vp]),
    "lora_apply_decode_planned": (_i32, [_vp, _vp, _vp, _i64, _vp, _i64, _vp]),
    "lora_apply_decode_multi": (_i32, [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "lora_plan_apply_decode_multi": (_i32, [_vp, _i32, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_plan_route": (_i32, [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp]),
    "moe_lora_apply_planned": (_i32, [_vp, _vp, _vp, _i64, _vp, _i64, _vp]),
    "moe_lora_apply_multi": (_i32, [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_down_workspace_bytes": (_i32, [_i32, _i32, _i32, C.POINTER(_sz)]),
    "moe_lora_apply_down": (_i32, [_vp, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _i64, _vp]),
    "mlora_resident_create": (_i32, [_i32, _i32, _i32, C.POINTER(_vp)]),
    "mlora_resident_destroy": (None, [_vp]),
    "mlora_resident_register": (_i32, [_vp, _i64]),
    "mlora_resident_lookup": (_i32, [_vp, _i64]),
    "mlora_resident_request": (_i32, [_vp, _i64, C.POINTER(_i32), C.POINTER(_i64)]),
    "mlora_resident_complete": (_i32, [_vp, _i64, _i32, C.POINTER(_i64), C.POINTER(_i32), C.POINTER(_i64)]),
    "mlora_resident_pin": (_i32, [_vp, _i32, _i32]),
    "mlora_resident_stats": (_i32, [_vp, C.POINTER(_i64)]),
    "lora_apply_decode": (_i32, [_vp, _vp, _i64, _vp, _i64, _vp, _i32, _vp]),
    "lora_apply_decode_noalloc": (_i32, [_vp, _vp, _i64, _vp, _i64, _vp, _i32, _vp]),
    "lora_apply_segmented": (_i32, [_vp, _vp, _i64, _vp, _i64, _vp, _vp, _i32, _i32, _vp]),
    "moe_lora_apply_packed": (_i32, [_vp, _vp, _i64, _vp, _i64, _vp, _vp, _i32, _i32, _vp, _vp, _vp]),
}


def load_library():
    """Load libmlora.so; there is no fallback path if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2605_13779_amd.build` "
                              "(the HIP library is the only implementation)")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _check(fn, status):
    if status != 0:
        raise MLoraError(fn, status, load_library().mlora_status_str(status).decode())


def set_tuning(name: str, value: int):
    _check("mlora_set_tuning", load_library().mlora_set_tuning(name.encode(), int(value)))


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev_ptr(t, dtype=None):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda, "expected a device tensor"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return C.c_void_p(t.data_ptr())


def _rows(t):
    assert t.dim() == 2 and t.stride(1) == 1 and t.dtype == torch.bfloat16 and t.is_cuda
    return C.c_void_p(t.data_ptr()), int(t.stride(0))


class Site:
    """One LoRA-targeted projection: owns the torch buffers that back the slot tables."""

    def __init__(self, d_in, d_out, r_max, n_slots, n_experts=0, device=0):
        lib = load_library()
        self.desc = SiteDesc(d_in, d_out, r_max, n_slots, n_experts, device)
        sizes = [_sz() for _ in range(4)]
        _check("mlora_site_bytes", lib.mlora_site_bytes(C.byref(self.desc), *[C.byref(s) for s in sizes]))
        dev = torch.device("cuda", device)
        self.bufs = [torch.empty(int(s.value), dtype=torch.uint8, device=dev) for s in sizes]
        self.bytes = [int(s.value) for s in sizes]
        h = _vp()
        _check("mlora_site_create", lib.mlora_site_create(
            C.byref(self.desc), *[C.c_void_p(b.data_ptr()) for b in self.bufs], C.byref(h)))
        self.handle = h
        self.d_in, self.d_out, self.r_max, self.n_slots, self.n_experts = d_in, d_out, r_max, n_slots, n_experts

    def meta(self):
        """(rank int32[n_slots], scale fp32[n_slots], catalog_id int64[n_slots]) read back to the host."""
        raw = self.bufs[2].cpu().numpy()
        n = self.n_slots
        return (raw[:4 * n].view(np.int32).copy(), raw[4 * n:8 * n].view(np.float32).copy(),
                raw[8 * n:16 * n].view(np.int64).copy())

    def check(self, stream=None):
        _check("mlora_site_check", load_library().mlora_site_check(self.handle, _stream(stream)))

    def close(self):
        if self.handle is not None:
            load_library().mlora_site_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Plan:
    def __init__(self, max_items, n_keys, device=0):
        lib = load_library()
        n = _sz()
        _check("mlora_plan_bytes", lib.mlora_plan_bytes(max_items, n_keys, C.byref(n)))
        self.buf = torch.empty(int(n.value), dtype=torch.uint8, device=torch.device("cuda", device))
        h = _vp()
        _check("mlora_plan_create", lib.mlora_plan_create(max_items, n_keys, device, C.c_void_p(self.buf.data_ptr()), C.byref(h)))
        self.handle = h

    def close(self):
        if self.handle is not None:
            load_library().mlora_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _host_or_dev(t):
    """A / B for upload: numpy uint16 / torch CPU bf16 (host) or torch CUDA bf16 (device)."""
    if isinstance(t, np.ndarray):
        t = np.ascontiguousarray(t)
        assert t.dtype == np.uint16
        return C.c_void_p(t.ctypes.data), 0, t
    assert t.dtype == torch.bfloat16 and t.is_contiguous()
    return C.c_void_p(t.data_ptr()), int(t.is_cuda), t


def lora_slots_upload(site, slot, catalog_id, A, B, r, alpha, stream=None):
    pa, da, ka = _host_or_dev(A)
    pb, db, kb = _host_or_dev(B)
    assert da == db
    E = max(site.n_experts, 1)
    na = ka.size if isinstance(ka, np.ndarray) else ka.numel()
    nb = kb.size if isinstance(kb, np.ndarray) else kb.numel()
    assert na == E * r * site.d_in and nb == E * site.d_out * r, "A/B do not match the site and rank"
    _check("lora_slots_upload", load_library().lora_slots_upload(
        site.handle, slot, int(catalog_id), pa, pb, r, float(alpha), da, _stream(stream)))
    if not da:
        torch.cuda.current_stream().synchronize()   # host source must outlive the copy
    return None


def _ptr_array(arrays):
    """ctypes array of host pointers to contiguous uint16 numpy arrays (kept alive by the caller)."""
    return (_vp * len(arrays))(*[a.ctypes.data for a in arrays])


def pack_experts(desc, A_e, B_e, r):
    """Host-only: stack per-expert bf16 tensors (uint16 numpy arrays [r, d_in] / [d_out, r]) into the
    slot image (a_img [E, r_pad, d_in], b_img [E, d_out, r_pad], uint16)."""
    import numpy as np
    lib = load_library()
    na, nb = _sz(), _sz()
    _check("mlora_slot_image_bytes", lib.mlora_slot_image_bytes(C.byref(desc), C.byref(na), C.byref(nb)))
    A_e = [np.ascontiguousarray(a, dtype=np.uint16) for a in A_e]
    B_e = [np.ascontiguousarray(b, dtype=np.uint16) for b in B_e]
    a_img = np.empty(na.value // 2, dtype=np.uint16)
    b_img = np.empty(nb.value // 2, dtype=np.uint16)
    _check("mlora_pack_experts", lib.mlora_pack_experts(C.byref(desc), _ptr_array(A_e), _ptr_array(B_e), r,
                                                        C.c_void_p(a_img.ctypes.data), C.c_void_p(b_img.ctypes.data)))
    return a_img, b_img


class ExpertTensors:
    """The host pointer arrays of an adapter's per-expert tensors (lists of uint16 numpy arrays
    [r, d_in] and [d_out, r]), marshalled once; keeps the arrays alive."""

    def __init__(self, A_e, B_e):
        import numpy as np
        self.A_e = [np.ascontiguousarray(a, dtype=np.uint16) for a in A_e]
        self.B_e = [np.ascontiguousarray(b, dtype=np.uint16) for b in B_e]
        self.pa, self.pb = _ptr_array(self.A_e), _ptr_array(self.B_e)


def lora_slots_upload_experts(site, slot, catalog_id, A_e, B_e, r, alpha, stream=None):
    """A_e / B_e: lists of per-expert uint16 numpy arrays ([r, d_in] and [d_out, r]), or A_e an
    ExpertTensors (then B_e is ignored)."""
    t = A_e if isinstance(A_e, ExpertTensors) else ExpertTensors(A_e, B_e)
    _check("lora_slots_upload_experts", load_library().lora_slots_upload_experts(
        site.handle, slot, catalog_id, t.pa, t.pb, r, alpha, _stream(stream)))


def lora_slot_lookup(site, token_catalog_id, token_slot_out, stream=None):
    """token_catalog_id: int64 device tensor [T]; token_slot_out: int32 device tensor [T]."""
    T = token_catalog_id.shape[0]
    _check("lora_slot_lookup", load_library().lora_slot_lookup(
        site.handle, _dev_ptr(token_catalog_id, torch.int64), T, _dev_ptr(token_slot_out, torch.int32), _stream(stream)))


def lora_slots_evict(site, slot, stream=None):
    _check("lora_slots_evict", load_library().lora_slots_evict(site.handle, slot, _stream(stream)))


def lora_apply_decode(site, x, y, token_slot, stream=None):
    px, ldx = _rows(x)
    py, ldy = _rows(y)
    T = x.shape[0]
    assert y.shape[0] == T and token_slot.shape == (T,)
    _check("lora_apply_decode", load_library().lora_apply_decode(
        site.handle, px, ldx, py, ldy, _dev_ptr(token_slot, torch.int32), T, _stream(stream)))


def lora_apply_decode_noalloc(site, x, y, token_slot, stream=None):
    px, ldx = _rows(x)
    py, ldy = _rows(y)
    T = x.shape[0]
    assert y.shape[0] == T and token_slot.shape == (T,)
    _check("lora_apply_decode_noalloc", load_library().lora_apply_decode_noalloc(
        site.handle, px, ldx, py, ldy, _dev_ptr(token_slot, torch.int32), T, _stream(stream)))


def lora_apply_segmented(site, x, y, seg_off, seg_slot, stream=None):
    px, ldx = _rows(x)
    py, ldy = _rows(y)
    seg_off = np.ascontiguousarray(seg_off, dtype=np.int32)
    seg_slot = np.ascontiguousarray(seg_slot, dtype=np.int32)
    S = seg_slot.shape[0]
    assert seg_off.shape == (S + 1,)
    _check("lora_apply_segmented", load_library().lora_apply_segmented(
        site.handle, px, ldx, py, ldy, C.c_void_p(seg_off.ctypes.data), C.c_void_p(seg_slot.ctypes.data),
        S, x.shape[0], _stream(stream)))


def moe_lora_apply_packed(site, x, y, topk_ids, token_slot, out_sorted_pair=None, out_group_off=None, stream=None):
    px, ldx = _rows(x)
    py, ldy = _rows(y)
    T, K = topk_ids.shape
    assert topk_ids.is_contiguous() and x.shape[0] == T and y.shape[0] == T * K
    _check("moe_lora_apply_packed", load_library().moe_lora_apply_packed(
        site.handle, px, ldx, py, ldy, _dev_ptr(topk_ids, torch.int32), _dev_ptr(token_slot, torch.int32),
        T, K, _dev_ptr(out_sorted_pair, torch.int32), _dev_ptr(out_group_off, torch.int32), _stream(stream)))


def lora_plan_decode(plan, token_slot, n_slots, ready_from=None, stream=None):
    _check("lora_plan_decode", load_library().lora_plan_decode(
        plan.handle, _dev_ptr(token_slot, torch.int32), token_slot.shape[0], n_slots,
        ready_from.handle if ready_from is not None else None, _stream(stream)))


def lora_apply_decode_planned(site, plan, x, y, stream=None):
    px, ldx = _rows(x)
    py, ldy = _rows(y)
    _check("lora_apply_decode_planned", load_library().lora_apply_decode_planned(
        site.handle, plan.handle, px, ldx, py, ldy, _stream(stream)))


def _apply_multi(name, sites, plan, xs, ys, stream):
    n = len(sites)
    assert len(xs) == n and len(ys) == n
    rows = [(_rows(x), _rows(y)) for x, y in zip(xs, ys)]
    hs = (_vp * n)(*[s.handle for s in sites])
    px = (_vp * n)(*[r[0][0] for r in rows])
    lx = (_i64 * n)(*[r[0][1] for r in rows])
    py = (_vp * n)(*[r[1][0] for r in rows])
    ly = (_i64 * n)(*[r[1][1] for r in rows])
    _check(name, getattr(load_library(), name)(hs, n, plan.handle, px, lx, py, ly, _stream(stream)))


def lora_apply_decode_multi(sites, plan, xs, ys, stream=None):
    _apply_multi("lora_apply_decode_multi", sites, plan, xs, ys, stream)


def lora_plan_apply_decode_multi(sites, plan, token_slot, n_slots, xs, ys, ready_from=None, stream=None):
    n = len(sites)
    assert len(xs) == n and len(ys) == n
    rows = [(_rows(x), _rows(y)) for x, y in zip(xs, ys)]
    hs = (_vp * n)(*[s.handle for s in sites])
    px = (_vp * n)(*[r[0][0] for r in rows])
    lx = (_i64 * n)(*[r[0][1] for r in rows])
    py = (_vp * n)(*[r[1][0] for r in rows])
    ly = (_i64 * n)(*[r[1][1] for r in rows])
    _check("lora_plan_apply_decode_multi", load_library().lora_plan_apply_decode_multi(
        hs, n, plan.handle, _dev_ptr(token_slot, torch.int32), token_slot.shape[0], n_slots,
        ready_from.handle if ready_from is not None else None, px, lx, py, ly, _stream(stream)))


def moe_lora_apply_multi(sites, plan, xs, ys, stream=None):
    _apply_multi("moe_lora_apply_multi", sites, plan, xs, ys, stream)


def moe_plan_route(plan, topk_ids, token_slot, n_slots, n_experts, ready_from=None,
                   out_sorted_pair=None, out_group_off=None, stream=None):
    T, K = topk_ids.shape
    assert topk_ids.is_contiguous()
    _check("moe_plan_route", load_library().moe_plan_route(
        plan.handle, _dev_ptr(topk_ids, torch.int32), _dev_ptr(token_slot, torch.int32), T, K, n_slots, n_experts,
        ready_from.handle if ready_from is not None else None,
        _dev_ptr(out_sorted_pair, torch.int32), _dev_ptr(out_group_off, torch.int32), _stream(stream)))


def moe_lora_apply_planned(site, plan, x, y, stream=None):
    px, ldx = _rows(x)
    py, ldy = _rows(y)
    _check("moe_lora_apply_planned", load_library().moe_lora_apply_planned(
        site.handle, plan.handle, px, ldx, py, ldy, _stream(stream)))


def moe_down_workspace_bytes(T, K, d_out):
    n = _sz()
    _check("moe_down_workspace_bytes", load_library().moe_down_workspace_bytes(T, K, d_out, C.byref(n)))
    return n.value


def moe_lora_apply_down(site, plan, x, pair_w, token_slot, workspace, y, stream=None):
    """x [T*K, d_in] pair-major, pair_w fp32 [T, K], y [T, d_out]; workspace: a uint8 device tensor of
    moe_down_workspace_bytes(T, K, d_out) bytes."""
    px, ldx = _rows(x)
    py, ldy = _rows(y)
    assert pair_w.is_contiguous() and workspace.is_contiguous()
    _check("moe_lora_apply_down", load_library().moe_lora_apply_down(
        site.handle, plan.handle, px, ldx, _dev_ptr(pair_w, torch.float32), _dev_ptr(token_slot, torch.int32),
        C.c_void_p(workspace.data_ptr()), py, ldy, _stream(stream)))


class Resident:
    """Host-side map catalog id -> GPU slot with LRU eviction and bounded, deduplicated load jobs."""
    READY, LOAD, PENDING, QUEUED, REJECTED = range(5)
    STATS = ("hits", "loads", "shared", "rejects", "evictions")

    def __init__(self, n_slots, max_in_flight=1, max_queue=1):
        h = _vp()
        _check("mlora_resident_create", load_library().mlora_resident_create(n_slots, max_in_flight, max_queue, C.byref(h)))
        self.handle = h

    def close(self):
        if self.handle:
            load_library().mlora_resident_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def register(self, catalog_id):
        _check("mlora_resident_register", load_library().mlora_resident_register(self.handle, catalog_id))

    def lookup(self, catalog_id):
        return load_library().mlora_resident_lookup(self.handle, catalog_id)

    def request(self, catalog_id):
        """-> (result, slot, evicted_id)"""
        slot, ev = _i32(-1), _i64(-1)
        rc = load_library().mlora_resident_request(self.handle, catalog_id, C.byref(slot), C.byref(ev))
        if rc < 0:
            _check("mlora_resident_request", rc)
        return rc, slot.value, ev.value

    def complete(self, catalog_id, ok=True):
        """-> (next_id, next_slot, evicted_id) of the queued job that starts now, or (-1, -1, -1)"""
        nid, ns, ev = _i64(-1), _i32(-1), _i64(-1)
        _check("mlora_resident_complete", load_library().mlora_resident_complete(
            self.handle, catalog_id, 1 if ok else 0, C.byref(nid), C.byref(ns), C.byref(ev)))
        return nid.value, ns.value, ev.value

    def pin(self, slot, pinned=True):
        _check("mlora_resident_pin", load_library().mlora_resident_pin(self.handle, slot, 1 if pinned else 0))

    def stats(self):
        out = (_i64 * len(self.STATS))()
        _check("mlora_resident_stats", load_library().mlora_resident_stats(self.handle, out))
        return dict(zip(self.STATS, list(out)))
