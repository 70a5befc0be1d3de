"""Thin ctypes binding of libhfxattn's C ABI (include/hfxattn.h).

Argument marshalling only: every step of the path runs inside the library's HIP kernels.
PyTorch appears here solely as the owner of device memory and streams.  There is no CPU
fallback: if the library has not been built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhfxattn.so")

HFX_OK = 0
HFX_ERR_NULL, HFX_ERR_SHAPE, HFX_ERR_KIND, HFX_ERR_LEN, HFX_ERR_PAGES = -1, -2, -3, -4, -5
HFX_ERR_PAGE_ID, HFX_ERR_BUFSIZE, HFX_ERR_DEVICE, HFX_ERR_DESC, HFX_ERR_ALIGN = -6, -7, -8, -9, -10
HFX_ERR_MODEL = -11
HFX_DECODE, HFX_PREFILL = 0, 1

EXPORTS = ["hfx_status_string", "hfx_version", "hfx_batch_desc_sizes", "hfx_build_batch_desc",
           "hfx_fill_batch_desc", "hfx_mixed_paged_attention", "hfx_mixed_paged_attention_static", "hfx_gather_kv", "hfx_append_kv",
           "hfx_copy_pages", "hfx_token_budget", "hfx_maturity_time", "hfx_fit_latency_model", "hfx_compose_step"]


class hfx_shape(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_pages", ctypes.c_int32), ("softmax_scale", ctypes.c_float)]


class hfx_latency_model(ctypes.Structure):
    _fields_ = [("a", ctypes.c_double), ("b", ctypes.c_double), ("e_d", ctypes.c_double)]


class hfx_decision(ctypes.Structure):
    _fields_ = [("budget", ctypes.c_int64), ("n_token", ctypes.c_int64), ("e_p", ctypes.c_double),
                ("k", ctypes.c_double), ("maturity", ctypes.c_double)]


class HfxError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {hfx_status_string(code)} ({code})")


_lib = None


def load() -> ctypes.CDLL:
    """Loads the built library; raises if it is missing (build it with paper_2508_15919_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2508_15919_amd.build` "
                               "(hipcc, gfx950).  There is no fallback path.")
        lib = ctypes.CDLL(LIB_PATH)
        i32p = ctypes.POINTER(ctypes.c_int32)
        szp = ctypes.POINTER(ctypes.c_size_t)
        shp = ctypes.POINTER(hfx_shape)
        vp = ctypes.c_void_p
        lib.hfx_status_string.argtypes = [ctypes.c_int32]
        lib.hfx_status_string.restype = ctypes.c_char_p
        lib.hfx_version.argtypes = [i32p, i32p]
        lib.hfx_version.restype = ctypes.c_int32
        lib.hfx_batch_desc_sizes.argtypes = [shp, ctypes.c_int32, i32p, i32p, i32p, szp, szp, szp]
        lib.hfx_batch_desc_sizes.restype = ctypes.c_int32
        lib.hfx_fill_batch_desc.argtypes = [shp, ctypes.c_int32, i32p, i32p, i32p, i32p, i32p, vp, ctypes.c_size_t]
        lib.hfx_fill_batch_desc.restype = ctypes.c_int32
        lib.hfx_build_batch_desc.argtypes = [shp, ctypes.c_int32, i32p, i32p, i32p, i32p, i32p, vp,
                                             ctypes.c_size_t, vp, ctypes.c_size_t, vp]
        lib.hfx_build_batch_desc.restype = ctypes.c_int32
        lib.hfx_mixed_paged_attention.argtypes = [shp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp]
        lib.hfx_mixed_paged_attention.restype = ctypes.c_int32
        lib.hfx_mixed_paged_attention_static.argtypes = [shp, vp, vp, vp, vp, vp, vp]
        lib.hfx_mixed_paged_attention_static.restype = ctypes.c_int32
        lib.hfx_gather_kv.argtypes = [shp, vp, vp, vp, ctypes.c_int32, vp, vp, vp]
        lib.hfx_gather_kv.restype = ctypes.c_int32
        lib.hfx_append_kv.argtypes = [shp, vp, vp, vp, vp, vp, vp]
        lib.hfx_append_kv.restype = ctypes.c_int32
        lib.hfx_copy_pages.argtypes = [shp, vp, vp, ctypes.c_int32, ctypes.c_int32, i32p, i32p, vp, vp,
                                       ctypes.c_size_t, vp]
        lib.hfx_copy_pages.restype = ctypes.c_int32
        dbl, dblp = ctypes.c_double, ctypes.POINTER(ctypes.c_double)
        i64p, lmp = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(hfx_latency_model)
        lib.hfx_token_budget.argtypes = [dbl, dbl, lmp, i64p]
        lib.hfx_token_budget.restype = ctypes.c_int32
        lib.hfx_maturity_time.argtypes = [dbl, dbl, dbl, dblp, dblp]
        lib.hfx_maturity_time.restype = ctypes.c_int32
        lib.hfx_fit_latency_model.argtypes = [ctypes.c_int32, i64p, dblp, lmp, dblp]
        lib.hfx_fit_latency_model.restype = ctypes.c_int32
        lib.hfx_compose_step.argtypes = [dbl, dbl, lmp, ctypes.c_int32, i32p, ctypes.c_int32, i32p, dblp,
                                         ctypes.c_int32, i32p, i32p, i32p, i32p, i32p,
                                         ctypes.POINTER(hfx_decision)]
        lib.hfx_compose_step.restype = ctypes.c_int32
        _lib = lib
    return _lib


def _i32(a):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _ptr(x):
    """Raw address of a torch tensor, numpy array, int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    if hasattr(x, "data_ptr"):
        return ctypes.c_void_p(x.data_ptr())
    if isinstance(x, np.ndarray):
        return ctypes.c_void_p(x.ctypes.data)
    raise TypeError(f"cannot take the address of {type(x)}")


def _nbytes(x) -> int:
    if x is None:
        return 0
    if hasattr(x, "element_size"):
        return x.numel() * x.element_size()
    return int(x.nbytes)


def _stream(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def make_shape(num_q_heads, num_kv_heads, head_dim, num_pages, softmax_scale=0.0, page_size=16) -> hfx_shape:
    return hfx_shape(int(num_q_heads), int(num_kv_heads), int(head_dim), int(page_size), int(num_pages),
                     float(softmax_scale))


def hfx_status_string(code: int) -> str:
    return load().hfx_status_string(int(code)).decode()


def hfx_version():
    a, b = ctypes.c_int32(), ctypes.c_int32()
    load().hfx_version(ctypes.byref(a), ctypes.byref(b))
    return a.value, b.value


def hfx_batch_desc_sizes(shape: hfx_shape, kind, q_len, ctx_len):
    """Returns (host_desc_bytes, device_desc_bytes, device_workspace_bytes)."""
    k, pk = _i32(kind)
    q, pq = _i32(q_len)
    c, pc = _i32(ctx_len)
    h, d, w = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    rc = load().hfx_batch_desc_sizes(ctypes.byref(shape), len(k), pk, pq, pc, ctypes.byref(h), ctypes.byref(d),
                                     ctypes.byref(w))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_batch_desc_sizes")
    return h.value, d.value, w.value


def hfx_fill_batch_desc(shape: hfx_shape, kind, q_len, ctx_len, bt_indptr, bt_pages, host_desc) -> None:
    k, pk = _i32(kind)
    q, pq = _i32(q_len)
    c, pc = _i32(ctx_len)
    bi, pbi = _i32(bt_indptr)
    bp, pbp = _i32(bt_pages)
    rc = load().hfx_fill_batch_desc(ctypes.byref(shape), len(k), pk, pq, pc, pbi, pbp, _ptr(host_desc),
                                    _nbytes(host_desc))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_fill_batch_desc")


def hfx_build_batch_desc(shape: hfx_shape, kind, q_len, ctx_len, bt_indptr, bt_pages, host_desc, device_desc,
                         stream=None) -> None:
    k, pk = _i32(kind)
    q, pq = _i32(q_len)
    c, pc = _i32(ctx_len)
    bi, pbi = _i32(bt_indptr)
    bp, pbp = _i32(bt_pages)
    rc = load().hfx_build_batch_desc(ctypes.byref(shape), len(k), pk, pq, pc, pbi, pbp, _ptr(host_desc),
                                     _nbytes(host_desc), _ptr(device_desc), _nbytes(device_desc), _stream(stream))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_build_batch_desc")


def hfx_mixed_paged_attention(shape: hfx_shape, q, kv_pool, host_desc, device_desc, workspace, out,
                              stream=None) -> None:
    rc = load().hfx_mixed_paged_attention(ctypes.byref(shape), _ptr(q), _ptr(kv_pool), _ptr(host_desc),
                                          _ptr(device_desc), _ptr(workspace), _nbytes(workspace), _ptr(out),
                                          _stream(stream))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_mixed_paged_attention")


def hfx_mixed_paged_attention_static(shape: hfx_shape, q, kv_pool, host_desc, device_desc, out, stream=None) -> None:
    rc = load().hfx_mixed_paged_attention_static(ctypes.byref(shape), _ptr(q), _ptr(kv_pool), _ptr(host_desc),
                                                 _ptr(device_desc), _ptr(out), _stream(stream))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_mixed_paged_attention_static")


def hfx_gather_kv(shape: hfx_shape, kv_pool, host_desc, device_desc, request: int, k_out, v_out,
                  stream=None) -> None:
    rc = load().hfx_gather_kv(ctypes.byref(shape), _ptr(kv_pool), _ptr(host_desc), _ptr(device_desc),
                              int(request), _ptr(k_out), _ptr(v_out), _stream(stream))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_gather_kv")


def hfx_append_kv(shape: hfx_shape, k_new, v_new, kv_pool, host_desc, device_desc, stream=None) -> None:
    rc = load().hfx_append_kv(ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(kv_pool), _ptr(host_desc),
                              _ptr(device_desc), _stream(stream))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_append_kv")


def hfx_copy_pages(shape: hfx_shape, src_pool, dst_pool, dst_num_pages: int, src_ids, dst_ids, host_stage,
                   device_stage, stream=None, stage_bytes=None) -> None:
    s_arr, ps = _i32(np.asarray(src_ids, dtype=np.int32))
    d_arr, pd = _i32(np.asarray(dst_ids, dtype=np.int32))
    assert len(s_arr) == len(d_arr)
    rc = load().hfx_copy_pages(ctypes.byref(shape), _ptr(src_pool), _ptr(dst_pool), int(dst_num_pages), len(s_arr),
                               ps, pd, _ptr(host_stage), _ptr(device_stage),
                               min(_nbytes(host_stage), _nbytes(device_stage)) if stage_bytes is None
                               else int(stage_bytes), _stream(stream))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_copy_pages")


def hfx_token_budget(ttft: float, tpot: float, model: hfx_latency_model) -> int:
    n = ctypes.c_int64(-1)
    rc = load().hfx_token_budget(ttft, tpot, ctypes.byref(model), ctypes.byref(n))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_token_budget")
    return int(n.value)


def hfx_maturity_time(e_p: float, tpot: float, e_d: float):
    k, m = ctypes.c_double(), ctypes.c_double()
    rc = load().hfx_maturity_time(e_p, tpot, e_d, ctypes.byref(k), ctypes.byref(m))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_maturity_time")
    return k.value, m.value


def hfx_fit_latency_model(n_token, seconds, e_d: float = 0.0):
    """Returns (model, r_squared)."""
    n = np.ascontiguousarray(n_token, dtype=np.int64)
    t = np.ascontiguousarray(seconds, dtype=np.float64)
    assert n.shape == t.shape and n.ndim == 1
    model, r2 = hfx_latency_model(0.0, 0.0, e_d), ctypes.c_double()
    rc = load().hfx_fit_latency_model(len(n), n.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                      t.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), ctypes.byref(model),
                                      ctypes.byref(r2))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_fit_latency_model")
    return model, r2.value


def hfx_compose_step(ttft: float, tpot: float, model: hfx_latency_model, running_ctx, prompt_len, urgency=None,
                     mixed: bool = False):
    """Returns (admitted flags, kind, q_len, ctx_len, hfx_decision)."""
    rc_arr, prc = _i32(np.asarray(running_ctx, dtype=np.int32))
    pl_arr, ppl = _i32(np.asarray(prompt_len, dtype=np.int32))
    urg = purg = None
    if urgency is not None:
        urg = np.ascontiguousarray(urgency, dtype=np.float64)
        purg = urg.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    cap = max(1, len(rc_arr) + len(pl_arr))
    i32p = ctypes.POINTER(ctypes.c_int32)
    adm = np.zeros(max(1, len(pl_arr)), np.int32)
    kind, ql, cl = (np.zeros(cap, np.int32) for _ in range(3))
    n_step, dec = ctypes.c_int32(), hfx_decision()
    rc = load().hfx_compose_step(ttft, tpot, ctypes.byref(model), len(rc_arr), prc, len(pl_arr), ppl, purg,
                                 int(bool(mixed)), adm.ctypes.data_as(i32p), kind.ctypes.data_as(i32p),
                                 ql.ctypes.data_as(i32p), cl.ctypes.data_as(i32p), ctypes.byref(n_step),
                                 ctypes.byref(dec))
    if rc != HFX_OK:
        raise HfxError(rc, "hfx_compose_step")
    n = n_step.value
    return adm[:len(pl_arr)], kind[:n], ql[:n], cl[:n], dec


# ------------------------------------------------------------------------------------------
# Read-only views of a descriptor blob, for inspection and for the planner's CPU tests.
# They mirror csrc/hfx_desc.h.
# ------------------------------------------------------------------------------------------
class DescHeader(ctypes.Structure):
    _fields_ = [("magic", ctypes.c_uint32), ("version", ctypes.c_uint32),
                ("num_requests", ctypes.c_int32), ("total_q", ctypes.c_int32),
                ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("page_size", ctypes.c_int32), ("num_pages", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("n_items", ctypes.c_int32), ("n_decode_items", ctypes.c_int32),
                ("n_prefill_items", ctypes.c_int32), ("n_groups", ctypes.c_int32),
                ("n_partial_rows", ctypes.c_int32), ("n_bt", ctypes.c_int32),
                ("off_ctrl", ctypes.c_uint32), ("off_req", ctypes.c_uint32), ("off_bt", ctypes.c_uint32),
                ("off_items", ctypes.c_uint32), ("off_groups", ctypes.c_uint32), ("n_ctrl", ctypes.c_uint32),
                ("total_bytes", ctypes.c_uint64), ("workspace_bytes", ctypes.c_uint64),
                ("ws_off_ml", ctypes.c_uint64), ("max_group_rows", ctypes.c_int32),
                ("n_units", ctypes.c_int32), ("off_units", ctypes.c_uint32), ("n_runs", ctypes.c_int32),
                ("off_runs", ctypes.c_uint32), ("queue_classes", ctypes.c_uint32), ("reserved", ctypes.c_uint32 * 2)]


ITEM_DTYPE = np.dtype([(n, np.int32) for n in ("type", "req", "group", "slot_row", "h0", "hn", "row0", "nrows",
                                               "kb", "ke", "cost", "home", "rq_kind", "rq_q_len", "rq_ctx_len",
                                               "rq_q_start", "rq_bt_start", "rq_n_pages", "rq_bt_len", "rq_pad1")])
REQ_DTYPE = np.dtype([(n, np.int32) for n in ("kind", "q_len", "ctx_len", "q_start", "bt_start", "n_pages",
                                              "bt_len", "pad1")])
GROUP_DTYPE = np.dtype([(n, np.int32) for n in ("nsplit", "base_row", "rows_per_split", "type", "req", "h0", "hn",
                                                "row0", "q_start", "q_len")])


def parse_desc(host_desc: np.ndarray) -> dict:
    """Decodes a host descriptor blob (uint8 numpy array) into header, requests, block table, items, groups."""
    buf = np.ascontiguousarray(host_desc).view(np.uint8)
    h = DescHeader.from_buffer_copy(buf[:ctypes.sizeof(DescHeader)].tobytes())
    return {
        "header": h,
        "ctrl": buf[h.off_ctrl:h.off_ctrl + 4 * h.n_ctrl].view(np.int32),
        "reqs": buf[h.off_req:h.off_req + REQ_DTYPE.itemsize * h.num_requests].view(REQ_DTYPE),
        "bt": buf[h.off_bt:h.off_bt + 4 * h.n_bt].view(np.int32),
        "items": buf[h.off_items:h.off_items + ITEM_DTYPE.itemsize * h.n_items].view(ITEM_DTYPE),
        "groups": buf[h.off_groups:h.off_groups + GROUP_DTYPE.itemsize * h.n_groups].view(GROUP_DTYPE),
        "units": buf[h.off_units:h.off_units + 8 * h.n_units].view(np.int32).reshape(-1, 2),
        # append runs: (first packed row, tokens, physical page, first slot)
        "runs": buf[h.off_runs:h.off_runs + 16 * h.n_runs].view(np.int32).reshape(-1, 4),
    }


# ------------------------------------------------------------------------------------------
# Device-memory plumbing for callers that hold a step as numpy arrays (tests, bench, smoke).
# ------------------------------------------------------------------------------------------
class DeviceStep:
    """Owns the torch buffers of one step (descriptor: pinned host + device; workspace; Q; out) and the
    marshalled arguments of the two calls, so that build() and run() are one ctypes call each."""

    def __init__(self, batch, pool_dev=None, device="cuda:0", softmax_scale=0.0, stream=None):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.batch = batch
        self.shape = make_shape(batch.num_q_heads, batch.num_kv_heads, batch.head_dim, batch.num_pages,
                                softmax_scale)
        hb, db, wb = hfx_batch_desc_sizes(self.shape, batch.kind, batch.q_len, batch.ctx_len)
        self.host_desc = torch.empty(hb, dtype=torch.uint8, pin_memory=True)
        self.device_desc = torch.empty(db, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(max(wb, 16), dtype=torch.uint8, device=self.device)
        self.workspace_bytes = wb
        self._pool = pool_dev if pool_dev is not None else torch.from_numpy(batch.pool.view(np.int16)).to(self.device)
        self.q = torch.from_numpy(batch.q.view(np.int16)).to(self.device)
        self.out = torch.full_like(self.q, 0x7FC0)      # bf16 NaN: a row no kernel writes shows up in any compare
        self._lib = load()
        self._keep = [_i32(a) for a in (batch.kind, batch.q_len, batch.ctx_len, batch.bt_indptr, batch.bt_pages)]
        self._build_args = (ctypes.byref(self.shape), len(self._keep[0][0]), *(p for _, p in self._keep),
                            _ptr(self.host_desc), _nbytes(self.host_desc), _ptr(self.device_desc),
                            _nbytes(self.device_desc))
        self._set_run_args()
        self.build(stream)

    def _set_run_args(self):
        self._run_args = (ctypes.byref(self.shape), _ptr(self.q), _ptr(self._pool), _ptr(self.host_desc),
                          _ptr(self.device_desc), _ptr(self.workspace) if self.workspace_bytes else None,
                          self.workspace_bytes, _ptr(self.out))

    @property
    def pool(self):
        return self._pool

    @pool.setter
    def pool(self, value):
        self._pool = value
        self._set_run_args()

    def _stream_ptr(self, stream):
        if stream is None:
            stream = self.torch.cuda.current_stream(self.device)
        return ctypes.c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)

    def build(self, stream=None):
        """hfx_build_batch_desc: plan the step on the host and enqueue the descriptor upload."""
        rc = self._lib.hfx_build_batch_desc(*self._build_args, self._stream_ptr(stream))
        if rc != HFX_OK:
            raise HfxError(rc, "hfx_build_batch_desc")

    def run(self, stream=None):
        """hfx_mixed_paged_attention on the step's buffers."""
        rc = self._lib.hfx_mixed_paged_attention(*self._run_args, self._stream_ptr(stream))
        if rc != HFX_OK:
            raise HfxError(rc, "hfx_mixed_paged_attention")
        return self.out

    def append(self, k_new, v_new, stream=None):
        """hfx_append_kv: the chunk tokens' K/V ([T, Hkv, D] device tensors) go into the step's pages."""
        rc = self._lib.hfx_append_kv(ctypes.byref(self.shape), _ptr(k_new), _ptr(v_new), _ptr(self._pool),
                                     _ptr(self.host_desc), _ptr(self.device_desc), self._stream_ptr(stream))
        if rc != HFX_OK:
            raise HfxError(rc, "hfx_append_kv")

    def out_bits(self) -> np.ndarray:
        self.torch.cuda.synchronize(self.device)
        return self.out.cpu().numpy().view(np.uint16)

    def gather(self, request: int):
        t = self.torch
        c = int(self.batch.ctx_len[request])
        k = t.zeros((c, self.batch.num_kv_heads, self.batch.head_dim), dtype=t.int16, device=self.device)
        v = t.zeros_like(k)
        hfx_gather_kv(self.shape, self._pool, self.host_desc, self.device_desc, request, k, v,
                      t.cuda.current_stream(self.device))
        t.cuda.synchronize(self.device)
        return k.cpu().numpy().view(np.uint16), v.cpu().numpy().view(np.uint16)
