"""ctypes binding of include/hat_mid.h -- argument marshalling only.

torch is used for device memory and streams (plumbing): tensors are allocated
by the caller or here with torch.empty, and their data pointers are handed to
the C ABI.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

HERE = os.path.dirname(os.path.abspath(__file__))

CHUNK, VERIFY = 0, 1
HAT_BF16, HAT_F32 = 0, 1
KV_DTYPES = {"bf16": 0, "f16": 1}
STATUS = {0: "HAT_OK", -1: "HAT_EINVAL", -2: "HAT_ENOMEM", -3: "HAT_EPOS", -4: "HAT_EDUP", -5: "HAT_EDEVICE",
          -6: "HAT_EHIP"}
KERNEL_NAMES = ["gather", "rmsnorm", "gemm_qkv", "rope_append", "attn_chunk", "attn_verify", "attn_merge",
                "gemm_o", "gemm_gateup", "gemm_down", "scatter"]
DUMP_IDS = {"xnorm": 0, "q": 1, "attn": 2, "xnorm2": 3, "act": 4}
EXPORTED_SYMBOLS = [
    "hat_mid_kv_bytes", "hat_mid_workspace_bytes", "hat_mid_create", "hat_mid_forward", "hat_mid_forward_host", "hat_mid_release",
    "hat_mid_destroy", "hat_mid_last_error", "hat_mid_kv_query", "hat_mid_kv_compact", "hat_mid_kv_import", "hat_mid_kv_export",
    "hat_mid_kv_export_static",
    "hat_mid_last_step_stats", "hat_mid_set_profiling", "hat_mid_kernel_times", "hat_mid_debug_dump", "hat_mid_debug_force_gemm",
    "hat_mid_debug_gemm_tile_count", "hat_mid_debug_gemm_tile_info", "hat_mid_debug_gemm_plan", "hat_mid_debug_create_host_only", "hat_mid_debug_plan",
    "hat_mid_debug_set_attn_targets", "hat_mid_debug_limit_plan", "hat_mid_debug_set_verify_probe", "hat_mid_debug_peak",
    "hat_sched_create", "hat_sched_destroy", "hat_sched_observe", "hat_sched_mu", "hat_sched_predict",
    "hat_sched_chunk_size", "hat_sched_parallel_draft_steps",
]


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ffn", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("page_size", C.c_int32),
                ("n_pages", C.c_int32), ("max_devices", C.c_int32), ("max_step_tokens", C.c_int32),
                ("max_pos", C.c_int32), ("io_dtype", C.c_int32), ("kv_dtype", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class CSegment(C.Structure):
    _fields_ = [("device_id", C.c_int32), ("kind", C.c_int32), ("n", C.c_int32), ("start_pos", C.c_int32),
                ("hidden_in", C.c_void_p), ("hidden_out", C.c_void_p), ("tree_mask", C.c_void_p)]


class HatError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("%s: %s" % (STATUS.get(code, code), msg))
        self.code = code


def lib_path():
    return os.path.join(HERE, "libhatmid.so")


_LIB = None


def load_library():
    """Loads the built library; raises if it is missing (there is no fallback)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    p = lib_path()
    if not os.path.exists(p):
        raise ImportError("libhatmid.so is not built: run `python -m paper_2503_18989_amd.build` "
                          "(hipcc, gfx950) first")
    lib = C.CDLL(p)
    vp, i32 = C.c_void_p, C.c_int32
    lib.hat_mid_kv_bytes.restype = C.c_size_t
    lib.hat_mid_kv_bytes.argtypes = [C.POINTER(Config)]
    lib.hat_mid_workspace_bytes.restype = C.c_size_t
    lib.hat_mid_workspace_bytes.argtypes = [C.POINTER(Config)]
    lib.hat_mid_create.restype = i32
    lib.hat_mid_create.argtypes = [C.POINTER(Config), C.POINTER(LayerWeights), vp, vp, vp, C.POINTER(vp)]
    lib.hat_mid_forward.restype = i32
    lib.hat_mid_forward.argtypes = [vp, C.POINTER(CSegment), i32, vp]
    lib.hat_mid_forward_host.restype = i32
    lib.hat_mid_forward_host.argtypes = [vp, C.POINTER(CSegment), i32, vp]
    lib.hat_mid_release.restype = i32
    lib.hat_mid_release.argtypes = [vp, i32]
    lib.hat_mid_destroy.restype = None
    lib.hat_mid_destroy.argtypes = [vp]
    lib.hat_mid_last_error.restype = C.c_char_p
    lib.hat_mid_last_error.argtypes = [vp]
    lib.hat_mid_kv_query.restype = i32
    lib.hat_mid_kv_query.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), i32, C.POINTER(i32)]
    lib.hat_mid_kv_compact.restype = i32
    lib.hat_mid_kv_compact.argtypes = [vp, i32, i32, C.POINTER(i32), i32, vp]
    lib.hat_mid_kv_import.restype = i32
    lib.hat_mid_kv_import.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
    lib.hat_mid_kv_export.restype = i32
    lib.hat_mid_kv_export.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
    lib.hat_mid_kv_export_static.restype = i32
    lib.hat_mid_kv_export_static.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
    lib.hat_mid_last_step_stats.restype = i32
    lib.hat_mid_last_step_stats.argtypes = [vp, C.POINTER(i32), C.POINTER(C.c_float)]
    lib.hat_mid_set_profiling.restype = i32
    lib.hat_mid_set_profiling.argtypes = [vp, i32]
    lib.hat_mid_kernel_times.restype = i32
    lib.hat_mid_kernel_times.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(i32)]
    lib.hat_mid_debug_dump.restype = i32
    lib.hat_mid_debug_dump.argtypes = [vp, i32, vp, vp]
    lib.hat_mid_debug_force_gemm.restype = i32
    lib.hat_mid_debug_force_gemm.argtypes = [vp, i32, i32, i32]
    lib.hat_mid_debug_gemm_tile_count.restype = i32
    lib.hat_mid_debug_gemm_tile_count.argtypes = []
    lib.hat_mid_debug_gemm_tile_info.restype = i32
    lib.hat_mid_debug_gemm_tile_info.argtypes = [i32] + [C.POINTER(i32)] * 5
    lib.hat_mid_debug_gemm_plan.restype = i32
    lib.hat_mid_debug_gemm_plan.argtypes = [i32, i32, i32, i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.hat_mid_debug_create_host_only.restype = i32
    lib.hat_mid_debug_create_host_only.argtypes = [C.POINTER(Config), C.POINTER(vp)]
    lib.hat_mid_debug_set_attn_targets.restype = i32
    lib.hat_mid_debug_set_attn_targets.argtypes = [vp, i32, i32]
    lib.hat_mid_debug_set_verify_probe.restype = i32
    lib.hat_mid_debug_set_verify_probe.argtypes = [vp, i32]
    lib.hat_mid_debug_peak.restype = i32
    lib.hat_mid_debug_peak.argtypes = [i32, vp, C.c_size_t, i32, vp, C.POINTER(C.c_double)]
    lib.hat_mid_debug_limit_plan.restype = i32
    lib.hat_mid_debug_limit_plan.argtypes = [vp, C.c_int64]
    pi = C.POINTER(i32)
    lib.hat_mid_debug_plan.restype = i32
    lib.hat_mid_debug_plan.argtypes = [vp, C.POINTER(CSegment), i32, pi, pi, i32, pi, pi, pi, pi, pi, pi, i32]
    f64 = C.c_double
    lib.hat_sched_create.restype = i32
    lib.hat_sched_create.argtypes = [C.POINTER(i32), i32, f64, C.POINTER(vp)]
    lib.hat_sched_destroy.restype = None
    lib.hat_sched_destroy.argtypes = [vp]
    lib.hat_sched_observe.restype = i32
    lib.hat_sched_observe.argtypes = [vp, f64, f64]
    lib.hat_sched_mu.restype = f64
    lib.hat_sched_mu.argtypes = [vp]
    lib.hat_sched_predict.restype = f64
    lib.hat_sched_predict.argtypes = [vp, f64]
    lib.hat_sched_chunk_size.restype = i32
    lib.hat_sched_chunk_size.argtypes = [vp, f64, f64, i32, i32, i32]
    lib.hat_sched_parallel_draft_steps.restype = i32
    lib.hat_sched_parallel_draft_steps.argtypes = [vp, f64, f64, f64, f64, f64]
    _LIB = lib
    return lib


@dataclass
class Segment:
    device_id: int
    kind: int
    start_pos: int
    hidden_in: "object"          # torch tensor [n, d] on the GPU
    hidden_out: "object" = None   # defaults to a fresh tensor
    tree_mask: "object" = None    # verify segments only: one visibility byte per row (a list of ints), or None


class HatMid:
    """hat_mid_create / hat_mid_forward / hat_mid_release and friends.

    cfg: dict with n_layers, d_model, n_heads, head_dim, d_ffn, rms_eps,
    rope_theta.  layers: list of dicts of bf16 CUDA tensors (names as in
    hat_mid_layer_weights_t).
    """

    def __init__(self, cfg, layers, n_pages, max_devices=64, max_step_tokens=8192, max_pos=16384,
                 io_dtype="bf16", kv_dtype="bf16", stream=None):
        import torch
        self.torch = torch
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2503_18989_amd needs a GPU: there is no CPU path")
        self.io_torch = torch.bfloat16 if io_dtype == "bf16" else torch.float32
        self.cfg = Config(cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ffn"],
                          cfg["rms_eps"], cfg["rope_theta"], 16, n_pages, max_devices, max_step_tokens, max_pos,
                          HAT_BF16 if io_dtype == "bf16" else HAT_F32, KV_DTYPES[kv_dtype])
        self.kv_dtype = kv_dtype
        self.d = cfg["d_model"]
        self.d_ffn = cfg["d_ffn"]
        self.n_heads, self.head_dim = cfg["n_heads"], cfg["head_dim"]
        kvb = self.lib.hat_mid_kv_bytes(C.byref(self.cfg))
        wsb = self.lib.hat_mid_workspace_bytes(C.byref(self.cfg))
        if kvb == 0 or wsb == 0:
            raise HatError(-1, "invalid configuration")
        self.kv_pool = torch.empty(kvb, dtype=torch.uint8, device="cuda")
        self.workspace = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        arr = (LayerWeights * cfg["n_layers"])()
        for l, w in enumerate(layers):
            for name, _ in LayerWeights._fields_:
                t = w[name]
                assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous(), name
                setattr(arr[l], name, t.data_ptr())
        self._handle = C.c_void_p()
        rc = self.lib.hat_mid_create(C.byref(self.cfg), arr, self.kv_pool.data_ptr(), self.workspace.data_ptr(),
                                     self._stream(stream), C.byref(self._handle))
        if rc != 0:
            raise HatError(rc, "hat_mid_create failed")
        torch.cuda.current_stream().synchronize() if stream is None else stream.synchronize()

    def _stream(self, stream=None):
        s = stream if stream is not None else self.torch.cuda.current_stream()
        return C.c_void_p(s.cuda_stream)

    def _check(self, rc):
        if rc != 0:
            raise HatError(rc, self.lib.hat_mid_last_error(self._handle).decode())

    @staticmethod
    def _mask_ptr(seg, keep):
        """Marshals a segment's tree mask into a byte array (kept alive in `keep` for the call)."""
        if seg.tree_mask is None:
            return None
        buf = (C.c_uint8 * len(seg.tree_mask))(*[int(m) for m in seg.tree_mask])
        keep.append(buf)
        return C.cast(buf, C.c_void_p)

    def forward(self, segments, stream=None):
        """segments: list of Segment.  Returns the list of output tensors."""
        torch = self.torch
        n = len(segments)
        arr = (CSegment * max(n, 1))()
        outs, keep = [], []
        for i, s in enumerate(segments):
            x = s.hidden_in
            assert x.is_cuda and x.dtype == self.io_torch and x.is_contiguous() and x.shape[1] == self.d
            out = s.hidden_out if s.hidden_out is not None else torch.empty_like(x)
            outs.append(out)
            arr[i] = CSegment(s.device_id, s.kind, x.shape[0], s.start_pos, x.data_ptr(), out.data_ptr(),
                              self._mask_ptr(s, keep))
        self._check(self.lib.hat_mid_forward(self._handle, arr, n, self._stream(stream)))
        return outs

    def forward_host(self, segments, stream=None):
        """segments: list of Segment whose hidden_in (and hidden_out, if given) are CPU tensors, pinned for
        overlap.  Returns the list of output CPU tensors, valid once the stream has been synchronised."""
        torch = self.torch
        n = len(segments)
        arr = (CSegment * max(n, 1))()
        outs, keep = [], []
        for i, s in enumerate(segments):
            x = s.hidden_in
            assert (not x.is_cuda) and x.dtype == self.io_torch and x.is_contiguous() and x.shape[1] == self.d
            out = s.hidden_out if s.hidden_out is not None else torch.empty_like(x, pin_memory=x.is_pinned())
            assert not out.is_cuda and out.is_contiguous()
            outs.append(out)
            arr[i] = CSegment(s.device_id, s.kind, x.shape[0], s.start_pos, x.data_ptr(), out.data_ptr(),
                              self._mask_ptr(s, keep))
        # the copies are asynchronous and two calls may be in flight (the upload of this one runs
        # while the previous step computes): hold the host tensors of the last two calls
        self._keep_host = (getattr(self, "_keep_host", [None, None]) + [(segments, outs)])[-2:]
        self._check(self.lib.hat_mid_forward_host(self._handle, arr, n, self._stream(stream)))
        return outs

    def forward_raw(self, arr, n, stream_ptr):
        """Pre-marshalled call for timing loops: arr = (CSegment * n)."""
        rc = self.lib.hat_mid_forward(self._handle, arr, n, stream_ptr)
        if rc != 0:
            self._check(rc)

    def release(self, device_id):
        self._check(self.lib.hat_mid_release(self._handle, device_id))

    def kv_compact(self, device_id, base_pos, keep, stream=None):
        arr = (C.c_int32 * max(len(keep), 1))(*[int(k) for k in keep])
        self._check(self.lib.hat_mid_kv_compact(self._handle, device_id, base_pos, arr, len(keep), self._stream(stream)))

    def kv_query(self, device_id, cap=1 << 16):
        ln, npg = C.c_int32(), C.c_int32()
        buf = (C.c_int32 * cap)()
        self._check(self.lib.hat_mid_kv_query(self._handle, device_id, C.byref(ln), buf, cap, C.byref(npg)))
        return ln.value, list(buf[: npg.value])

    def kv_import(self, device_id, layer, pos0, k, v, stream=None):
        assert k.is_cuda and k.dtype == self.torch.bfloat16 and k.is_contiguous() and k.shape == v.shape
        assert tuple(k.shape[1:]) == (self.n_heads, self.head_dim)
        self._check(self.lib.hat_mid_kv_import(self._handle, device_id, layer, pos0, k.shape[0], k.data_ptr(),
                                               v.data_ptr(), self._stream(stream)))

    def kv_export(self, device_id, layer, pos0, n, stream=None):
        torch = self.torch
        k = torch.empty((n, self.n_heads, self.head_dim), dtype=torch.bfloat16, device="cuda")
        v = torch.empty_like(k)
        self._check(self.lib.hat_mid_kv_export(self._handle, device_id, layer, pos0, n, k.data_ptr(), v.data_ptr(),
                                               self._stream(stream)))
        return k, v

    def kv_export_static(self, device_id, layer, pos0, n, k, v, stream=None):
        """hat_mid_kv_export_static into the caller's k, v ([n, n_heads, head_dim] bf16 CUDA tensors): the
        call itself allocates nothing and does not wait for the stream."""
        assert k.is_cuda and k.dtype == self.torch.bfloat16 and k.is_contiguous() and k.shape == v.shape
        assert tuple(k.shape) == (n, self.n_heads, self.head_dim) and v.is_contiguous()
        self._check(self.lib.hat_mid_kv_export_static(self._handle, device_id, layer, pos0, n, k.data_ptr(),
                                                      v.data_ptr(), self._stream(stream)))

    def last_step_stats(self):
        tok, ms = C.c_int32(), C.c_float()
        self._check(self.lib.hat_mid_last_step_stats(self._handle, C.byref(tok), C.byref(ms)))
        return tok.value, ms.value

    def set_profiling(self, on):
        self._check(self.lib.hat_mid_set_profiling(self._handle, 1 if on else 0))

    def kernel_times(self):
        ms = (C.c_float * len(KERNEL_NAMES))()
        cnt = (C.c_int32 * len(KERNEL_NAMES))()
        self._check(self.lib.hat_mid_kernel_times(self._handle, ms, cnt))
        return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_NAMES)}

    def debug_dump(self, which, T, stream=None):
        torch = self.torch
        cols = self.d_ffn if which == "act" else self.d
        out = torch.empty((T, cols), dtype=torch.float32, device="cuda")
        self._check(self.lib.hat_mid_debug_dump(self._handle, DUMP_IDS[which], out.data_ptr(), self._stream(stream)))
        return out

    def force_gemm(self, which, tile, ksplit=1):
        self._check(self.lib.hat_mid_debug_force_gemm(self._handle, which, tile, ksplit))

    def gemm_tile_count(self):
        return int(self.lib.hat_mid_debug_gemm_tile_count())

    def set_attn_targets(self, chunk_target=0, verify_target=0):
        self._check(self.lib.hat_mid_debug_set_attn_targets(self._handle, chunk_target, verify_target))

    def set_verify_probe(self, on):
        """Measurement aid: verify attention replaced by its loads only -- outputs become meaningless."""
        self._check(self.lib.hat_mid_debug_set_verify_probe(self._handle, 1 if on else 0))

    def close(self):
        if getattr(self, "_handle", None) is not None and self._handle.value:
            self.lib.hat_mid_destroy(self._handle)
            self._handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


PEAK_KINDS = {"stream_read": 0, "stream_read_nt": 1, "copy": 2, "mfma_f16": 3, "lds_load": 4}


def measure_peak(kind, nbytes=1 << 30, iters=20):
    """hat_mid_debug_peak on a scratch tensor of nbytes: bytes/s or FLOP/s (see include/hat_mid.h)."""
    import torch
    lib = load_library()
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    buf.zero_()
    rate = C.c_double()
    rc = lib.hat_mid_debug_peak(PEAK_KINDS[kind], buf.data_ptr(), nbytes, iters,
                                C.c_void_p(torch.cuda.current_stream().cuda_stream), C.byref(rate))
    if rc != 0:
        raise HatError(rc, "hat_mid_debug_peak(%s) failed" % kind)
    return rate.value


class HatPlanner:
    """The host half of the library on its own (hat_mid_debug_create_host_only / hat_mid_debug_plan): validation,
    page bookkeeping and the per-step plan, without a GPU.  For tests of the host logic."""

    ATTN_FIELDS = ("seg", "q0", "nq", "kv_begin", "kv_end", "part_row", "start", "tok0", "kv_len", "pt_off", "vis_lo", "vis_hi")
    MERGE_FIELDS = ("row0", "nrows", "part_row", "nsplit", "stride")

    def __init__(self, cfg, n_pages, max_devices=64, max_step_tokens=8192, max_pos=16384):
        self.lib = load_library()
        self.max_step_tokens = max_step_tokens
        self.ccfg = Config(cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ffn"],
                           cfg["rms_eps"], cfg["rope_theta"], 16, n_pages, max_devices, max_step_tokens, max_pos, HAT_BF16, 0)
        self._handle = C.c_void_p()
        rc = self.lib.hat_mid_debug_create_host_only(C.byref(self.ccfg), C.byref(self._handle))
        if rc != 0:
            raise HatError(rc, "hat_mid_debug_create_host_only failed")

    def _check(self, rc):
        if rc != 0:
            raise HatError(rc, self.lib.hat_mid_last_error(self._handle).decode())

    def plan(self, segments, cap_items=4096):
        """segments: list of (device, kind, start, n) or (device, kind, start, n, tree masks).  Returns a dict with
        pos, kv_dst (lists) and chunk_items / verify_items / merge_items (lists of dicts)."""
        n = len(segments)
        arr = (CSegment * max(n, 1))()
        keep = []
        rows = 0
        for i, sg in enumerate(segments):
            mask = None
            if len(sg) > 4 and sg[4] is not None:
                buf = (C.c_uint8 * len(sg[4]))(*[int(m) for m in sg[4]])
                keep.append(buf)
                mask = C.cast(buf, C.c_void_p)
            arr[i] = CSegment(sg[0], sg[1], sg[3], sg[2], 1, 1, mask)   # hidden pointers: non-null placeholders
            rows += max(int(sg[3]), 0)
        cap_rows = max(rows, 1)
        i32 = C.c_int32
        pos, dst = (i32 * cap_rows)(), (i32 * cap_rows)()
        ci, vi, mi = (i32 * (12 * cap_items))(), (i32 * (12 * cap_items))(), (i32 * (8 * cap_items))()
        nc, nv, nm = i32(), i32(), i32()
        self._check(self.lib.hat_mid_debug_plan(self._handle, arr, n, pos, dst, cap_rows, ci, C.byref(nc), vi, C.byref(nv),
                                                mi, C.byref(nm), cap_items))
        u32 = lambda x: x & 0xFFFFFFFF
        items = lambda raw, cnt: [dict(zip(self.ATTN_FIELDS, [raw[12 * k + j] if j < 10 else u32(raw[12 * k + j]) for j in range(12)]))
                                  for k in range(cnt)]
        merges = [dict(zip(self.MERGE_FIELDS, [mi[8 * k + j] for j in range(5)])) for k in range(nm.value)]
        return dict(pos=list(pos[:rows]), kv_dst=list(dst[:rows]), chunk_items=items(ci, nc.value),
                    verify_items=items(vi, nv.value), merge_items=merges)

    def release(self, device_id):
        self._check(self.lib.hat_mid_release(self._handle, device_id))

    def limit_plan(self, max_words):
        self._check(self.lib.hat_mid_debug_limit_plan(self._handle, int(max_words)))

    def set_attn_targets(self, chunk_target=0, verify_target=0):
        self._check(self.lib.hat_mid_debug_set_attn_targets(self._handle, chunk_target, verify_target))

    def kv_compact(self, device_id, base_pos, keep):
        arr = (C.c_int32 * max(len(keep), 1))(*[int(k) for k in keep])
        self._check(self.lib.hat_mid_kv_compact(self._handle, device_id, base_pos, arr, len(keep), None))

    def kv_query(self, device_id, cap=1 << 16):
        ln, npg = C.c_int32(), C.c_int32()
        buf = (C.c_int32 * cap)()
        self._check(self.lib.hat_mid_kv_query(self._handle, device_id, C.byref(ln), buf, cap, C.byref(npg)))
        return ln.value, list(buf[: npg.value])

    def close(self):
        if getattr(self, "_handle", None) is not None and self._handle.value:
            self.lib.hat_mid_destroy(self._handle)
            self._handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class HatSched:
    """hat_sched_*: state monitor (Sec. 3.2) and chunk-size rule (Sec. 3.3) of the cloud.  Host code; needs no GPU."""

    def __init__(self, knots, alpha=0.8):
        self.lib = load_library()
        arr = (C.c_int32 * len(knots))(*[int(k) for k in knots])
        self._handle = C.c_void_p()
        if self.lib.hat_sched_create(arr, len(knots), float(alpha), C.byref(self._handle)) != 0:
            raise ValueError("hat_sched_create: invalid knots or alpha")

    def observe(self, mu_hat, eta_hat):
        if self.lib.hat_sched_observe(self._handle, float(mu_hat), float(eta_hat)) != 0:
            raise ValueError("hat_sched_observe: invalid sample")

    @property
    def mu(self):
        return self.lib.hat_sched_mu(self._handle)

    def predict(self, tokens):
        return self.lib.hat_sched_predict(self._handle, float(tokens))

    def chunk_size(self, bytes_per_token, beta_up, pipeline_len, x_min, x_max):
        x = self.lib.hat_sched_chunk_size(self._handle, float(bytes_per_token), float(beta_up), int(pipeline_len),
                                          int(x_min), int(x_max))
        if x < 0:
            raise ValueError("hat_sched_chunk_size: invalid argument")
        return x

    def parallel_draft_steps(self, draft_len, bytes_per_token, beta_up, beta_down, gamma):
        n = self.lib.hat_sched_parallel_draft_steps(self._handle, float(draft_len), float(bytes_per_token),
                                                    float(beta_up), float(beta_down), float(gamma))
        if n < 0:
            raise ValueError("hat_sched_parallel_draft_steps: invalid argument")
        return n

    def close(self):
        if getattr(self, "_handle", None) is not None and self._handle.value:
            self.lib.hat_sched_destroy(self._handle)
            self._handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
