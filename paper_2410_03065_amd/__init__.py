"""Thin ctypes binding over libcake.so (the C ABI declared in include/cake.h).

Argument marshalling only: every step of the path (embedding, norms, GEMMs,
rotary, page writes, attention, throttled loads, planning, the race) runs
inside the library.  PyTorch is used to own device / pinned memory and the two
HIP streams.  If the library has not been built, importing succeeds but any use
raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcake.so")
_lib = None

OK, E_INVAL, E_NOMEM, E_HIP, E_STORE_MISS, E_STATE, E_CAPACITY = 0, -1, -2, -3, -4, -5, -6
F32, BF16 = 0, 1
MODES = {"bidir": 0, "compute_only": 1, "load_only": 2, "forced": 3, "greedy": 4}
SRC_COMPUTE, SRC_LOAD = 0, 1

EXPORTS = [
    "cake_create", "cake_destroy", "cake_last_error", "cake_set_tuning", "cake_prefill_chunk",
    "cake_load_chunk", "cake_plan_meet_point", "cake_bidirectional_prefill", "cake_set_bandwidth",
    "cake_schedule_bandwidth_step", "cake_chunk_state", "cake_sync_compute", "cake_sync_load",
    "cake_range_flops", "cake_page_image_bytes", "cake_simulate_race", "cake_op_rmsnorm",
    "cake_op_gemm", "cake_op_gemm_residual", "cake_op_gemm_swiglu", "cake_op_gemm_plan", "cake_op_mfma_rate", "cake_device_info", "cake_op_rope_kv_write",
    "cake_op_attention", "cake_profile_enable", "cake_profile_read", "cake_adaptive_serve", "cake_first_token",
    "cake_op_decode_attention", "cake_op_decode_attention_static", "cake_set_traces", "cake_store_image_bytes", "cake_write_store", "cake_prefix_keys", "cake_prefix_lookup",
]
STORE_RAW, STORE_INT8, STORE_INT4 = 0, 1, 2
STORE_PINNED, STORE_FILE = 0, 1
KERNEL_CLASSES = ["embed", "rmsnorm", "gemm_qkv", "rope_kv", "attention", "gemm_o", "gemm_gateup", "gemm_down",
                  "gemv", "decode_attention"]


class CakeError(RuntimeError):
    def __init__(self, code, msg=""):
        super().__init__("cake status %d: %s" % (code, msg))
        self.code = code


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                          "ffn_dim", "vocab", "dtype")] + [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("layers", C.POINTER(LayerWeights)), ("final_norm", C.c_void_p),
                ("lm_head", C.c_void_p)]


class Kv(C.Structure):
    _fields_ = [("pool", C.c_void_p), ("block_table_host", C.c_void_p), ("block_table_dev", C.c_void_p),
                ("page_tokens", C.c_int32), ("n_physical_pages", C.c_int32), ("n_logical_pages", C.c_int32)]


class KvStore(C.Structure):
    _fields_ = [("base", C.c_void_p), ("page_stride_bytes", C.c_uint64), ("page_tokens", C.c_int32),
                ("n_pages", C.c_int32), ("format", C.c_int32), ("source", C.c_int32), ("fd", C.c_int32),
                ("pad_", C.c_int32), ("file_offset", C.c_uint64)]


class ChunkLog(C.Structure):
    _fields_ = [("source", C.c_int32), ("tok_begin", C.c_int32), ("tok_count", C.c_int32),
                ("start_ns", C.c_uint64), ("end_ns", C.c_uint64), ("work", C.c_uint64), ("device_ns", C.c_uint64)]


class DecisionLog(C.Structure):
    _fields_ = [("who", C.c_int32), ("f", C.c_int32), ("b", C.c_int32), ("m_star", C.c_int32),
                ("claimed", C.c_int32), ("f_off", C.c_int32), ("claimed_tokens", C.c_int32), ("pad_", C.c_int32),
                ("now_ns", C.c_uint64), ("o_c", C.c_uint64),
                ("o_l", C.c_uint64), ("est_compute_ns", C.c_uint64), ("est_compute_flops", C.c_uint64),
                ("est_load_ns", C.c_uint64), ("est_load_bytes", C.c_uint64), ("partial_ns", C.c_uint64)]


class Request(C.Structure):
    _fields_ = [("token_ids", C.c_void_p), ("n_tokens", C.c_int32), ("has_prefix_cache", C.c_int32),
                ("arrival_ns", C.c_uint64), ("kv", C.c_void_p), ("store", C.c_void_p), ("ttft_ns", C.c_uint64),
                ("tokens_computed", C.c_int32), ("tokens_loaded", C.c_int32),
                ("want_first_token", C.c_int32), ("first_token", C.c_int32)]


class StepLog(C.Structure):
    _fields_ = [("start_ns", C.c_uint64), ("end_ns", C.c_uint64), ("decode_tokens", C.c_int32),
                ("nonprefix_tokens", C.c_int32), ("prefix_tokens", C.c_int32), ("prefix_tok_begin", C.c_int32),
                ("first_nonprefix_req", C.c_int32), ("other_tokens", C.c_int32)]


class Traces(C.Structure):
    _fields_ = [("other_tokens", C.c_void_p), ("n_other_tokens", C.c_int32), ("n_scratch_tokens", C.c_int32),
                ("scratch_kv", C.c_void_p), ("scratch_token_ids", C.c_void_p), ("gbps", C.c_void_p),
                ("n_gbps", C.c_int32), ("pad_", C.c_int32), ("gbps_interval_ns", C.c_uint64)]


class Result(C.Structure):
    _fields_ = [("chunks", C.POINTER(ChunkLog)), ("chunks_cap", C.c_int32),
                ("decisions", C.POINTER(DecisionLog)), ("decisions_cap", C.c_int32),
                ("n_chunks", C.c_int32), ("n_decisions", C.c_int32), ("meet_point", C.c_int32),
                ("load_failed_chunk", C.c_int32), ("ttft_ns", C.c_uint64), ("compute_busy_ns", C.c_uint64),
                ("compute_device_ns", C.c_uint64), ("compute_flops", C.c_uint64), ("load_busy_ns", C.c_uint64),
                ("load_bytes", C.c_uint64), ("stored_chunks", C.c_int32), ("pad_", C.c_int32)]


class KernelStats(C.Structure):
    _fields_ = [("launches", C.c_uint64), ("total_ns", C.c_uint64), ("flops", C.c_uint64), ("bytes", C.c_uint64)]


class Tuning(C.Structure):
    _fields_ = [("prior_compute_ns", C.c_uint64), ("prior_compute_flops", C.c_uint64), ("piece_bytes", C.c_uint64),
                ("kernel_path", C.c_int32), ("gemm_config", C.c_int32), ("attn_variant", C.c_int32), ("gemm_ksplit", C.c_int32)]


def load_library():
    """Loads libcake.so and declares the prototypes.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise CakeError(E_STATE, "libcake.so is not built (run `python __graft_entry__.py`); there is no fallback")
    lib = C.CDLL(LIB_PATH)
    vp, i32, u64, dbl = C.c_void_p, C.c_int32, C.c_uint64, C.c_double
    P = C.POINTER
    sig = {
        "cake_create": (i32, [P(vp), P(ModelDesc), P(Weights), i32, i32, vp, vp]),
        "cake_destroy": (i32, [vp]),
        "cake_last_error": (C.c_char_p, [vp]),
        "cake_set_tuning": (i32, [vp, P(Tuning)]),
        "cake_prefill_chunk": (i32, [vp, vp, i32, i32, P(Kv)]),
        "cake_load_chunk": (i32, [vp, P(KvStore), i32, i32, P(Kv), dbl]),
        "cake_plan_meet_point": (i32, [vp, vp, i32, u64, u64, P(i32), P(u64)]),
        "cake_bidirectional_prefill": (i32, [vp, vp, i32, P(KvStore), i32, dbl, i32, i32, P(Kv), P(Result)]),
        "cake_first_token": (i32, [vp, vp, i32, P(Kv), P(i32), vp, P(u64)]),
        "cake_set_traces": (i32, [vp, P(Traces)]),
        "cake_store_image_bytes": (u64, [P(ModelDesc), i32, i32]),
        "cake_prefix_keys": (i32, [vp, i32, i32, vp, i32]),
        "cake_prefix_lookup": (i32, [vp, i32, vp, i32]),
        "cake_write_store": (i32, [vp, P(Kv), i32, P(KvStore)]),
        "cake_op_decode_attention": (i32, [vp, vp, vp, i32, i32, P(Kv)]),
        "cake_op_decode_attention_static": (i32, [vp, vp, vp, i32, i32, P(Kv)]),
        "cake_set_bandwidth": (i32, [vp, dbl]),
        "cake_schedule_bandwidth_step": (i32, [vp, i32, dbl]),
        "cake_chunk_state": (i32, [vp, i32]),
        "cake_sync_compute": (i32, [vp]),
        "cake_sync_load": (i32, [vp]),
        "cake_range_flops": (u64, [P(ModelDesc), i32, i32]),
        "cake_page_image_bytes": (u64, [P(ModelDesc), i32]),
        "cake_simulate_race": (i32, [i32, vp, vp, vp, vp, u64, u64, u64, u64, i32, i32, i32, vp, P(u64),
                                     P(DecisionLog), i32, P(i32)]),
        "cake_adaptive_serve": (i32, [vp, P(Request), i32, i32, i32, dbl, P(Result), P(StepLog), i32, P(i32)]),
        "cake_profile_enable": (i32, [vp, i32]),
        "cake_profile_read": (i32, [vp, P(KernelStats)]),
        "cake_op_rmsnorm": (i32, [vp, vp, vp, vp, i32, i32]),
        "cake_op_gemm": (i32, [vp, vp, vp, vp, i32, i32, i32]),
        "cake_op_gemm_residual": (i32, [vp, vp, vp, vp, i32, i32, i32]),
        "cake_op_gemm_swiglu": (i32, [vp, vp, vp, vp, vp, i32, i32, i32]),
        "cake_op_gemm_plan": (i32, [vp, i32, i32, i32, i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
        "cake_op_mfma_rate": (i32, [vp, i32, i32, P(C.c_double)]),
        "cake_device_info": (i32, [vp, P(i32), P(i32), P(C.c_uint64)]),
        "cake_op_rope_kv_write": (i32, [vp, vp, vp, i32, i32, i32, P(Kv)]),
        "cake_op_attention": (i32, [vp, vp, vp, i32, i32, i32, P(Kv)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


# --------------------------------------------------------------------------- host-only calls
def _u64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint64))


def plan_meet_point(compute_ns, load_ns, compute_offset_ns=0, load_offset_ns=0):
    """cake_plan_meet_point -> (m, ttft_ns)."""
    lib = load_library()
    c, l = _u64(compute_ns), _u64(load_ns)
    if len(c) != len(l):
        raise ValueError("length mismatch")
    m, t = C.c_int32(), C.c_uint64()
    rc = lib.cake_plan_meet_point(c.ctypes.data, l.ctypes.data, len(c), int(compute_offset_ns),
                                  int(load_offset_ns), C.byref(m), C.byref(t))
    if rc != OK:
        raise CakeError(rc, "cake_plan_meet_point")
    return m.value, t.value


def _decisions_to_list(arr, n):
    keys = [f[0] for f in DecisionLog._fields_]
    return [{k: getattr(arr[i], k) for k in keys} for i in range(n)]


def simulate_race(chunk_flops, chunk_bytes, actual_compute_ns, actual_load_ns, prior_compute=(1, 1),
                  prior_load=(1, 1), mode="bidir", forced_m=0, fail_load_chunk=-1, decisions_cap=4096):
    """cake_simulate_race -> (ttft_ns, sources list, decisions list of dicts)."""
    lib = load_library()
    fl, by, ac, al = _u64(chunk_flops), _u64(chunk_bytes), _u64(actual_compute_ns), _u64(actual_load_ns)
    n = len(fl)
    src = np.zeros(max(n, 1), dtype=np.int32)
    dec = (DecisionLog * decisions_cap)()
    nd, t = C.c_int32(), C.c_uint64()
    rc = lib.cake_simulate_race(n, fl.ctypes.data, by.ctypes.data, ac.ctypes.data, al.ctypes.data,
                                int(prior_compute[0]), int(prior_compute[1]), int(prior_load[0]),
                                int(prior_load[1]), MODES[mode], forced_m, fail_load_chunk, src.ctypes.data,
                                C.byref(t), dec, decisions_cap, C.byref(nd))
    if rc != OK:
        raise CakeError(rc, "cake_simulate_race")
    return t.value, [int(s) for s in src[:n]], _decisions_to_list(dec, nd.value)


def prefix_keys(tokens, chunk_tokens):
    """cake_prefix_keys -> list of uint64 keys, one per full chunk."""
    lib = load_library()
    ids = np.ascontiguousarray(tokens, dtype=np.int32)
    n = len(ids) // chunk_tokens if chunk_tokens > 0 else 0
    out = np.zeros(max(n, 1), dtype=np.uint64)
    rc = lib.cake_prefix_keys(ids.ctypes.data, len(ids), chunk_tokens, out.ctypes.data, n)
    if rc < 0:
        raise CakeError(rc, "cake_prefix_keys")
    return [int(k) for k in out[:n]]


def prefix_lookup(stored_sorted, keys):
    """cake_prefix_lookup -> number of leading chunks held by the store."""
    lib = load_library()
    st = np.ascontiguousarray(stored_sorted, dtype=np.uint64)
    ks = np.ascontiguousarray(keys, dtype=np.uint64)
    rc = lib.cake_prefix_lookup(st.ctypes.data if len(st) else None, len(st), ks.ctypes.data if len(ks) else None, len(ks))
    if rc < 0:
        raise CakeError(rc, "cake_prefix_lookup")
    return rc


def model_desc(shape) -> ModelDesc:
    return ModelDesc(shape.n_layers, shape.d_model, shape.n_q, shape.n_kv, shape.head_dim, shape.ffn, shape.vocab,
                     F32 if shape.dtype == "f32" else BF16, shape.rms_eps, shape.rope_theta)


def range_flops(shape, tok_begin, tok_count) -> int:
    return int(load_library().cake_range_flops(C.byref(model_desc(shape)), tok_begin, tok_count))


def page_image_bytes(shape, page_tokens) -> int:
    return int(load_library().cake_page_image_bytes(C.byref(model_desc(shape)), page_tokens))


# --------------------------------------------------------------------------- device side
@dataclass
class PrefillResult:
    meet_point: int
    ttft_ns: int
    n_chunks: int
    load_failed_chunk: int
    compute_busy_ns: int
    compute_device_ns: int
    compute_flops: int
    load_busy_ns: int
    load_bytes: int
    chunks: List[dict] = field(default_factory=list)
    decisions: List[dict] = field(default_factory=list)
    status: int = 0
    stored_chunks: int = -1

    @property
    def achieved_gbps(self) -> float:
        return self.load_bytes / self.load_busy_ns if self.load_busy_ns else 0.0

    @property
    def compute_tflops(self) -> float:
        return self.compute_flops / self.compute_device_ns / 1e3 if self.compute_device_ns else 0.0


class Engine:
    """Owns the device tensors (weights in ABI layout, KV pool, block tables), the pinned
    store and the two streams, and forwards to the C ABI."""

    def __init__(self, shape, weights=None, *, max_tokens, max_chunk, page_tokens=256, block_table=None,
                 n_physical_pages=None, device="cuda:0", seed=0, with_head=False):
        import torch
        self.torch = torch
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise CakeError(E_STATE, "no GPU: the HIP path cannot run and there is no CPU fallback")
        self.shape = shape
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.tdtype = torch.float32 if shape.dtype == "f32" else torch.bfloat16
        self.page_tokens = page_tokens
        self.max_tokens, self.max_chunk = max_tokens, max_chunk
        self.compute_stream = torch.cuda.Stream(device=self.dev)
        self.copy_stream = torch.cuda.Stream(device=self.dev)
        self._tensors = []
        self.with_head = with_head or (weights is not None and "lm_head" in weights)
        self._build_weights(weights, seed)
        n_logical = (max_tokens + page_tokens - 1) // page_tokens
        n_phys = n_physical_pages or n_logical
        bt = np.arange(n_logical, dtype=np.int32) if block_table is None else np.asarray(block_table, dtype=np.int32)
        assert len(bt) == n_logical
        self.block_table_host = np.ascontiguousarray(bt)
        self.block_table_dev = torch.from_numpy(self.block_table_host).to(self.dev)
        self.layer_page_elems = 2 * shape.n_kv * page_tokens * shape.head_dim
        self.pool = torch.zeros((shape.n_layers, n_phys, self.layer_page_elems), dtype=self.tdtype, device=self.dev)
        self.kv = Kv(self.pool.data_ptr(), self.block_table_host.ctypes.data, self.block_table_dev.data_ptr(),
                     page_tokens, n_phys, n_logical)
        self.store_tensor = None
        self.store = None
        self.ctx = C.c_void_p()
        desc = model_desc(shape)
        rc = self.lib.cake_create(C.byref(self.ctx), C.byref(desc), C.byref(self._weights), max_tokens, max_chunk,
                                  self.compute_stream.cuda_stream, self.copy_stream.cuda_stream)
        if rc != OK:
            raise CakeError(rc, "cake_create")
        torch.cuda.synchronize()

    # -- weights ---------------------------------------------------------------------
    def _dev(self, a, dtype=None):
        """numpy [in, out] matrix -> device tensor [out, in] of the model dtype."""
        t = self.torch.from_numpy(np.ascontiguousarray(a)).to(self.dev).to(dtype or self.tdtype).contiguous()
        self._tensors.append(t)
        return t

    def _build_weights(self, weights, seed):
        torch, s = self.torch, self.shape
        self.layer_tensors = []
        arr = (LayerWeights * s.n_layers)()
        if weights is not None:
            self.embed = self._dev(weights["embed"])
            for l, lw in enumerate(weights["layers"]):
                wqkv = np.concatenate([lw["wq"].T, lw["wk"].T, lw["wv"].T], axis=0)
                t = dict(attn_norm=self._dev(lw["attn_norm"], torch.float32), wqkv=self._dev(wqkv),
                         wo=self._dev(lw["wo"].T), ffn_norm=self._dev(lw["ffn_norm"], torch.float32),
                         w_gate=self._dev(lw["w_gate"].T), w_up=self._dev(lw["w_up"].T),
                         w_down=self._dev(lw["w_down"].T))
                self.layer_tensors.append(t)
        else:  # random N(0, 0.02) generated on the device, for shapes too large to draw on the host
            g = torch.Generator(device=self.dev)
            g.manual_seed(seed)

            def rnd(*dims):
                t = torch.empty(dims, dtype=self.tdtype, device=self.dev)
                t.normal_(0.0, 0.02, generator=g)
                return t
            hq, hkv = s.n_q * s.head_dim, s.n_kv * s.head_dim
            self.embed = rnd(s.vocab, s.d_model)
            for l in range(s.n_layers):
                t = dict(attn_norm=torch.ones(s.d_model, dtype=torch.float32, device=self.dev),
                         wqkv=rnd(hq + 2 * hkv, s.d_model), wo=rnd(s.d_model, hq),
                         ffn_norm=torch.ones(s.d_model, dtype=torch.float32, device=self.dev),
                         w_gate=rnd(s.ffn, s.d_model), w_up=rnd(s.ffn, s.d_model), w_down=rnd(s.d_model, s.ffn))
                self.layer_tensors.append(t)
        for l, t in enumerate(self.layer_tensors):
            for k, v in t.items():
                setattr(arr[l], k, v.data_ptr())
        self._layer_arr = arr
        self.final_norm = self.lm_head = None
        if self.with_head:
            if weights is not None:
                self.final_norm = self._dev(weights["final_norm"], torch.float32)
                self.lm_head = self._dev(weights["lm_head"].T)
            else:
                self.final_norm = torch.ones(s.d_model, dtype=torch.float32, device=self.dev)
                self.lm_head = rnd(s.vocab, s.d_model)
        self._weights = Weights(self.embed.data_ptr(), arr,
                                self.final_norm.data_ptr() if self.with_head else None,
                                self.lm_head.data_ptr() if self.with_head else None)

    # -- store -----------------------------------------------------------------------
    def set_store(self, images: np.ndarray):
        """images: [n_pages, L, 2, words] raw storage words (uint32 for f32, uint16 for bf16)."""
        torch = self.torch
        flat = np.ascontiguousarray(images).reshape(images.shape[0], -1)
        t = torch.empty(flat.shape, dtype=torch.int32 if flat.dtype == np.uint32 else torch.int16, pin_memory=True)
        t.numpy()[:] = flat.view(np.int32 if flat.dtype == np.uint32 else np.int16)
        self._set_store_tensor(t)

    def _set_store_tensor(self, t, fmt=STORE_RAW):
        self.store_tensor = t
        stride = t.shape[1] * t.element_size()
        self.store = KvStore(t.data_ptr(), stride, self.page_tokens, t.shape[0], fmt, STORE_PINNED, -1, 0, 0)

    def set_file_store(self, fd, n_pages, stride, fmt=STORE_RAW, file_offset=0):
        """A store read from an open file (two hops: file -> pinned staging -> pages)."""
        self.store_tensor = None
        self.store = KvStore(None, stride, self.page_tokens, n_pages, fmt, STORE_FILE, fd, 0, file_offset)

    def set_store_int8(self, images: np.ndarray, fmt=STORE_INT8):
        """images: [n_pages, L, 2, bytes] uint8 in a quantised store format (codes then scales per layer and K|V)."""
        torch = self.torch
        flat = np.ascontiguousarray(images).reshape(images.shape[0], -1)
        t = torch.empty(flat.shape, dtype=torch.uint8, pin_memory=True)
        t.numpy()[:] = flat
        self._set_store_tensor(t, fmt)

    def set_store_int4(self, images: np.ndarray):
        """As set_store_int8 for the 4-bit format (two codes per byte)."""
        self.set_store_int8(images, STORE_INT4)

    def write_store(self, n_tokens, fmt=STORE_INT8):
        """The pool's KV of [0, n_tokens) written into a new pinned store of the given format (cake_write_store)."""
        torch = self.torch
        n_pages = (n_tokens + self.page_tokens - 1) // self.page_tokens
        image = int(self.lib.cake_store_image_bytes(C.byref(model_desc(self.shape)), self.page_tokens, fmt))
        t = torch.empty((n_pages, image), dtype=torch.uint8, pin_memory=True)
        self._set_store_tensor(t, fmt)
        self._check(self.lib.cake_write_store(self.ctx, C.byref(self.kv), n_tokens, C.byref(self.store)), "cake_write_store")
        return t

    def store_from_pool(self, n_tokens):
        """Copies the pool's current KV of [0, n_tokens) into a new pinned store (page images)."""
        torch = self.torch
        n_pages = (n_tokens + self.page_tokens - 1) // self.page_tokens
        words = self.shape.n_layers * self.layer_page_elems
        idt = torch.int32 if self.shape.dtype == "f32" else torch.int16
        t = torch.empty((n_pages, words), dtype=idt, pin_memory=True)
        torch.cuda.synchronize()
        phys = torch.from_numpy(self.block_table_host[:n_pages].astype(np.int64)).to(self.dev)
        for p0 in range(0, n_pages, 8):
            p1 = min(p0 + 8, n_pages)
            blk = self.pool[:, phys[p0:p1]].permute(1, 0, 2).contiguous().view(idt).reshape(p1 - p0, words)
            t[p0:p1].copy_(blk)
        torch.cuda.synchronize()
        self._set_store_tensor(t)

    def clear_pool(self):
        self.pool.zero_()
        self.torch.cuda.synchronize()

    def pool_images(self, n_tokens) -> np.ndarray:
        """Decoded pool contents in logical page order: float64 [n_pages, L, 2, words/2]."""
        torch = self.torch
        torch.cuda.synchronize()
        n_pages = (n_tokens + self.page_tokens - 1) // self.page_tokens
        phys = torch.from_numpy(self.block_table_host[:n_pages].astype(np.int64)).to(self.dev)
        blk = self.pool[:, phys].permute(1, 0, 2).float().cpu().numpy().astype(np.float64)
        return blk.reshape(n_pages, self.shape.n_layers, 2, self.layer_page_elems // 2)

    def pool_raw(self, n_tokens) -> np.ndarray:
        """Raw pool words in logical page order (for byte comparisons)."""
        torch = self.torch
        torch.cuda.synchronize()
        n_pages = (n_tokens + self.page_tokens - 1) // self.page_tokens
        phys = torch.from_numpy(self.block_table_host[:n_pages].astype(np.int64)).to(self.dev)
        idt = torch.int32 if self.shape.dtype == "f32" else torch.int16
        blk = self.pool[:, phys].permute(1, 0, 2).contiguous().view(idt).cpu().numpy()
        return blk.reshape(n_pages, self.shape.n_layers, 2, self.layer_page_elems // 2)

    # -- calls -----------------------------------------------------------------------
    def _check(self, rc, what, allow=()):
        if rc != OK and rc not in allow:
            raise CakeError(rc, "%s: %s" % (what, self.lib.cake_last_error(self.ctx).decode()))
        return rc

    def set_tuning(self, prior_compute_ns=0, prior_compute_flops=0, piece_bytes=0, kernel_path=0, gemm_config=0,
                   attn_variant=0, gemm_ksplit=0):
        t = Tuning(prior_compute_ns, prior_compute_flops, piece_bytes, kernel_path, gemm_config, attn_variant, gemm_ksplit)
        self._check(self.lib.cake_set_tuning(self.ctx, C.byref(t)), "cake_set_tuning")

    def _ids(self, tokens):
        return np.ascontiguousarray(np.asarray(tokens, dtype=np.int32))

    def prefill_chunk(self, tokens, tok_begin, tok_count, sync=True):
        ids = self._ids(tokens)
        self._keep = ids
        self._check(self.lib.cake_prefill_chunk(self.ctx, ids.ctypes.data, tok_begin, tok_count, C.byref(self.kv)),
                    "cake_prefill_chunk")
        if sync:
            self._check(self.lib.cake_sync_compute(self.ctx), "cake_sync_compute")

    def load_chunk(self, tok_begin, tok_count, gbps=0.0, sync=True):
        self._check(self.lib.cake_load_chunk(self.ctx, C.byref(self.store), tok_begin, tok_count, C.byref(self.kv),
                                             float(gbps)), "cake_load_chunk")
        if sync:
            self._check(self.lib.cake_sync_load(self.ctx), "cake_sync_load")

    def bidirectional_prefill(self, tokens, chunk, gbps, mode="bidir", forced_m=0, log=True) -> PrefillResult:
        ids = self._ids(tokens)
        n = (len(ids) + chunk - 1) // chunk
        res = Result()
        chunks = (ChunkLog * max(n, 1))()
        dcap = 8 * n + 16
        dec = (DecisionLog * dcap)()
        if log:
            res.chunks, res.chunks_cap, res.decisions, res.decisions_cap = chunks, n, dec, dcap
        store = C.byref(self.store) if self.store is not None else None
        rc = self.lib.cake_bidirectional_prefill(self.ctx, ids.ctypes.data, len(ids), store, chunk, float(gbps),
                                                 MODES[mode], forced_m, C.byref(self.kv), C.byref(res))
        self._check(rc, "cake_bidirectional_prefill", allow=(E_CAPACITY,))
        out = PrefillResult(res.meet_point, res.ttft_ns, res.n_chunks, res.load_failed_chunk, res.compute_busy_ns,
                            res.compute_device_ns, res.compute_flops, res.load_busy_ns, res.load_bytes, status=rc,
                            stored_chunks=res.stored_chunks)
        if log:
            ck = [f[0] for f in ChunkLog._fields_]
            out.chunks = [{k: getattr(chunks[i], k) for k in ck} for i in range(min(n, res.n_chunks))]
            out.decisions = _decisions_to_list(dec, res.n_decisions)
        return out

    def op_decode_attention(self, q, layer, n_keys, out=None, static=False):
        """q: float32 device tensor [n_q][hd] -> float32 [n_q][hd].  static: the entry point that
        allocates nothing (its partial results live in the library's own static buffer); `out` may be
        a tensor made beforehand so that nothing is allocated around the call either."""
        if out is None:
            out = self.torch.empty_like(q)
        fn = self.lib.cake_op_decode_attention_static if static else self.lib.cake_op_decode_attention
        self._check(fn(self.ctx, q.data_ptr(), out.data_ptr(), layer, n_keys, C.byref(self.kv)),
                    "cake_op_decode_attention_static" if static else "cake_op_decode_attention")
        self.sync()
        return out

    def first_token(self, tokens, want_logits=False):
        """The first output token from the complete KV of `tokens` (cake_first_token).
        Returns (token id, device ns, logits as float32 numpy or None)."""
        ids = self._ids(tokens)
        tok, ns = C.c_int32(-1), C.c_uint64(0)
        logits = np.empty(self.shape.vocab, dtype=np.float32) if want_logits else None
        rc = self.lib.cake_first_token(self.ctx, ids.ctypes.data, len(ids), C.byref(self.kv), C.byref(tok),
                                       logits.ctypes.data if want_logits else None, C.byref(ns))
        self._check(rc, "cake_first_token")
        return tok.value, ns.value, logits

    def new_kv(self, n_tokens):
        """A further KV pool + block table of this shape (one per concurrent request)."""
        torch = self.torch
        n_log = (n_tokens + self.page_tokens - 1) // self.page_tokens
        bt_host = np.arange(n_log, dtype=np.int32)
        bt_dev = torch.from_numpy(bt_host).to(self.dev)
        pool = torch.zeros((self.shape.n_layers, n_log, self.layer_page_elems), dtype=self.tdtype, device=self.dev)
        kv = Kv(pool.data_ptr(), bt_host.ctypes.data, bt_dev.data_ptr(), self.page_tokens, n_log, n_log)
        self._tensors.append((bt_host, bt_dev, pool))
        return kv, pool

    def set_traces(self, other_tokens=None, gbps_trace=None, gbps_interval_ns=0, scratch_seed=99):
        """Resource traces of the next adaptive_serve (cake_set_traces): per-step tokens of other users,
        bandwidth samples over time.  The scratch pages and ids for the other users' prefill are made here."""
        t = Traces()
        keep = []
        if other_tokens is not None and len(other_tokens):
            ot = np.ascontiguousarray(other_tokens, dtype=np.int32)
            n_scr = max(int(ot.max()), 1)
            if getattr(self, "_scratch", None) is None or self._scratch[2] < n_scr:
                kv, pool = self.new_kv(n_scr)
                self._scratch = (kv, pool, n_scr)
            ids = np.random.default_rng(scratch_seed).integers(0, self.shape.vocab, n_scr).astype(np.int32)
            t.other_tokens, t.n_other_tokens, t.n_scratch_tokens = ot.ctypes.data, len(ot), n_scr
            t.scratch_kv, t.scratch_token_ids = C.addressof(self._scratch[0]), ids.ctypes.data
            keep += [ot, ids]
        if gbps_trace is not None and len(gbps_trace):
            g = np.ascontiguousarray(gbps_trace, dtype=np.float64)
            t.gbps, t.n_gbps, t.gbps_interval_ns = g.ctypes.data, len(g), int(gbps_interval_ns)
            keep.append(g)
        self._check(self.lib.cake_set_traces(self.ctx, C.byref(t)), "cake_set_traces")

    def adaptive_serve(self, requests, token_budget, fetch_chunk, gbps):
        """requests: list of dicts {tokens, arrival_ns, prefix (bool), kv (Kv or None = the engine's own),
        first_token (bool: the request also takes its first decode step)}.
        Returns (PrefillResult for the prefix request, per-request dicts, step list)."""
        n = len(requests)
        arr = (Request * n)()
        keep = []
        for i, r in enumerate(requests):
            ids = self._ids(r["tokens"])
            keep.append(ids)
            kv = r.get("kv") or self.kv
            keep.append(kv)
            arr[i].token_ids = ids.ctypes.data
            arr[i].n_tokens = len(ids)
            arr[i].has_prefix_cache = 1 if r.get("prefix") else 0
            arr[i].arrival_ns = int(r.get("arrival_ns", 0))
            arr[i].kv = C.addressof(kv)
            arr[i].store = C.addressof(self.store) if r.get("prefix") else None
            arr[i].want_first_token = 1 if r.get("first_token") else 0
        nc = max(1, max((len(r["tokens"]) + fetch_chunk - 1) // fetch_chunk for r in requests))
        res = Result()
        chunks = (ChunkLog * nc)()
        total_tokens = sum(len(r["tokens"]) for r in requests)
        scap = 4 * (total_tokens // max(1, min(token_budget, 64)) + n) + 64
        dcap = 4 * scap
        dec = (DecisionLog * dcap)()
        steps = (StepLog * scap)()
        res.chunks, res.chunks_cap, res.decisions, res.decisions_cap = chunks, nc, dec, dcap
        ns = C.c_int32()
        rc = self.lib.cake_adaptive_serve(self.ctx, arr, n, token_budget, fetch_chunk, float(gbps), C.byref(res), steps,
                                          scap, C.byref(ns))
        self._check(rc, "cake_adaptive_serve", allow=(E_CAPACITY,))
        out = PrefillResult(res.meet_point, res.ttft_ns, res.n_chunks, res.load_failed_chunk, res.compute_busy_ns,
                            res.compute_device_ns, res.compute_flops, res.load_busy_ns, res.load_bytes, status=rc)
        ck = [f[0] for f in ChunkLog._fields_]
        out.chunks = [{k: getattr(chunks[i], k) for k in ck} for i in range(res.n_chunks)]
        out.decisions = _decisions_to_list(dec, res.n_decisions)
        per_req = [dict(ttft_ns=arr[i].ttft_ns, tokens_computed=arr[i].tokens_computed, tokens_loaded=arr[i].tokens_loaded,
                        first_token=arr[i].first_token) for i in range(n)]
        sk = [f[0] for f in StepLog._fields_]
        step_list = [{k: getattr(steps[i], k) for k in sk} for i in range(ns.value)]
        return out, per_req, step_list

    def mfma_rate(self, workgroups=2048, iters=4096):
        """TFLOP/s of bf16 MFMAs on register operands only (cake_op_mfma_rate): what the matrix pipes of this GPU
        sustain at the clock the device holds under that load, a yardstick for the GEMM and attention figures."""
        v = C.c_double(0.0)
        self._check(self.lib.cake_op_mfma_rate(self.ctx, workgroups, iters, C.byref(v)), "cake_op_mfma_rate")
        return v.value

    def device_info(self):
        """(compute units, peak engine clock in kHz, device memory in bytes) of the context's GPU."""
        cu, khz, mem = C.c_int32(0), C.c_int32(0), C.c_uint64(0)
        self._check(self.lib.cake_device_info(self.ctx, C.byref(cu), C.byref(khz), C.byref(mem)), "cake_device_info")
        return cu.value, khz.value, mem.value

    def set_bandwidth(self, gbps):
        self._check(self.lib.cake_set_bandwidth(self.ctx, float(gbps)), "cake_set_bandwidth")

    def schedule_bandwidth_step(self, after_loaded_chunks, gbps):
        self._check(self.lib.cake_schedule_bandwidth_step(self.ctx, after_loaded_chunks, float(gbps)),
                    "cake_schedule_bandwidth_step")

    def profile_enable(self, on=True, classes=None):
        """classes: names from KERNEL_CLASSES to bracket (default: all)."""
        arg = 1 if on else 0
        if on and classes:
            arg = 2 * sum(1 << KERNEL_CLASSES.index(n) for n in classes)
        self._check(self.lib.cake_profile_enable(self.ctx, arg), "cake_profile_enable")

    def profile_read(self):
        """{class name: dict(launches, total_ns, flops, bytes)} since the last read."""
        arr = (KernelStats * len(KERNEL_CLASSES))()
        self._check(self.lib.cake_profile_read(self.ctx, arr), "cake_profile_read")
        return {n: dict(launches=arr[i].launches, total_ns=arr[i].total_ns, flops=arr[i].flops, bytes=arr[i].bytes)
                for i, n in enumerate(KERNEL_CLASSES)}

    def chunk_state(self, i):
        return self.lib.cake_chunk_state(self.ctx, i)

    def sync(self):
        self._check(self.lib.cake_sync_compute(self.ctx), "cake_sync_compute")
        self._check(self.lib.cake_sync_load(self.ctx), "cake_sync_load")

    # -- single kernels (tensors are torch device tensors) -----------------------------
    def op_rmsnorm(self, x, gain):
        out = self.torch.empty(x.shape, dtype=self.tdtype, device=self.dev)
        self._check(self.lib.cake_op_rmsnorm(self.ctx, x.data_ptr(), gain.data_ptr(), out.data_ptr(), x.shape[0],
                                             x.shape[1]), "cake_op_rmsnorm")
        self.sync()
        return out

    def op_gemm(self, a, w):
        out = self.torch.empty((a.shape[0], w.shape[0]), dtype=self.torch.float32, device=self.dev)
        self._check(self.lib.cake_op_gemm(self.ctx, a.data_ptr(), w.data_ptr(), out.data_ptr(), a.shape[0], w.shape[0],
                                          a.shape[1]), "cake_op_gemm")
        self.sync()
        return out

    def op_gemm_residual(self, a, w, x):
        self._check(self.lib.cake_op_gemm_residual(self.ctx, a.data_ptr(), w.data_ptr(), x.data_ptr(), a.shape[0],
                                                   w.shape[0], a.shape[1]), "cake_op_gemm_residual")
        self.sync()
        return x

    def op_gemm_plan(self, M, N, K, residual=True):
        """(tile rows, tile columns, K ranges per tile) of the GEMM kernel chosen for this shape."""
        tile = (C.c_int32 * 2)()
        ks = C.c_int32(0)
        self._check(self.lib.cake_op_gemm_plan(self.ctx, int(bool(residual)), M, N, K, tile, C.byref(ks)), "cake_op_gemm_plan")
        return tile[0], tile[1], ks.value

    def op_gemm_swiglu(self, a, wg, wu):
        out = self.torch.empty((a.shape[0], wg.shape[0]), dtype=self.tdtype, device=self.dev)
        self._check(self.lib.cake_op_gemm_swiglu(self.ctx, a.data_ptr(), wg.data_ptr(), wu.data_ptr(), out.data_ptr(),
                                                 a.shape[0], wg.shape[0], a.shape[1]), "cake_op_gemm_swiglu")
        self.sync()
        return out

    def op_rope_kv_write(self, qkv, layer, tok_begin):
        rows = qkv.shape[0]
        q = self.torch.empty((self.shape.n_q, rows, self.shape.head_dim), dtype=self.tdtype, device=self.dev)
        self._check(self.lib.cake_op_rope_kv_write(self.ctx, qkv.data_ptr(), q.data_ptr(), layer, tok_begin, rows,
                                                   C.byref(self.kv)), "cake_op_rope_kv_write")
        self.sync()
        return q

    def op_attention(self, q, layer, tok_begin):
        rows = q.shape[1]
        out = self.torch.empty((rows, self.shape.n_q * self.shape.head_dim), dtype=self.tdtype, device=self.dev)
        self._check(self.lib.cake_op_attention(self.ctx, q.data_ptr(), out.data_ptr(), layer, tok_begin, rows,
                                               C.byref(self.kv)), "cake_op_attention")
        self.sync()
        return out

    def close(self):
        if getattr(self, "ctx", None) and self.ctx.value:
            self.lib.cake_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
