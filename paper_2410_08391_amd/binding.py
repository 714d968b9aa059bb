"""ctypes binding of libkvp's C ABI (include/kvp.h): argument marshalling only.

Every step of the path runs inside the library's HIP kernels; this module turns
torch tensors into raw device pointers and hands over the current HIP stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Mapping, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))

STAGE_AUX, STAGE_PREDICT, STAGE_BASE, STAGE_ALL = 1, 2, 4, 7
STAGE_BASE_ABSORBED = 8       # the base step with the predictor absorbed into its attention (reads the auxiliary cache)
KERNEL_CLASSES = ("embed_norm", "aux_gemm", "aux_attn", "predictor", "base_gemv", "decode_attn", "argmax")
DTYPE_F32, DTYPE_BF16 = 0, 1

MODEL_BASE, MODEL_AUX = 0, 1
EXPORTS = ("kvp_load_weights", "kvp_workspace_bytes", "kvp_prefill_predict", "kvp_run_stages",
           "kvp_aux_cache_offsets", "kvp_reference_workspace_bytes", "kvp_reference_prefill",
           "kvp_generation_workspace_bytes", "kvp_generation_step", "kvp_generation_step_static", "kvp_static_scratch_bytes",
           "kvp_check_flags", "kvp_debug_plan", "kvp_probe_mfma", "kvp_probe_stream", "kvp_debug_flash_guard", "kvp_profile_enable", "kvp_profile_reset", "kvp_profile_read",
           "kvp_free", "kvp_last_error", "kvp_version")
FLAG_TOKEN_CLAMPED = 1


class KVPError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libkvp error {code}: {msg}")
        self.code = code


class ModelShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "ffn_dim")] + \
               [(n, C.POINTER(C.c_int32)) for n in ("layer_n_q_heads", "layer_n_kv_heads", "layer_ffn_dim")]


class Config(C.Structure):
    _fields_ = [("base", ModelShape), ("aux", ModelShape), ("vocab", C.c_int32), ("dtype", C.c_int32),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("layer_map", C.POINTER(C.c_int32)),
                ("max_batch", C.c_int32), ("max_seq", C.c_int32)]


PP = C.POINTER(C.c_void_p)


class ModelWeights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + \
               [(n, PP) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down", "q_norm", "k_norm")]


class Weights(C.Structure):
    _fields_ = [("base", ModelWeights), ("aux", ModelWeights), ("pred_wk", PP), ("pred_wv", PP)]


class PlanRegion(C.Structure):
    _fields_ = [("name", C.c_char * 24), ("offset", C.c_uint64), ("bytes", C.c_uint64), ("bytes_touched", C.c_uint64)]


_lib: Optional[C.CDLL] = None


def library_path() -> str:
    return os.environ.get("KVP_LIBRARY", os.path.join(HERE, "libkvp.so"))


def lib() -> C.CDLL:
    """Loads libkvp.so once.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2410_08391_amd.build`")
    L = C.CDLL(path)
    L.kvp_load_weights.argtypes = [C.POINTER(Config), C.POINTER(Weights), C.POINTER(C.c_void_p)]
    L.kvp_load_weights.restype = C.c_int
    L.kvp_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    L.kvp_workspace_bytes.restype = C.c_size_t
    run_args = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                C.c_void_p, C.c_size_t, C.c_void_p]
    L.kvp_prefill_predict.argtypes = [C.c_void_p] + run_args
    L.kvp_prefill_predict.restype = C.c_int
    L.kvp_run_stages.argtypes = [C.c_void_p, C.c_uint32] + run_args
    L.kvp_run_stages.restype = C.c_int
    L.kvp_reference_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
    L.kvp_reference_workspace_bytes.restype = C.c_size_t
    L.kvp_reference_prefill.argtypes = [C.c_void_p, C.c_int32] + run_args
    L.kvp_reference_prefill.restype = C.c_int
    L.kvp_generation_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    L.kvp_generation_workspace_bytes.restype = C.c_size_t
    L.kvp_generation_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.kvp_generation_step.restype = C.c_int
    L.kvp_generation_step_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64,
                                             C.c_void_p, C.c_void_p, C.c_void_p]
    L.kvp_generation_step_static.restype = C.c_int
    L.kvp_static_scratch_bytes.argtypes = []
    L.kvp_static_scratch_bytes.restype = C.c_size_t
    L.kvp_check_flags.argtypes = [C.c_void_p, C.POINTER(C.c_uint32), C.c_int32]
    L.kvp_check_flags.restype = C.c_int
    L.kvp_debug_plan.argtypes = [C.POINTER(Config), C.c_int32, C.c_int32, C.POINTER(PlanRegion), C.c_int32,
                                 C.POINTER(C.c_int32), C.POINTER(C.c_uint64)]
    L.kvp_debug_plan.restype = C.c_int
    L.kvp_debug_flash_guard.argtypes = [C.c_float]
    L.kvp_debug_flash_guard.restype = None
    L.kvp_probe_mfma.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.c_void_p]
    L.kvp_probe_mfma.restype = C.c_int
    L.kvp_probe_stream.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.kvp_probe_stream.restype = C.c_int
    L.kvp_aux_cache_offsets.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    L.kvp_aux_cache_offsets.restype = C.c_int
    L.kvp_profile_enable.argtypes = [C.c_void_p, C.c_int32]
    L.kvp_profile_enable.restype = C.c_int
    L.kvp_profile_reset.argtypes = [C.c_void_p]
    L.kvp_profile_reset.restype = C.c_int
    L.kvp_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.kvp_profile_read.restype = C.c_int
    L.kvp_free.argtypes = [C.c_void_p]
    L.kvp_free.restype = None
    L.kvp_last_error.restype = C.c_char_p
    L.kvp_version.restype = C.c_char_p
    _lib = L
    return L


def kvp_last_error() -> str:
    return lib().kvp_last_error().decode()


def kvp_version() -> str:
    return lib().kvp_version().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise KVPError(rc, kvp_last_error())


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    return int(t.data_ptr())


def _ptr_array(tensors: Sequence) -> "C.Array":
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = _ptr(t)
    return arr


def _shape(m) -> ModelShape:
    sh = ModelShape(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn_dim)
    keep = []
    for f in ("layer_n_q_heads", "layer_n_kv_heads", "layer_ffn_dim"):   # layers of different width (optional)
        v = getattr(m, f, None)
        if v is not None:
            arr = (C.c_int32 * len(v))(*v)
            keep.append(arr)
            setattr(sh, f, C.cast(arr, C.POINTER(C.c_int32)))
    sh._keep = keep            # the arrays are copied by kvp_load_weights; alive until then
    return sh


def _config(cfg, max_batch: int, max_seq: int) -> Config:
    """kvp_config for an object with the fields of kvp_synth.KVPConfig (the arrays it points to stay
    alive as attributes of the returned structure)."""
    c = Config()
    sb, sa = _shape(cfg.base), _shape(cfg.aux)
    c.base, c.aux = sb, sa
    c.vocab = cfg.vocab
    c.dtype = DTYPE_F32 if cfg.dtype == "fp32" else DTYPE_BF16
    c.rope_theta, c.rms_eps = cfg.rope_theta, cfg.rms_eps
    lm = (C.c_int32 * len(cfg.layer_map))(*cfg.layer_map)
    c.layer_map = C.cast(lm, C.POINTER(C.c_int32))
    c.max_batch, c.max_seq = max_batch, max_seq
    c._keep = (sb, sa, lm)
    return c


def kvp_debug_plan(cfg, B: int, T: int, max_batch: Optional[int] = None, max_seq: Optional[int] = None):
    """The workspace plan of a B x T call, computed on the host (no GPU needed): returns
    (regions, total_bytes) with regions = [(name, offset, bytes, bytes_touched), ...] in address order."""
    c = _config(cfg, max_batch or B, max_seq or T)
    n, total = C.c_int32(), C.c_uint64()
    _check(lib().kvp_debug_plan(C.byref(c), B, T, None, 0, C.byref(n), C.byref(total)))
    arr = (PlanRegion * n.value)()
    _check(lib().kvp_debug_plan(C.byref(c), B, T, arr, n.value, C.byref(n), C.byref(total)))
    return [(r.name.decode(), int(r.offset), int(r.bytes), int(r.bytes_touched)) for r in arr], int(total.value)


def kvp_load_weights(cfg, tensors: Mapping[str, "object"], max_batch: int, max_seq: int) -> int:
    """cfg: an object with the fields of kvp_synth.KVPConfig; tensors: name -> contiguous device
    tensor in the configuration's dtype (names as in kvp_synth.tensor_specs; the auxiliary
    final_norm / lm_head and the base wk / wv may be absent).  Returns the opaque handle."""
    def model(side: str, m) -> ModelWeights:
        mw = ModelWeights()
        mw.embed = _ptr(tensors.get(f"{side}.embed"))
        mw.final_norm = _ptr(tensors.get(f"{side}.final_norm"))
        mw.lm_head = _ptr(tensors.get(f"{side}.lm_head"))
        keep = []
        for f in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down", "q_norm", "k_norm"):
            ts = [tensors.get(f"{side}.L{l}.{f}") for l in range(m.n_layers)]
            if all(t is None for t in ts):
                setattr(mw, f, None)
                continue
            arr = _ptr_array(ts)
            keep.append(arr)
            setattr(mw, f, C.cast(arr, PP))
        mw._keep = keep
        return mw

    c = _config(cfg, max_batch, max_seq)
    w = Weights()
    w.base, w.aux = model("base", cfg.base), model("aux", cfg.aux)
    pk = _ptr_array([tensors.get(f"pred.L{i}.wk") for i in range(cfg.base.n_layers)])
    pv = _ptr_array([tensors.get(f"pred.L{i}.wv") for i in range(cfg.base.n_layers)])
    w.pred_wk, w.pred_wv = C.cast(pk, PP), C.cast(pv, PP)
    h = C.c_void_p()
    _check(lib().kvp_load_weights(C.byref(c), C.byref(w), C.byref(h)))
    return h.value


def kvp_workspace_bytes(handle: int, B: int, T: int) -> int:
    return int(lib().kvp_workspace_bytes(handle, B, T))


def kvp_run_stages(handle: int, stages: int, tokens, B: int, T: int, k_cache, v_cache, T_cap: int, logits, argmax,
                   workspace, stream: int = 0) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().kvp_run_stages(handle, stages, _ptr(tokens), B, T, _ptr(k_cache), _ptr(v_cache), T_cap,
                                _ptr(logits), _ptr(argmax), _ptr(workspace), ws_bytes, stream))


def kvp_prefill_predict(handle: int, tokens, B: int, T: int, k_cache, v_cache, T_cap: int, logits, argmax,
                        workspace, stream: int = 0) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().kvp_prefill_predict(handle, _ptr(tokens), B, T, _ptr(k_cache), _ptr(v_cache), T_cap,
                                     _ptr(logits), _ptr(argmax), _ptr(workspace), ws_bytes, stream))


def kvp_reference_workspace_bytes(handle: int, model: int, B: int, T: int) -> int:
    return int(lib().kvp_reference_workspace_bytes(handle, model, B, T))


def kvp_reference_prefill(handle: int, model: int, tokens, B: int, T: int, k_cache, v_cache, T_cap: int, logits,
                          argmax, workspace, stream: int = 0) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().kvp_reference_prefill(handle, model, _ptr(tokens), B, T, _ptr(k_cache), _ptr(v_cache), T_cap,
                                       _ptr(logits), _ptr(argmax), _ptr(workspace), ws_bytes, stream))


def kvp_generation_workspace_bytes(handle: int, B: int, T_total: int) -> int:
    return int(lib().kvp_generation_workspace_bytes(handle, B, T_total))


def kvp_generation_step(handle: int, tokens, B: int, pos: int, k_cache, v_cache, T_cap: int, logits, argmax,
                        workspace, stream: int = 0) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().kvp_generation_step(handle, _ptr(tokens), B, pos, _ptr(k_cache), _ptr(v_cache), T_cap,
                                     _ptr(logits), _ptr(argmax), _ptr(workspace), ws_bytes, stream))


def kvp_generation_step_static(handle: int, tokens, B: int, pos: int, k_cache, v_cache, T_cap: int, logits, argmax,
                               stream: int = 0) -> None:
    _check(lib().kvp_generation_step_static(handle, _ptr(tokens), B, pos, _ptr(k_cache), _ptr(v_cache), T_cap,
                                            _ptr(logits), _ptr(argmax), stream))


def kvp_static_scratch_bytes() -> int:
    return int(lib().kvp_static_scratch_bytes())


def kvp_check_flags(handle: int, clear: bool = False) -> int:
    v = C.c_uint32()
    _check(lib().kvp_check_flags(handle, C.byref(v), 1 if clear else 0))
    return int(v.value)


def kvp_debug_flash_guard(limit: float) -> None:
    """Sets the overflow guard of the attention kernels' fixed-reference softmax for the process (<= 0: default)."""
    lib().kvp_debug_flash_guard(limit)


def kvp_probe_mfma(sink, iters: int, stream: int = 0) -> float:
    """Enqueues the matrix-core probe; returns the floating-point operations it performs."""
    f = C.c_double()
    rc = lib().kvp_probe_mfma(_ptr(sink), iters, C.byref(f), stream)
    if rc != 0:
        raise KVPError(rc, "kvp_probe_mfma")
    return float(f.value)


def kvp_probe_stream(kind: int, src, dst, nbytes: int, stream: int = 0) -> None:
    """Enqueues a streaming probe over nbytes: kind 0 read src, 1 copy src -> dst, 2 fill dst."""
    rc = lib().kvp_probe_stream(kind, _ptr(src), _ptr(dst), nbytes, stream)
    if rc != 0:
        raise KVPError(rc, "kvp_probe_stream")


def kvp_free(handle: int) -> None:
    lib().kvp_free(handle)


class KVP:
    """Convenience owner of a handle plus the caller-side buffers (torch tensors) for one
    maximum batch shape.  All compute happens in libkvp."""

    def __init__(self, cfg, tensors: Mapping[str, "object"], max_batch: Optional[int] = None,
                 max_seq: Optional[int] = None, T_cap: Optional[int] = None):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.max_batch = max_batch or cfg.batch
        self.max_seq = max_seq or cfg.seq_len
        self.T_cap = T_cap or self.max_seq
        self.tensors = dict(tensors)          # keeps the device weights alive
        self.dtype = torch.float32 if cfg.dtype == "fp32" else torch.bfloat16
        self.handle = kvp_load_weights(cfg, self.tensors, self.max_batch, self.max_seq)
        dev = "cuda"
        b = cfg.base
        self.k_cache = torch.zeros((b.n_layers, self.max_batch, b.n_kv_heads, self.T_cap, b.head_dim), dtype=self.dtype, device=dev)
        self.v_cache = torch.zeros_like(self.k_cache)
        self.logits = torch.empty((self.max_batch, cfg.vocab), dtype=torch.float32, device=dev)
        self.argmax = torch.empty((self.max_batch,), dtype=torch.int32, device=dev)
        # the size is non-decreasing in T but not in B (the attention splits per sequence shrink as B grows): one
        # buffer for every batch size up to max_batch takes the maximum over them
        nbytes = max(kvp_workspace_bytes(self.handle, b, self.max_seq) for b in range(1, self.max_batch + 1))
        if nbytes == 0:
            raise KVPError(-3, "workspace size query failed")
        self.workspace = torch.empty((nbytes + 255) // 256 * 256, dtype=torch.uint8, device=dev)

    def caches(self, B: int):
        """Views [L_B, B, n_kv, T_cap, hd] of the caches as laid out for a batch of B."""
        b = self.cfg.base
        n = b.n_layers * B * b.n_kv_heads * self.T_cap * b.head_dim
        shape = (b.n_layers, B, b.n_kv_heads, self.T_cap, b.head_dim)
        return self.k_cache.view(-1)[:n].view(shape), self.v_cache.view(-1)[:n].view(shape)

    def cache_layer(self, i: int, B: int):
        """Dense views [B, n_kv_i, T_cap, hd] of base layer i's keys and values (layers of different
        width occupy the start of equally sized blocks)."""
        b = self.cfg.base
        nkv = b.layer_n_kv_heads[i] if getattr(b, "layer_n_kv_heads", None) else b.n_kv_heads
        block = B * b.n_kv_heads * self.T_cap * b.head_dim
        n = B * nkv * self.T_cap * b.head_dim
        shape = (B, nkv, self.T_cap, b.head_dim)
        return (self.k_cache.view(-1)[i * block: i * block + n].view(shape),
                self.v_cache.view(-1)[i * block: i * block + n].view(shape))

    def run(self, tokens, stages: int = STAGE_ALL, stream: Optional[int] = None):
        """tokens: device int32 [B, T].  Enqueues the path on the current torch stream."""
        B, T = tokens.shape
        s = self.torch.cuda.current_stream().cuda_stream if stream is None else stream
        kvp_run_stages(self.handle, stages, tokens, B, T, self.k_cache, self.v_cache, self.T_cap, self.logits,
                       self.argmax, self.workspace, s)

    def reference(self, tokens, model: int = MODEL_BASE, keep_cache: bool = False, stream: Optional[int] = None):
        """Ordinary inference of one model alone (kvp_reference_prefill) on tokens [B, T].  Logits and
        first tokens land in self.logits / self.argmax; with keep_cache returns (K, V) of that
        model, [L, B, n_kv, T, hd].  Buffers are created on first use and reused."""
        torch = self.torch
        B, T = tokens.shape
        m = self.cfg.base if model == MODEL_BASE else self.cfg.aux
        nbytes = kvp_reference_workspace_bytes(self.handle, model, B, T)
        if nbytes == 0:
            raise KVPError(-3, "reference workspace size query failed")
        ws = getattr(self, "_ref_ws", None)
        if ws is None or ws.numel() < nbytes:
            ws = self._ref_ws = torch.empty((nbytes + 255) // 256 * 256, dtype=torch.uint8, device="cuda")
        kc = vc = None
        if keep_cache:
            kc = torch.zeros((m.n_layers, B, m.n_kv_heads, T, m.head_dim), dtype=self.dtype, device="cuda")
            vc = torch.zeros_like(kc)
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        kvp_reference_prefill(self.handle, model, tokens, B, T, kc, vc, T, self.logits, self.argmax, ws, s)
        return kc, vc

    def generation_step(self, tokens, pos: int, stream: Optional[int] = None):
        """One pass of the generation loop (kvp_generation_step): tokens int32 [B] on the device are fed
        at position pos; the caches of this object grow by one entry, logits / argmax are updated.
        The object must have been created with max_seq and T_cap >= pos + 1."""
        B = tokens.shape[0]
        s = self.torch.cuda.current_stream().cuda_stream if stream is None else stream
        kvp_generation_step(self.handle, tokens, B, pos, self.k_cache, self.v_cache, self.T_cap, self.logits,
                            self.argmax, self.workspace, s)

    def check_flags(self, clear: bool = False) -> int:
        """KVP_FLAG_* bits set by the kernels of earlier calls (synchronise first)."""
        return kvp_check_flags(self.handle, clear)

    def aux_cache_layer(self, l: int, B: int, T: int):
        """Dense views [B*T, n_kv_l*hd] of auxiliary layer l's keys and values in the workspace
        (layers of different width occupy the start of equally sized blocks)."""
        ko, vo = C.c_size_t(), C.c_size_t()
        _check(lib().kvp_aux_cache_offsets(self.handle, B, T, C.byref(ko), C.byref(vo)))
        a = self.cfg.aux
        nkv = a.layer_n_kv_heads[l] if getattr(a, "layer_n_kv_heads", None) else a.n_kv_heads
        es = 4 if self.cfg.dtype == "fp32" else 2
        block, n = B * T * a.kv_dim * es, B * T * nkv * a.head_dim * es
        k = self.workspace[ko.value + l * block: ko.value + l * block + n].view(self.dtype).view(B * T, nkv * a.head_dim)
        v = self.workspace[vo.value + l * block: vo.value + l * block + n].view(self.dtype).view(B * T, nkv * a.head_dim)
        return k, v

    def aux_cache(self, B: int, T: int):
        """Views of the auxiliary cache left in the workspace: K_A, V_A [L_A, B*T, n_kv_a*hd]
        (stacks with one width per layer; see aux_cache_layer otherwise)."""
        if getattr(self.cfg.aux, "layer_n_kv_heads", None):
            raise ValueError("layers of different width: use aux_cache_layer")
        ko, vo = C.c_size_t(), C.c_size_t()
        _check(lib().kvp_aux_cache_offsets(self.handle, B, T, C.byref(ko), C.byref(vo)))
        a = self.cfg.aux
        n = a.n_layers * B * T * a.kv_dim
        es = 4 if self.cfg.dtype == "fp32" else 2
        k = self.workspace[ko.value: ko.value + n * es].view(self.dtype).view(a.n_layers, B * T, a.kv_dim)
        v = self.workspace[vo.value: vo.value + n * es].view(self.dtype).view(a.n_layers, B * T, a.kv_dim)
        return k, v

    def profile(self, on: bool) -> None:
        _check(lib().kvp_profile_enable(self.handle, 1 if on else 0))
        _check(lib().kvp_profile_reset(self.handle))

    def profile_read(self) -> Dict[str, Dict[str, float]]:
        ms = (C.c_double * len(KERNEL_CLASSES))()
        n = (C.c_int64 * len(KERNEL_CLASSES))()
        _check(lib().kvp_profile_read(self.handle, ms, n))
        return {k: {"ms": ms[i], "launches": int(n[i])} for i, k in enumerate(KERNEL_CLASSES)}

    def close(self) -> None:
        if self.handle:
            kvp_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
