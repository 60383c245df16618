"""ctypes binding of libhe.so (include/he.h): argument marshalling only.

Every step of the generation path runs inside the library's HIP kernels;
torch is used here to own device memory and to name the stream.  There is no
CPU fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhe.so")

HE_OK = 0
HE_ERR_INVALID_ARG, HE_ERR_SHAPE, HE_ERR_CAPACITY, HE_ERR_OOM, HE_ERR_DEVICE, HE_ERR_STATE = 1, 2, 3, 4, 5, 6
STATUS_NAMES = {0: "HE_OK", 1: "HE_ERR_INVALID_ARG", 2: "HE_ERR_SHAPE", 3: "HE_ERR_CAPACITY", 4: "HE_ERR_OOM",
                5: "HE_ERR_DEVICE", 6: "HE_ERR_STATE"}
HE_F32, HE_BF16 = 0, 1


class he_config(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("hidden", C.c_int), ("n_heads", C.c_int), ("ffn", C.c_int),
                ("vocab", C.c_int), ("max_positions", C.c_int), ("pos_offset", C.c_int), ("ln_eps", C.c_float),
                ("dtype", C.c_int), ("max_batch", C.c_int), ("max_seq_len", C.c_int), ("device", C.c_int),
                ("stream", C.c_void_p), ("impl", C.c_int), ("weights_tiled", C.c_int), ("weights_fp8", C.c_int)]


class he_lora(C.Structure):
    _fields_ = [("a", C.c_void_p), ("b", C.c_void_p)]


class he_lora_layer(C.Structure):
    _fields_ = [("wqkv", he_lora), ("wo", he_lora), ("w1", he_lora), ("w2", he_lora)]


LAYER_FIELDS = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


class he_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_FIELDS]


class he_weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("pos_emb", C.c_void_p), ("lnf_g", C.c_void_p), ("lnf_b", C.c_void_p),
                ("lm_head", C.c_void_p), ("layers", C.POINTER(he_layer_weights))]


class he_scratch_account(C.Structure):
    _fields_ = [("scratch_floats", C.c_size_t), ("scratch_reserved", C.c_size_t), ("static_floats", C.c_size_t),
                ("counters", C.c_int), ("counters_reserved", C.c_int), ("stat_pairs", C.c_int),
                ("stat_pairs_reserved", C.c_int), ("ksplit", C.c_int)]


class he_sampling(C.Structure):
    _fields_ = [("mode", C.c_int), ("temperature", C.c_float), ("seed", C.c_uint64)]


class HeError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Loads libhe.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2308_01320_amd.build` "
                           "(or __graft_entry__.build()); the engine has no other implementation")
    L = C.CDLL(LIB_PATH)
    vp, ip, fp = C.c_void_p, C.c_void_p, C.c_void_p
    L.he_workspace_bytes.restype = C.c_size_t
    L.he_workspace_bytes.argtypes = [C.POINTER(he_config)]
    L.he_create.restype = C.c_int
    L.he_create.argtypes = [C.POINTER(he_config), C.POINTER(he_weights), C.POINTER(vp)]
    L.he_refresh_weights.restype = C.c_int
    L.he_refresh_weights.argtypes = [vp]
    L.he_prefill.restype = C.c_int
    L.he_prefill.argtypes = [vp, ip, C.c_int, C.c_int, C.POINTER(he_sampling), ip, fp, fp]
    L.he_decode_step.restype = C.c_int
    L.he_decode_step.argtypes = [vp, ip, C.POINTER(he_sampling), ip, fp, fp]
    L.he_decode_step_static.restype = C.c_int
    L.he_decode_step_static.argtypes = [vp, ip, C.POINTER(he_sampling), ip, fp, fp]
    L.he_generate.restype = C.c_int
    L.he_generate.argtypes = [vp, ip, C.c_int, C.c_int, C.c_int, C.POINTER(he_sampling), ip, fp]
    L.he_prefill_ragged.restype = C.c_int
    L.he_prefill_ragged.argtypes = [vp, ip, ip, C.c_int, C.c_int, C.POINTER(he_sampling), ip, fp, fp]
    L.he_generate_ragged.restype = C.c_int
    L.he_generate_ragged.argtypes = [vp, ip, ip, C.c_int, C.c_int, C.c_int, C.POINTER(he_sampling), C.c_int, C.c_int, ip, fp, ip]
    L.he_refresh_weights_lora.restype = C.c_int
    L.he_refresh_weights_lora.argtypes = [vp, C.POINTER(he_lora_layer), C.c_int, C.c_float]
    L.he_release_arena.restype = C.c_int
    L.he_release_arena.argtypes = [vp]
    L.he_acquire_arena.restype = C.c_int
    L.he_acquire_arena.argtypes = [vp]
    L.he_score.restype = C.c_int
    L.he_score.argtypes = [vp, ip, C.c_int, C.c_int, fp]
    L.he_reset.restype = C.c_int
    L.he_reset.argtypes = [vp]
    L.he_destroy.restype = C.c_int
    L.he_destroy.argtypes = [vp]
    L.he_last_error.restype = C.c_char_p
    L.he_last_error.argtypes = [vp]
    L.he_cache_len.restype = C.c_int
    L.he_cache_len.argtypes = [vp]
    L.he_timing_enable.restype = C.c_int
    L.he_timing_enable.argtypes = [vp, C.c_int]
    L.he_timing_read.restype = C.c_int
    L.he_timing_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_long), C.c_int]
    L.he_tiled_bytes.restype = C.c_size_t
    L.he_tiled_bytes.argtypes = [C.c_int, C.c_int]
    L.he_tile_matrix.restype = C.c_int
    L.he_tile_matrix.argtypes = [vp, vp, C.c_int, C.c_int, vp]
    L.he_tile_matrix_lora.restype = C.c_int
    L.he_tile_matrix_lora.argtypes = [vp, vp, C.c_int, C.c_int, vp, vp, C.c_int, C.c_float, vp]
    L.he_fp8_quantize_rows.restype = C.c_int
    L.he_fp8_quantize_rows.argtypes = [vp, C.c_int, C.c_int, vp, vp, vp, vp]
    L.he_plan_decode_gemm.restype = C.c_int
    L.he_plan_decode_gemm.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_size_t, C.c_int, C.POINTER(C.c_int),
                                      C.POINTER(C.c_int), C.POINTER(C.c_int)]
    L.he_decode_scratch_account.restype = C.c_int
    L.he_decode_scratch_account.argtypes = [C.POINTER(he_config), C.c_int, C.c_int, C.c_int, C.POINTER(he_scratch_account)]
    L.he_arrival_counters_nonzero.restype = C.c_int
    L.he_arrival_counters_nonzero.argtypes = [vp, C.POINTER(C.c_int)]
    L.he_last_step_rows.restype = C.c_int
    L.he_last_step_rows.argtypes = [vp]
    L.he_plan_prompt_gemm.restype = C.c_int
    L.he_plan_prompt_gemm.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_size_t, C.c_int, C.POINTER(C.c_int),
                                      C.POINTER(C.c_int), C.POINTER(C.c_int)]
    L.he_kernel_sweep.restype = C.c_int
    L.he_kernel_sweep.argtypes = [vp, C.c_int, C.c_int]
    L.he_calibration_copy.restype = C.c_int
    L.he_calibration_copy.argtypes = [vp, vp, C.c_size_t, vp]
    L.he_rng_words.restype = C.c_int
    L.he_rng_words.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int, vp, vp]
    _lib = L
    return L


EXPORTS = ("he_workspace_bytes", "he_create", "he_refresh_weights", "he_prefill", "he_decode_step", "he_generate",
           "he_reset", "he_destroy", "he_last_error", "he_cache_len", "he_rng_words", "he_timing_enable",
           "he_timing_read", "he_calibration_copy", "he_kernel_sweep", "he_tiled_bytes",
           "he_tile_matrix", "he_score", "he_prefill_ragged",
           "he_generate_ragged", "he_refresh_weights_lora", "he_release_arena", "he_acquire_arena",
           "he_tile_matrix_lora", "he_plan_decode_gemm", "he_fp8_quantize_rows", "he_decode_step_static",
           "he_decode_scratch_account", "he_arrival_counters_nonzero", "he_last_step_rows",
           "he_plan_prompt_gemm")

KERNEL_CLASSES = ("layernorm", "qkv", "attention", "out_proj", "fc1", "fc2", "lm_head", "empty")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def sampling(mode: str = "greedy", temperature: float = 1.0, seed: int = 0) -> he_sampling:
    return he_sampling({"greedy": 0, "gumbel": 1}[mode], float(temperature), int(seed) & 0xFFFFFFFFFFFFFFFF)


def make_config(dims, max_batch=None, max_seq_len=None, device=0, stream=None, impl=0, weights_tiled=0,
                weights_fp8=0) -> he_config:
    """he_config from a synth.ModelDims (or anything with the same fields)."""
    return he_config(dims.n_layers, dims.hidden, dims.n_heads, dims.ffn, dims.vocab, dims.max_positions,
                     dims.pos_offset, dims.ln_eps, HE_BF16 if dims.dtype == "bf16" else HE_F32,
                     max_batch or dims.batch, max_seq_len or (dims.prompt_len + dims.gen_len), device,
                     stream, impl, weights_tiled, weights_fp8)


def upload_weights(w: dict, dtype: str, device="cuda:0") -> dict:
    """numpy weight dict (synth.make_weights) -> same structure of device tensors."""
    import torch
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32

    def up(a):
        return torch.from_numpy(a).to(device=device, dtype=tdt).contiguous()

    out = {k: up(v) for k, v in w.items() if k not in ("layers", "lm_head")}
    out["lm_head"] = out["tok_emb"] if w["lm_head"] is w["tok_emb"] else up(w["lm_head"])
    out["layers"] = [{k: up(v) for k, v in lw.items()} for lw in w["layers"]]
    return out


class Engine:
    """Owns one he_engine handle and keeps the borrowed weight tensors alive."""

    def __init__(self, cfg: he_config, weights: dict):
        import torch
        self._torch = torch
        self.cfg = cfg
        self.weights = weights  # device tensors; the engine borrows their memory
        self._layers = (he_layer_weights * max(1, cfg.n_layers))()
        for i, lw in enumerate(weights["layers"]):
            for n in LAYER_FIELDS:
                setattr(self._layers[i], n, lw[n].data_ptr())
        self._w = he_weights(weights["tok_emb"].data_ptr(), weights["pos_emb"].data_ptr(),
                             weights["lnf_g"].data_ptr(), weights["lnf_b"].data_ptr(),
                             weights["lm_head"].data_ptr(), self._layers)
        self.handle = C.c_void_p()
        rc = lib().he_create(C.byref(cfg), C.byref(self._w), C.byref(self.handle))
        if rc != HE_OK:
            self.handle = None
            raise HeError(rc, (lib().he_last_error(None) or b"").decode())
        self.device = torch.device("cuda", cfg.device)

    # -- helpers
    def _check(self, rc):
        if rc != HE_OK:
            raise HeError(rc, (lib().he_last_error(self.handle) or b"").decode())

    def last_error(self) -> str:
        return (lib().he_last_error(self.handle) or b"").decode()

    def he_last_step_rows(self) -> int:
        return lib().he_last_step_rows(self.handle)

    def cache_len(self) -> int:
        return lib().he_cache_len(self.handle)

    # -- the ABI calls, same names
    def he_prefill(self, prompt_ids, samp: he_sampling, want_logits=False):
        t = self._torch
        B, S = prompt_ids.shape
        ids = t.empty(B, dtype=t.int32, device=self.device)
        lp = t.empty(B, dtype=t.float32, device=self.device)
        lg = t.empty(B, self.cfg.vocab, dtype=t.float32, device=self.device) if want_logits else None
        self._check(lib().he_prefill(self.handle, prompt_ids.data_ptr(), B, S, C.byref(samp), ids.data_ptr(),
                                     lp.data_ptr(), _ptr(lg)))
        return ids, lp, lg

    def he_prefill_ragged(self, prompt_ids, prompt_lens, samp: he_sampling, want_logits=False):
        t = self._torch
        B, S = prompt_ids.shape
        ids = t.empty(B, dtype=t.int32, device=self.device)
        lp = t.empty(B, dtype=t.float32, device=self.device)
        lg = t.empty(B, self.cfg.vocab, dtype=t.float32, device=self.device) if want_logits else None
        self._check(lib().he_prefill_ragged(self.handle, prompt_ids.data_ptr(), prompt_lens.data_ptr(), B, S,
                                            C.byref(samp), ids.data_ptr(), lp.data_ptr(), _ptr(lg)))
        return ids, lp, lg

    def he_generate_ragged(self, prompt_ids, prompt_lens, G: int, samp: he_sampling, eos_id: int, pad_id: int):
        t = self._torch
        B, S = prompt_ids.shape
        out_ids = t.empty(B, G, dtype=t.int32, device=self.device)
        out_lp = t.empty(B, G, dtype=t.float32, device=self.device)
        out_lens = t.empty(B, dtype=t.int32, device=self.device)
        self._check(lib().he_generate_ragged(self.handle, prompt_ids.data_ptr(), prompt_lens.data_ptr(), B, S, G,
                                             C.byref(samp), eos_id, pad_id, out_ids.data_ptr(), out_lp.data_ptr(),
                                             out_lens.data_ptr()))
        return out_ids, out_lp, out_lens

    def he_decode_step(self, in_ids, samp: he_sampling, want_logits=False):
        t = self._torch
        B = in_ids.shape[0]
        ids = t.empty(B, dtype=t.int32, device=self.device)
        lp = t.empty(B, dtype=t.float32, device=self.device)
        lg = t.empty(B, self.cfg.vocab, dtype=t.float32, device=self.device) if want_logits else None
        self._check(lib().he_decode_step(self.handle, in_ids.data_ptr(), C.byref(samp), ids.data_ptr(),
                                         lp.data_ptr(), _ptr(lg)))
        return ids, lp, lg

    def he_decode_step_static(self, in_ids, samp: he_sampling, want_logits=False):
        t = self._torch
        B = in_ids.shape[0]
        ids = t.empty(B, dtype=t.int32, device=self.device)
        lp = t.empty(B, dtype=t.float32, device=self.device)
        lg = t.empty(B, self.cfg.vocab, dtype=t.float32, device=self.device) if want_logits else None
        self._check(lib().he_decode_step_static(self.handle, in_ids.data_ptr(), C.byref(samp), ids.data_ptr(),
                                                lp.data_ptr(), _ptr(lg)))
        return ids, lp, lg

    def he_generate(self, prompt_ids, G: int, samp: he_sampling, out_ids=None, out_lp=None):
        t = self._torch
        B, S = prompt_ids.shape
        if out_ids is None:
            out_ids = t.empty(B, G, dtype=t.int32, device=self.device)
        if out_lp is None:
            out_lp = t.empty(B, G, dtype=t.float32, device=self.device)
        self._check(lib().he_generate(self.handle, prompt_ids.data_ptr(), B, S, G, C.byref(samp),
                                      out_ids.data_ptr(), out_lp.data_ptr()))
        return out_ids, out_lp

    def he_score(self, ids, out_lp=None):
        t = self._torch
        B, T = ids.shape
        if out_lp is None:
            out_lp = t.empty(B, T - 1, dtype=t.float32, device=self.device)
        self._check(lib().he_score(self.handle, ids.data_ptr(), B, T, out_lp.data_ptr()))
        return out_lp

    def he_reset(self):
        self._check(lib().he_reset(self.handle))

    def he_refresh_weights(self):
        self._check(lib().he_refresh_weights(self.handle))

    def he_refresh_weights_lora(self, adapters, rank: int, scale: float):
        """adapters: per layer a dict {"wqkv"|"wo"|"w1"|"w2": (A, B)} of bf16 device tensors A [rank,in], B [out,rank]."""
        arr = (he_lora_layer * len(adapters))()
        for l, ad in enumerate(adapters):
            for name, (a, b) in ad.items():
                getattr(arr[l], name).a = a.data_ptr()
                getattr(arr[l], name).b = b.data_ptr()
        self._check(lib().he_refresh_weights_lora(self.handle, arr, rank, scale))

    def he_release_arena(self):
        self._check(lib().he_release_arena(self.handle))

    def he_acquire_arena(self):
        self._check(lib().he_acquire_arena(self.handle))

    def he_timing_enable(self, on: bool):
        self._check(lib().he_timing_enable(self.handle, 1 if on else 0))

    def he_timing_read(self) -> dict:
        n = len(KERNEL_CLASSES)
        ms = (C.c_double * n)()
        cnt = (C.c_long * n)()
        self._check(lib().he_timing_read(self.handle, ms, cnt, n))
        return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_CLASSES)}

    def he_arrival_counters_nonzero(self) -> int:
        n = C.c_int()
        self._check(lib().he_arrival_counters_nonzero(self.handle, C.byref(n)))
        return n.value

    def he_kernel_sweep(self, kernel_class: str, reps: int = 1):
        self._check(lib().he_kernel_sweep(self.handle, KERNEL_CLASSES.index(kernel_class), reps))

    def he_destroy(self):
        if self.handle:
            lib().he_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.he_destroy()
        except Exception:
            pass


def he_rng_words(seed: int, b: int, n: int, v0: int, count: int, device="cuda:0"):
    import torch
    out = torch.empty(count, dtype=torch.int32, device=device)
    rc = lib().he_rng_words(int(seed) & 0xFFFFFFFFFFFFFFFF, b, n, v0, count, out.data_ptr(),
                            torch.cuda.current_stream().cuda_stream)
    if rc != HE_OK:
        raise HeError(rc, "he_rng_words")
    return out


def he_calibration_copy(src, dst, stream=None):
    """Plain copy kernel of known size (src -> dst, equal-sized device tensors)."""
    nbytes = src.numel() * src.element_size()
    rc = lib().he_calibration_copy(src.data_ptr(), dst.data_ptr(), nbytes, stream)
    if rc != HE_OK:
        raise HeError(rc, "he_calibration_copy")
    return nbytes


def he_tile_matrix(src, stream=None):
    """Tiled copy (uint8 tensor of he_tiled_bytes) of a row-major bf16 [rows, cols] device tensor."""
    import torch
    rows, cols = src.shape
    n = lib().he_tiled_bytes(rows, cols)
    if n == 0:
        raise HeError(1, "he_tiled_bytes: bad shape")
    dst = torch.empty(n, dtype=torch.uint8, device=src.device)
    rc = lib().he_tile_matrix(src.data_ptr(), dst.data_ptr(), rows, cols, stream)
    if rc != HE_OK:
        raise HeError(rc, "he_tile_matrix")
    return dst


def he_fp8_quantize_rows(src, stream=None):
    """(codes uint8 [rows, cols], exponents int32 [rows], scales float32 [rows]) of a bf16 [rows, cols] device tensor."""
    import torch
    rows, cols = src.shape
    codes = torch.empty(rows, cols, dtype=torch.uint8, device=src.device)
    exps = torch.empty(rows, dtype=torch.int32, device=src.device)
    scales = torch.empty(rows, dtype=torch.float32, device=src.device)
    rc = lib().he_fp8_quantize_rows(src.data_ptr(), rows, cols, codes.data_ptr(), exps.data_ptr(), scales.data_ptr(), stream)
    if rc != HE_OK:
        raise HeError(rc, "he_fp8_quantize_rows")
    return codes, exps, scales


def he_plan_decode_gemm(M, N, K, ksplit_allowed=False, scratch_floats=0, cus=256):
    """(rows per unit, units per workgroup, k-splits) of a decode-shaped GEMM; host logic only."""
    u, n, k = C.c_int(), C.c_int(), C.c_int()
    rc = lib().he_plan_decode_gemm(M, N, K, 1 if ksplit_allowed else 0, scratch_floats, cus, C.byref(u), C.byref(n), C.byref(k))
    if rc != HE_OK:
        raise HeError(rc, "he_plan_decode_gemm")
    return u.value, n.value, k.value


def he_plan_prompt_gemm(M, N, K, may_cut=False, scratch_floats=0, cus=256):
    """(tile columns, k ranges, first cut column) of a prompt-pass GEMM; host logic only."""
    t, k, c = C.c_int(), C.c_int(), C.c_int()
    rc = lib().he_plan_prompt_gemm(M, N, K, 1 if may_cut else 0, scratch_floats, cus, C.byref(t), C.byref(k), C.byref(c))
    if rc != HE_OK:
        raise HeError(rc, "he_plan_prompt_gemm")
    return t.value, k.value, c.value


def he_decode_scratch_account(cfg: he_config, B: int, which: int, cus: int = 256) -> he_scratch_account:
    """What the k-split GEMM (which = 0 out-projection, 1 FC2) of a B-row decode step indexes; host logic only."""
    out = he_scratch_account()
    rc = lib().he_decode_scratch_account(C.byref(cfg), B, which, cus, C.byref(out))
    if rc != HE_OK:
        raise HeError(rc, "he_decode_scratch_account")
    return out


def he_tile_matrix_lora(src, a, b, scale, stream=None):
    """Tiled copy of bf16(src + scale * b @ a): src [rows, cols], a [rank, cols], b [rows, rank], bf16 device tensors."""
    import torch
    rows, cols = src.shape
    dst = torch.empty(lib().he_tiled_bytes(rows, cols), dtype=torch.uint8, device=src.device)
    rc = lib().he_tile_matrix_lora(src.data_ptr(), dst.data_ptr(), rows, cols, a.data_ptr(), b.data_ptr(), a.shape[0],
                                   scale, stream)
    if rc != HE_OK:
        raise HeError(rc, "he_tile_matrix_lora")
    return dst


TILED_KINDS = ("wqkv", "wo", "w1", "w2")


def tile_weights_in_place(weights: dict) -> dict:
    """Replaces the GEMM matrices of a device weight dict by their tiled forms, one at a time, so that
    at most one matrix exists twice (for he_config.weights_tiled = 1)."""
    import torch
    out = dict(weights)
    out["layers"] = []
    for lw in weights["layers"]:
        nl = dict(lw)
        for k in TILED_KINDS:
            nl[k] = he_tile_matrix(lw[k])
            torch.cuda.synchronize()
            lw[k] = None
        out["layers"].append(nl)
    out["lm_head"] = he_tile_matrix(weights["lm_head"])
    torch.cuda.synchronize()
    return out
