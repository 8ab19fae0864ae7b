"""ctypes binding of include/rollout.h.  Function and struct names follow the C header.

PyTorch appears here only as the owner of device memory (weights are uploaded as torch
tensors and their data pointers handed to rollout_init) and of the stream.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librollout.so")

OK, E_INVAL, E_NOMEM, E_HIP, E_STATE = 0, -1, -2, -3, -4
DTYPE_F32, DTYPE_BF16 = 0, 1
RT_SIMPLE_KERNELS = 1
RT_RECORD_ROUTING = 2
RT_KERNEL_TIMING = 4
RT_PROMPT_GROUPS = 8
RT_GROW_PAGES = 16


class RolloutError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"rollout error {code}: {msg}")
        self.code = code


class rollout_model_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim",
                                         "ffn_dim", "vocab", "n_experts", "top_k", "expert_ffn_dim")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32), ("flags", C.c_uint32)]


class rollout_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("norm1", "wq", "wk", "wv", "wo", "norm2", "w_gate", "w_up",
                                          "w_down", "router", "bq", "bk", "bv", "q_norm", "k_norm")]


class rollout_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(rollout_layer_weights))]


class rollout_runtime_desc(C.Structure):
    _fields_ = [("kv_pool_bytes", C.c_size_t), ("page_tokens", C.c_int32), ("max_live_samples", C.c_int32),
                ("max_context", C.c_int32), ("max_batch_tokens", C.c_int32), ("hip_stream", C.c_void_p),
                ("seed", C.c_uint64), ("flags", C.c_uint32), ("timing_stride", C.c_uint32)]


class rollout_stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("decode_steps", "tokens_emitted", "prompts_prefilled",
                                          "prompt_tokens", "samples_admitted", "samples_finished",
                                          "samples_aborted")] + \
               [(n, C.c_int32) for n in ("live_samples", "pages_total", "pages_in_use", "pages_reserved",
                                         "pages_peak", "matrix_core_path")] + \
               [(n, C.c_double) for n in ("prefill_ms", "decode_ms", "extend_ms", "logprobs_ms")]


class rollout_queue_stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("prompts_pushed", "prompts_admitted", "prompts_completed",
                                          "samples_aborted", "prompts_preempted")] + \
               [("prompts_waiting", C.c_int32), ("closed", C.c_int32), ("prompts_pending", C.c_int32)]


class rollout_tensor_update(C.Structure):
    _fields_ = [("layer", C.c_int32), ("tensor", C.c_int32), ("data", C.c_void_p)]


W_IDS = {"embed": 0, "final_norm": 1, "lm_head": 2, "norm1": 3, "wq": 4, "wk": 5, "wv": 6, "wo": 7, "norm2": 8,
         "w_gate": 9, "w_up": 10, "w_down": 11, "router": 12, "bq": 13, "bk": 14, "bv": 15, "q_norm": 16,
         "k_norm": 17}
MODEL_QKV_BIAS, MODEL_QK_NORM, MODEL_TIED_LM_HEAD = 1, 2, 4


class rollout_loss_params(C.Structure):
    _fields_ = [(n, C.c_float) for n in ("gamma", "kl_coef", "reward_clip", "adv_clip", "eps_low", "eps_high")]


class rollout_kernel_stat(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("launches", C.c_uint64), ("ms", C.c_double), ("bytes", C.c_double),
                ("flops", C.c_double)]


# every symbol include/rollout.h declares: name -> (restype, argtypes)
_P = C.c_void_p
SIGNATURES = {
    "rollout_init": (C.c_int, [C.POINTER(_P), C.POINTER(rollout_model_desc), C.POINTER(rollout_weights),
                               C.POINTER(rollout_runtime_desc)]),
    "rollout_prefill": (C.c_int, [_P, C.c_int32, _P, _P, C.c_int32, _P, C.c_int32, C.c_float, C.c_float,
                                  _P, _P, _P, _P, _P, _P]),
    "rollout_live_samples": (C.c_int, [_P, C.c_int32, _P]),
    "rollout_decode_step": (C.c_int, [_P, _P, _P, C.POINTER(C.c_int32), _P, _P, _P, _P]),
    "rollout_logprobs": (C.c_int, [_P, C.c_int32, _P, _P, C.c_float, _P]),
    "rollout_abort": (C.c_int, [_P, C.c_int32, _P]),
    "rollout_update_weights": (C.c_int, [_P, C.c_int32, C.POINTER(rollout_tensor_update)]),
    "rollout_extend": (C.c_int, [_P, C.c_int32, _P, _P, _P, _P, _P, _P, _P, _P]),
    "rollout_queue_push": (C.c_int, [_P, C.c_int32, _P, _P, C.c_int32, _P, C.c_int32, C.c_float, C.c_float, _P]),
    "rollout_queue_policy": (C.c_int, [_P, C.c_int32, C.c_int32]),
    "rollout_queue_chunking": (C.c_int, [_P, C.c_int32]),
    "rollout_queue_step": (C.c_int, [_P, C.POINTER(C.c_int32), C.POINTER(C.c_int32), _P, _P, _P, _P]),
    "rollout_queue_get_stats": (C.c_int, [_P, C.POINTER(rollout_queue_stats)]),
    "rollout_debug_logits": (C.c_int, [_P, C.POINTER(C.c_int32), _P]),
    "rollout_debug_routing": (C.c_int, [_P, C.POINTER(C.c_int32), _P]),
    "rollout_get_stats": (C.c_int, [_P, C.POINTER(rollout_stats)]),
    "rollout_kernel_stats": (C.c_int, [_P, C.POINTER(C.c_int32), C.POINTER(rollout_kernel_stat)]),
    "rollout_last_error": (C.c_char_p, [_P]),
    "rollout_destroy": (None, [_P]),
    "rollout_abi_version": (C.c_int, []),
    "rollout_sample": (C.c_int, [_P, C.c_int32, C.c_int32, C.c_float, C.c_float, _P, _P, _P, _P, _P, _P]),
    "rollout_sample_static": (C.c_int, [_P, C.c_int32, C.c_int32, C.c_float, C.c_float, _P, _P, _P, _P, _P, _P]),
    "rollout_sample_static_prepare": (C.c_int, []),
    "rollout_sample_static_error": (C.c_char_p, []),
    "rollout_philox_words": (C.c_int, [C.c_uint64, C.c_int32, _P, _P, _P]),
    "rollout_policy_loss": (C.c_int, [C.c_int32, _P, _P, _P, _P, _P, _P, C.POINTER(rollout_loss_params), _P,
                                      C.POINTER(C.c_float), _P, _P]),
    "rollout_pool_create": (_P, [C.c_int32]),
    "rollout_pool_destroy": (None, [_P]),
    "rollout_pool_free_pages": (C.c_int32, [_P]),
    "rollout_pool_unreserved": (C.c_int32, [_P]),
    "rollout_pool_reserve": (C.c_int, [_P, C.c_int32]),
    "rollout_pool_unreserve": (None, [_P, C.c_int32]),
    "rollout_pool_alloc": (C.c_int32, [_P, C.c_int]),
    "rollout_pool_retain": (C.c_int, [_P, C.c_int32]),
    "rollout_pool_release": (C.c_int, [_P, C.c_int32]),
    "rollout_pool_refcount": (C.c_int32, [_P, C.c_int32]),
    "rollout_plan_pages": (C.c_int64, [C.c_int32, C.c_int32, C.c_int32, _P, C.POINTER(C.c_int32),
                                       C.POINTER(C.c_int32), _P]),
}

_lib = None


def load_library() -> C.CDLL:
    """Loads librollout.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -c 'import __graft_entry__ as g; g.build()'`")
        try:   # torch brings its own HIP runtime: when this library starts HIP first, torch finds no GPU later
            import torch
            torch.cuda.is_available()
        except ImportError:
            pass
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _ptr(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def model_desc_from_shape(shape) -> rollout_model_desc:
    return rollout_model_desc(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                              shape.ffn_dim, shape.vocab, shape.n_experts, shape.top_k, shape.expert_ffn_dim,
                              shape.rms_eps, shape.rope_theta,
                              DTYPE_BF16 if shape.dtype == "bf16" else DTYPE_F32,
                              (MODEL_QKV_BIAS if getattr(shape, "qkv_bias", False) else 0) |
                              (MODEL_QK_NORM if getattr(shape, "qk_norm", False) else 0) |
                              (MODEL_TIED_LM_HEAD if getattr(shape, "tied_lm_head", False) else 0))


def _to_device(a: np.ndarray, bf16: bool):
    import torch
    if bf16:
        bits = (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


class Rollout:
    """One rollout context.  Methods mirror the C entry points and return numpy arrays."""

    def __init__(self, shape, weights: dict, *, kv_pool_bytes: int, page_tokens: int = 32,
                 max_live_samples: int = 64, max_context: int = 1024, max_batch_tokens: int = 4096,
                 seed: int = 0, flags: int = 0, stream=None, timing_stride: int = 0):
        import torch
        self.lib = load_library()
        self.shape = shape
        bf16 = shape.dtype == "bf16"
        dev = {}                                   # device copies live only until rollout_init returns
        layers = (rollout_layer_weights * shape.n_layers)()

        def up(name):
            w = weights[name]
            t = w if isinstance(w, torch.Tensor) else _to_device(w, bf16)
            dev[name] = t
            return t.data_ptr()

        for i in range(shape.n_layers):
            p = f"layers.{i}."
            lw = layers[i]
            for f in ("norm1", "wq", "wk", "wv", "wo", "norm2"):
                setattr(lw, f, up(p + f))
            if getattr(shape, "qkv_bias", False):
                for f in ("bq", "bk", "bv"):
                    setattr(lw, f, up(p + f))
            if getattr(shape, "qk_norm", False):
                for f in ("q_norm", "k_norm"):
                    setattr(lw, f, up(p + f))
            if shape.n_experts:
                lw.router = up(p + "router")
                for f in ("w_gate", "w_up", "w_down"):
                    setattr(lw, f, up(p + "experts." + f))
            else:
                for f in ("w_gate", "w_up", "w_down"):
                    setattr(lw, f, up(p + f))
        tied = getattr(shape, "tied_lm_head", False)
        w = rollout_weights(up("embed"), up("final_norm"), None if tied else up("lm_head"), layers)
        md = model_desc_from_shape(shape)
        rd = rollout_runtime_desc(kv_pool_bytes, page_tokens, max_live_samples, max_context, max_batch_tokens,
                                  stream, seed, flags, timing_stride)
        torch.cuda.synchronize()
        ctx = C.c_void_p()
        rc = self.lib.rollout_init(C.byref(ctx), C.byref(md), C.byref(w), C.byref(rd))
        if rc != OK:
            raise RolloutError(rc, self.lib.rollout_last_error(None).decode())
        self.ctx = ctx
        self.max_live = max_live_samples
        del dev

    def _check(self, rc: int):
        if rc < 0:
            raise RolloutError(rc, self.lib.rollout_last_error(self.ctx).decode())
        return rc

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.rollout_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def rollout_prefill(self, tokens, offsets, n_samples, max_new_tokens, eos_id=-1, temperature=1.0,
                        top_p=1.0, forced_first=None, uniform_override=None):
        tokens, offsets = _arr(tokens, np.int32), _arr(offsets, np.int32)
        max_new = _arr(max_new_tokens, np.int32)
        n = (len(offsets) - 1) * n_samples
        forced, uni = _arr(forced_first, np.int32), _arr(uniform_override, np.uint32)
        ids, toks = np.empty(n, np.int64), np.empty(n, np.int32)
        lps, fin = np.empty(n, np.float32), np.empty(n, np.uint8)
        self._check(self.lib.rollout_prefill(self.ctx, len(offsets) - 1, _ptr(tokens), _ptr(offsets), n_samples,
                                             _ptr(max_new), eos_id, temperature, top_p, _ptr(forced), _ptr(uni),
                                             _ptr(ids), _ptr(toks), _ptr(lps), _ptr(fin)))
        return ids, toks, lps, fin.astype(bool)

    def rollout_live_samples(self):
        ids = np.empty(self.max_live, np.int64)
        n = self._check(self.lib.rollout_live_samples(self.ctx, self.max_live, _ptr(ids)))
        return ids[:n].copy()

    def rollout_decode_step(self, forced_tokens=None, uniform_override=None):
        cap = self.max_live
        forced, uni = _arr(forced_tokens, np.int32), _arr(uniform_override, np.uint32)
        ids, toks = np.empty(cap, np.int64), np.empty(cap, np.int32)
        lps, fin = np.empty(cap, np.float32), np.empty(cap, np.uint8)
        n = C.c_int32(cap)
        self._check(self.lib.rollout_decode_step(self.ctx, _ptr(forced), _ptr(uni), C.byref(n), _ptr(ids),
                                                 _ptr(toks), _ptr(lps), _ptr(fin)))
        k = n.value
        return ids[:k], toks[:k], lps[:k], fin[:k].astype(bool)

    def rollout_logprobs(self, tokens, cu_seqlens, temperature=1.0):
        tokens, cu = _arr(tokens, np.int32), _arr(cu_seqlens, np.int32)
        out = np.empty(len(tokens), np.float32)
        self._check(self.lib.rollout_logprobs(self.ctx, len(cu) - 1, _ptr(tokens), _ptr(cu), temperature, _ptr(out)))
        return out

    def rollout_extend(self, sample_ids, tokens, offsets, forced_next=None, uniform_override=None):
        ids, tokens, offsets = _arr(sample_ids, np.int64), _arr(tokens, np.int32), _arr(offsets, np.int32)
        forced, uni = _arr(forced_next, np.int32), _arr(uniform_override, np.uint32)
        n = len(ids)
        toks, lps, fin = np.empty(n, np.int32), np.empty(n, np.float32), np.empty(n, np.uint8)
        self._check(self.lib.rollout_extend(self.ctx, n, _ptr(ids), _ptr(tokens), _ptr(offsets), _ptr(forced),
                                            _ptr(uni), _ptr(toks), _ptr(lps), _ptr(fin)))
        return toks, lps, fin.astype(bool)

    def rollout_update_weights(self, tensors: dict):
        """One bucket: {checkpoint name ("layers.3.wq", "lm_head", "layers.0.experts.w_up", ...): array or
        device tensor}.  Host arrays are uploaded first; the call returns when the library holds
        its own copy."""
        import torch
        bf16 = self.shape.dtype == "bf16"
        arr = (rollout_tensor_update * len(tensors))()
        keep = []
        for k, (name, w) in enumerate(tensors.items()):
            t = w if isinstance(w, torch.Tensor) else _to_device(w, bf16)
            keep.append(t)
            parts = name.split(".")
            layer = int(parts[1]) if parts[0] == "layers" else -1
            arr[k] = rollout_tensor_update(layer, W_IDS[parts[-1]], t.data_ptr())
        torch.cuda.synchronize()
        self._check(self.lib.rollout_update_weights(self.ctx, len(tensors), arr))
        del keep

    def rollout_abort(self, sample_ids):
        ids = _arr(sample_ids, np.int64)
        return self._check(self.lib.rollout_abort(self.ctx, len(ids), _ptr(ids)))

    def rollout_queue_push(self, tokens, offsets, n_samples, max_new_tokens, eos_id=-1, temperature=1.0,
                           top_p=1.0):
        tokens, offsets = _arr(tokens, np.int32), _arr(offsets, np.int32)
        max_new = _arr(max_new_tokens, np.int32)
        pids = np.empty(len(offsets) - 1, np.int64)
        self._check(self.lib.rollout_queue_push(self.ctx, len(offsets) - 1, _ptr(tokens), _ptr(offsets), n_samples,
                                                _ptr(max_new), eos_id, temperature, top_p, _ptr(pids)))
        return pids

    def rollout_queue_policy(self, admit_min_prompts=1, target_prompts=0):
        self._check(self.lib.rollout_queue_policy(self.ctx, admit_min_prompts, target_prompts))

    def rollout_queue_chunking(self, chunk_rows):
        self._check(self.lib.rollout_queue_chunking(self.ctx, chunk_rows))

    def rollout_queue_busy(self) -> bool:
        """True while the queue still has work: prompts waiting or partly cached, or live samples."""
        qs = self.rollout_queue_get_stats()
        return not qs["closed"] and (qs["prompts_waiting"] > 0 or qs["prompts_pending"] > 0 or
                                     self.rollout_get_stats()["live_samples"] > 0)

    def rollout_queue_step(self):
        """Returns (sample_ids, tokens, logprobs, finished, n_admitted)."""
        cap = 3 * self.max_live
        ids, toks = np.empty(cap, np.int64), np.empty(cap, np.int32)
        lps, fin = np.empty(cap, np.float32), np.empty(cap, np.uint8)
        n, adm = C.c_int32(cap), C.c_int32(0)
        self._check(self.lib.rollout_queue_step(self.ctx, C.byref(n), C.byref(adm), _ptr(ids), _ptr(toks),
                                                _ptr(lps), _ptr(fin)))
        k = n.value
        return ids[:k], toks[:k], lps[:k], fin[:k].astype(bool), adm.value

    def rollout_queue_get_stats(self) -> dict:
        st = rollout_queue_stats()
        self._check(self.lib.rollout_queue_get_stats(self.ctx, C.byref(st)))
        return {n: getattr(st, n) for n, _ in rollout_queue_stats._fields_}

    def rollout_debug_logits(self, max_rows=None):
        rows = C.c_int32(max_rows or max(self.max_live, 1024))
        out = np.empty((rows.value, self.shape.vocab), np.float32)
        self._check(self.lib.rollout_debug_logits(self.ctx, C.byref(rows), _ptr(out)))
        return out[:rows.value]

    def rollout_debug_routing(self, max_rows):
        rows = C.c_int32(max_rows)
        out = np.empty(self.shape.n_layers * max_rows * self.shape.top_k, np.int32)
        self._check(self.lib.rollout_debug_routing(self.ctx, C.byref(rows), _ptr(out)))
        n = rows.value
        return out[:self.shape.n_layers * n * self.shape.top_k].reshape(self.shape.n_layers, n, self.shape.top_k)

    def rollout_get_stats(self) -> dict:
        st = rollout_stats()
        self._check(self.lib.rollout_get_stats(self.ctx, C.byref(st)))
        return {n: getattr(st, n) for n, _ in rollout_stats._fields_}


def _kernel_stats(self) -> list:
    n = C.c_int32(32)
    arr = (rollout_kernel_stat * 32)()
    self._check(self.lib.rollout_kernel_stats(self.ctx, C.byref(n), arr))
    return [dict(name=arr[i].name.decode(), launches=arr[i].launches, ms=arr[i].ms, bytes=arr[i].bytes,
                 flops=arr[i].flops) for i in range(n.value)]


Rollout.rollout_kernel_stats = _kernel_stats


def rollout_sample(logits, temperature, top_p, uniforms, forced=None, stream=None):
    """logits: torch float32 CUDA tensor [rows][vocab].  Returns (tokens, logprobs, weight_sums)."""
    lib = load_library()
    assert logits.is_cuda and logits.is_contiguous() and logits.dtype.is_floating_point and logits.element_size() == 4
    rows, vocab = logits.shape
    uni, forced = _arr(uniforms, np.uint32), _arr(forced, np.int32)
    toks, lps, sums = np.empty(rows, np.int32), np.empty(rows, np.float32), np.empty(rows, np.uint64)
    rc = lib.rollout_sample(logits.data_ptr(), rows, vocab, temperature, top_p, _ptr(uni), _ptr(forced), stream,
                            _ptr(toks), _ptr(lps), _ptr(sums))
    if rc != OK:
        raise RolloutError(rc, lib.rollout_last_error(None).decode())
    return toks, lps, sums


SAMPLE_STATIC_MAX_ROWS = 256


def rollout_sample_static(logits, temperature, top_p, uniforms, tokens, logprobs, forced=None, weight_sums=None,
                          stream=None):
    """Every array is a CUDA tensor the caller owns (logits float32 [rows][vocab]; uniforms int32 or
    uint32 bits [rows]; forced int32 [rows] or None; tokens int32, logprobs float32, weight_sums int64
    out).  Only enqueues kernels on `stream`: synchronise before reading the outputs."""
    lib = load_library()
    rows, vocab = logits.shape
    for t in (logits, uniforms, tokens, logprobs) + tuple(x for x in (forced, weight_sums) if x is not None):
        assert t.is_cuda and t.is_contiguous()
    rc = lib.rollout_sample_static(logits.data_ptr(), rows, vocab, temperature, top_p, uniforms.data_ptr(),
                                   forced.data_ptr() if forced is not None else None, stream, tokens.data_ptr(),
                                   logprobs.data_ptr(), weight_sums.data_ptr() if weight_sums is not None else None)
    if rc != OK:
        raise RolloutError(rc, lib.rollout_sample_static_error().decode())


def rollout_policy_loss(cu_seqlens, logp_new, logp_old, logp_ref, mask, rewards, *, gamma=1.0, kl_coef=0.0,
                        reward_clip=20.0, adv_clip=10.0, eps_low=0.2, eps_high=0.2, stream=None):
    """Per-token arrays are torch CUDA tensors (float32; mask uint8), logp_ref may be None.
    Returns (loss, grad, advantages) with grad and advantages as new CUDA tensors."""
    import torch
    lib = load_library()
    cu, rw = _arr(cu_seqlens, np.int32), _arr(rewards, np.float32)
    for t in (logp_new, logp_old, mask) + ((logp_ref,) if logp_ref is not None else ()):
        assert t.is_cuda and t.is_contiguous() and len(t) == int(cu[-1])
    assert logp_new.dtype == torch.float32 and logp_old.dtype == torch.float32 and mask.dtype == torch.uint8
    grad, adv = torch.empty_like(logp_new), torch.empty_like(logp_new)
    params = rollout_loss_params(gamma, kl_coef, reward_clip, adv_clip, eps_low, eps_high)
    loss = C.c_float(0)
    torch.cuda.synchronize()
    rc = lib.rollout_policy_loss(len(cu) - 1, _ptr(cu), logp_new.data_ptr(), logp_old.data_ptr(),
                                 logp_ref.data_ptr() if logp_ref is not None else None, mask.data_ptr(), _ptr(rw),
                                 C.byref(params), stream, C.byref(loss), grad.data_ptr(), adv.data_ptr())
    if rc != OK:
        raise RolloutError(rc, lib.rollout_last_error(None).decode())
    return loss.value, grad, adv


def rollout_philox_words(seed, sample_ids, steps):
    lib = load_library()
    ids, st = _arr(sample_ids, np.int64), _arr(steps, np.uint32)
    out = np.empty(len(ids), np.uint32)
    rc = lib.rollout_philox_words(seed, len(ids), _ptr(ids), _ptr(st), _ptr(out))
    if rc != OK:
        raise RolloutError(rc, lib.rollout_last_error(None).decode())
    return out


def rollout_plan_pages(prompt_len, page_tokens, max_new_tokens):
    lib = load_library()
    mn = _arr(max_new_tokens, np.int32)
    shared, tail = C.c_int32(), C.c_int32()
    priv = np.zeros(len(mn), np.int32)
    total = lib.rollout_plan_pages(prompt_len, page_tokens, len(mn), _ptr(mn), C.byref(shared), C.byref(tail), _ptr(priv))
    if total < 0:
        raise RolloutError(int(total), "bad argument")
    return int(total), shared.value, tail.value, priv


class PagePool:
    """The library's host-side page allocator (rollout_pool_*), usable without a GPU."""

    def __init__(self, n_pages: int):
        self.lib = load_library()
        self.p = self.lib.rollout_pool_create(n_pages)
        if not self.p:
            raise RolloutError(E_INVAL, "rollout_pool_create failed")

    def __del__(self):
        if getattr(self, "p", None):
            self.lib.rollout_pool_destroy(self.p)
            self.p = None

    def free_pages(self): return self.lib.rollout_pool_free_pages(self.p)
    def unreserved(self): return self.lib.rollout_pool_unreserved(self.p)
    def reserve(self, n): return self.lib.rollout_pool_reserve(self.p, n)
    def unreserve(self, n): self.lib.rollout_pool_unreserve(self.p, n)
    def alloc(self, from_reservation=False): return self.lib.rollout_pool_alloc(self.p, int(from_reservation))
    def retain(self, page): return self.lib.rollout_pool_retain(self.p, page)
    def release(self, page): return self.lib.rollout_pool_release(self.p, page)
    def refcount(self, page): return self.lib.rollout_pool_refcount(self.p, page)
