"""ctypes binding of libapril.so: same names as include/april.h, argument marshalling only.

Every step of the rollout path runs in the library's HIP kernels; nothing here
computes.  Loading fails loudly when the library is missing: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libapril.so")

APRIL_OK, APRIL_EINVAL, APRIL_ENOMEM, APRIL_ESTARVED, APRIL_EHANDLE, APRIL_EDEVICE = 0, -1, -2, -3, -4, -5
APRIL_DTYPE_FP32, APRIL_DTYPE_BF16 = 0, 1
APRIL_SAMPLER_GREEDY, APRIL_SAMPLER_TOPK, APRIL_SAMPLER_CATEGORICAL = 0, 1, 2
APRIL_MEM_KV, APRIL_MEM_WEIGHTS = 1, 2
APRIL_KERNEL_CLASSES = 24

EXPORTS = [
    "april_init", "april_rollout_step", "april_resume", "april_buffer_size", "april_buffer_export",
    "april_buffer_import", "april_buffer_drop_kv", "april_buffer_free", "april_update_weights", "april_memory_pause", "april_memory_resume", "april_debug_watch",
    "april_debug_logits", "april_sample_rows", "april_sample_rows_logprobs", "april_sample_rows_noalloc", "april_profile_enable", "april_profile_get",
    "april_profile_reset", "april_get_info", "april_last_error", "april_destroy",
]


class AprilError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"april error {code}: {msg}")
        self.code = code


class april_model_cfg(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
        ("n_experts", C.c_int32), ("experts_per_tok", C.c_int32), ("d_expert_ffn", C.c_int32),
        ("dtype", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float),
        ("kv_block_tokens", C.c_int32), ("kv_pool_bytes", C.c_int64),
        ("max_inflight", C.c_int32), ("max_ctx", C.c_int32),
        ("sampler", C.c_int32), ("top_k", C.c_int32), ("temperature", C.c_float), ("seed", C.c_uint64),
        ("eos_token", C.c_int32), ("debug_logits", C.c_int32), ("top_p", C.c_float), ("logprobs", C.c_int32),
        ("n_samples_per_prompt", C.c_int32), ("pausable", C.c_int32), ("stream", C.c_void_p),
    ]


class april_tensor(C.Structure):
    _fields_ = [("name", C.c_char_p), ("data", C.c_void_p), ("nbytes", C.c_int64), ("on_device", C.c_int32)]


class april_request(C.Structure):
    _fields_ = [("request_id", C.c_int64), ("tokens", C.POINTER(C.c_int32)), ("n_tokens", C.c_int32),
                ("forced_len", C.c_int32), ("forced_tokens", C.POINTER(C.c_int32)), ("n_forced_tokens", C.c_int32),
                ("group_id", C.c_int64)]


class april_step_result(C.Structure):
    _fields_ = [
        ("n_completed", C.c_int32), ("request_id", C.POINTER(C.c_int64)),
        ("tokens", C.POINTER(C.POINTER(C.c_int32))), ("n_tokens", C.POINTER(C.c_int32)),
        ("n_resumes", C.POINTER(C.c_int32)), ("logprobs", C.POINTER(C.POINTER(C.c_float))),
        ("group_id", C.POINTER(C.c_int64)), ("buffer", C.c_void_p), ("n_new_consumed", C.c_int32),
        ("decode_iters", C.c_int64), ("tokens_generated", C.c_int64), ("prefill_tokens", C.c_int64),
        ("reprefill_tokens", C.c_int64), ("n_preempted", C.c_int64), ("sum_live", C.c_int64), ("sum_ctx", C.c_int64),
        ("dec_sum_live", C.c_int64), ("dec_sum_ctx", C.c_int64), ("dec_sum_experts", C.c_int64),
        ("t_prefill_s", C.c_double), ("t_decode_s", C.c_double), ("t_total_s", C.c_double),
    ]


class april_partial(C.Structure):
    _fields_ = [("request_id", C.c_int64), ("prompt", C.POINTER(C.c_int32)), ("n_prompt", C.c_int32),
                ("generated", C.POINTER(C.c_int32)), ("n_generated", C.c_int32), ("limit", C.c_int32),
                ("n_resumes", C.c_int32), ("done", C.c_int32), ("kv_resident", C.c_int32),
                ("logprobs", C.POINTER(C.c_float)), ("group_id", C.c_int64)]


class april_kernel_stat(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("alg_bytes", C.c_double), ("alg_flops", C.c_double)]


class april_info(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("hbm_total", "hbm_free", "kv_pool_bytes", "kv_blocks_total",
                                         "kv_blocks_free", "weight_bytes", "decode_weight_bytes",
                                         "kv_bytes_per_token", "expert_bytes")]


_lib = None


def load_library():
    """dlopen libapril.so (built in-tree by build.py) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2509_18521_amd.build` "
                                "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    lib.april_init.argtypes = [C.POINTER(april_model_cfg), C.POINTER(april_tensor), C.c_int32, C.POINTER(vp)]
    lib.april_rollout_step.argtypes = [vp, C.POINTER(april_request), C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                       C.POINTER(april_step_result)]
    lib.april_resume.argtypes = [vp, vp]
    lib.april_buffer_size.argtypes = [vp, vp]
    lib.april_buffer_export.argtypes = [vp, vp, C.POINTER(april_partial), C.c_int32]
    lib.april_buffer_import.argtypes = [vp, C.POINTER(april_partial), C.c_int32, C.POINTER(vp)]
    lib.april_buffer_drop_kv.argtypes = [vp, vp]
    lib.april_buffer_free.argtypes = [vp, vp]
    lib.april_buffer_free.restype = None
    lib.april_update_weights.argtypes = [vp, C.POINTER(april_tensor), C.c_int32, C.c_int32]
    lib.april_memory_pause.argtypes = [vp, C.c_int32]
    lib.april_memory_resume.argtypes = [vp, C.c_int32]
    lib.april_debug_watch.argtypes = [vp, C.c_int64, C.c_int32, C.c_int32]
    lib.april_debug_logits.argtypes = [vp, C.c_int64, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    lib.april_sample_rows.argtypes = [vp, vp, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int32),
                                      C.POINTER(C.c_int32)]
    lib.april_sample_rows_noalloc.argtypes = lib.april_sample_rows.argtypes
    lib.april_sample_rows_logprobs.argtypes = lib.april_sample_rows.argtypes + [C.POINTER(C.c_float)]
    lib.april_profile_enable.argtypes = [vp, C.c_int32]
    lib.april_profile_get.argtypes = [vp, C.POINTER(april_kernel_stat), C.c_int32]
    lib.april_profile_reset.argtypes = [vp]
    lib.april_get_info.argtypes = [vp, C.POINTER(april_info)]
    lib.april_last_error.argtypes = [vp]
    lib.april_last_error.restype = C.c_char_p
    lib.april_destroy.argtypes = [vp]
    lib.april_destroy.restype = None
    for name in EXPORTS:
        if name not in ("april_buffer_free", "april_destroy", "april_last_error"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(ctx, rc):
    if rc < 0:
        msg = load_library().april_last_error(ctx)
        raise AprilError(rc, msg.decode() if msg else "")
    return rc


def _i32ptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


# ---------------------------------------------------------------------------
# same-name wrappers
# ---------------------------------------------------------------------------
def _tensor_table(weights: Dict[str, object]):
    """name -> numpy array (host) or an object with .data_ptr() / .numel() / .element_size() on
    the GPU (e.g. a torch CUDA tensor)  ->  (april_tensor array, objects to keep alive)."""
    arr = (april_tensor * len(weights))()
    keep = []
    for i, (name, w) in enumerate(weights.items()):
        name = name.encode()
        keep.append(name)
        if isinstance(w, np.ndarray):
            w = np.ascontiguousarray(w)
            keep.append(w)
            arr[i] = april_tensor(name, w.ctypes.data, w.nbytes, 0)
        else:
            keep.append(w)
            arr[i] = april_tensor(name, w.data_ptr(), w.numel() * w.element_size(), 1)
    return arr, keep


def april_init(cfg: april_model_cfg, weights: Dict[str, object]) -> C.c_void_p:
    """weights: see _tensor_table.  Arrays are borrowed for the duration of the call."""
    lib = load_library()
    arr, keep = _tensor_table(weights)
    out = C.c_void_p()
    _check(None, lib.april_init(C.byref(cfg), arr, len(weights), C.byref(out)))
    return out


def april_update_weights(ctx, weights: Dict[str, object], keep_kv: bool = False):
    arr, keep = _tensor_table(weights)
    _check(ctx, load_library().april_update_weights(ctx, arr, len(weights), 1 if keep_kv else 0))


def april_destroy(ctx):
    load_library().april_destroy(ctx)


@dataclass
class StepResult:
    request_id: List[int]
    tokens: List[np.ndarray]
    n_resumes: List[int]
    buffer: C.c_void_p
    n_new_consumed: int
    decode_iters: int
    tokens_generated: int
    prefill_tokens: int
    reprefill_tokens: int
    n_preempted: int
    sum_live: int
    sum_ctx: int
    dec_sum_live: int
    dec_sum_ctx: int
    dec_sum_experts: int
    t_prefill_s: float
    t_decode_s: float
    t_total_s: float
    logprobs: Optional[List[np.ndarray]] = None      # per completed rollout (contexts created with logprobs)
    group_id: Optional[List[int]] = None             # per completed rollout (n_samples_per_prompt > 1)


def april_rollout_step(ctx, requests: Sequence[dict], n_target: int, n_overprovision: int, max_new: int) -> StepResult:
    """requests: dicts with request_id, tokens (int32 array), forced_len, optional forced_tokens."""
    lib = load_library()
    n = len(requests)
    arr = (april_request * max(n, 1))()
    keep = []
    for i, r in enumerate(requests):
        t = np.ascontiguousarray(r["tokens"], dtype=np.int32)
        keep.append(t)
        ft = r.get("forced_tokens")
        if ft is not None:
            ft = np.ascontiguousarray(ft, dtype=np.int32)
            keep.append(ft)
        arr[i] = april_request(int(r["request_id"]), _i32ptr(t), t.shape[0], int(r.get("forced_len", 0)),
                               _i32ptr(ft) if ft is not None else None, 0 if ft is None else ft.shape[0],
                               int(r.get("group_id", -1)))
    res = april_step_result()
    _check(ctx, lib.april_rollout_step(ctx, arr, n, n_target, n_overprovision, max_new, C.byref(res)))
    ids, toks, nres = [], [], []
    lps = [] if res.logprobs else None
    for i in range(res.n_completed):
        ids.append(int(res.request_id[i]))
        nt = int(res.n_tokens[i])
        toks.append(np.ctypeslib.as_array(res.tokens[i], shape=(nt,)).copy() if nt > 0 else np.zeros(0, np.int32))
        nres.append(int(res.n_resumes[i]))
        if lps is not None:
            lps.append(np.ctypeslib.as_array(res.logprobs[i], shape=(nt,)).copy() if nt > 0 else np.zeros(0, np.float32))
    return StepResult(ids, toks, nres, C.c_void_p(res.buffer), res.n_new_consumed, res.decode_iters,
                      res.tokens_generated, res.prefill_tokens, res.reprefill_tokens, res.n_preempted, res.sum_live, res.sum_ctx, res.dec_sum_live, res.dec_sum_ctx, res.dec_sum_experts,
                      res.t_prefill_s, res.t_decode_s, res.t_total_s, lps,
                      [int(res.group_id[i]) for i in range(res.n_completed)] if res.group_id else None)


def april_resume(ctx, buffer):
    _check(ctx, load_library().april_resume(ctx, buffer))


def april_buffer_size(ctx, buffer) -> int:
    return _check(ctx, load_library().april_buffer_size(ctx, buffer))


def april_buffer_export(ctx, buffer) -> List[dict]:
    lib = load_library()
    n = april_buffer_size(ctx, buffer)
    arr = (april_partial * max(n, 1))()
    _check(ctx, lib.april_buffer_export(ctx, buffer, arr, n))
    out = []
    for i in range(n):
        p = arr[i]
        out.append(dict(
            request_id=int(p.request_id),
            prompt=np.ctypeslib.as_array(p.prompt, shape=(p.n_prompt,)).copy(),
            generated=(np.ctypeslib.as_array(p.generated, shape=(p.n_generated,)).copy()
                       if p.n_generated > 0 else np.zeros(0, np.int32)),
            limit=int(p.limit), n_resumes=int(p.n_resumes), done=int(p.done), kv_resident=int(p.kv_resident),
            logprobs=(np.ctypeslib.as_array(p.logprobs, shape=(p.n_generated,)).copy()
                      if p.logprobs and p.n_generated > 0 else None), group_id=int(p.group_id)))
    return out


def april_buffer_import(ctx, partials: Sequence[dict]):
    lib = load_library()
    n = len(partials)
    arr = (april_partial * max(n, 1))()
    keep = []
    for i, p in enumerate(partials):
        pr = np.ascontiguousarray(p["prompt"], dtype=np.int32)
        ge = np.ascontiguousarray(p["generated"], dtype=np.int32)
        lp = p.get("logprobs")
        if lp is not None:
            lp = np.ascontiguousarray(lp, dtype=np.float32)
        keep += [pr, ge, lp]
        arr[i] = april_partial(int(p["request_id"]), _i32ptr(pr), pr.shape[0],
                               _i32ptr(ge) if ge.shape[0] else None, ge.shape[0], int(p["limit"]),
                               int(p.get("n_resumes", 0)), int(p.get("done", 0)), 0,
                               lp.ctypes.data_as(C.POINTER(C.c_float)) if lp is not None and lp.shape[0] else None,
                               int(p.get("group_id", -1)))
    out = C.c_void_p()
    _check(ctx, lib.april_buffer_import(ctx, arr, n, C.byref(out)))
    return out


def april_memory_pause(ctx, tags: int):
    _check(ctx, load_library().april_memory_pause(ctx, tags))


def april_memory_resume(ctx, tags: int):
    _check(ctx, load_library().april_memory_resume(ctx, tags))


def april_buffer_drop_kv(ctx, buffer):
    _check(ctx, load_library().april_buffer_drop_kv(ctx, buffer))


def april_buffer_free(ctx, buffer):
    load_library().april_buffer_free(ctx, buffer)


def april_debug_watch(ctx, request_id: int, first_gen: int, n_gen: int):
    _check(ctx, load_library().april_debug_watch(ctx, request_id, first_gen, n_gen))


def april_debug_logits(ctx, request_id: int, gen_index: int, vocab: int):
    out = np.empty(vocab, dtype=np.float32)
    sampled = C.c_int32(-1)
    _check(ctx, load_library().april_debug_logits(ctx, request_id, gen_index,
                                                  out.ctypes.data_as(C.POINTER(C.c_float)), C.byref(sampled)))
    return out, int(sampled.value)


def april_sample_rows(ctx, logits_device_ptr: int, n_rows: int, request_ids, gen_index) -> np.ndarray:
    rid = np.ascontiguousarray(request_ids, dtype=np.int64)
    gi = np.ascontiguousarray(gen_index, dtype=np.int32)
    out = np.empty(n_rows, dtype=np.int32)
    _check(ctx, load_library().april_sample_rows(ctx, C.c_void_p(logits_device_ptr), n_rows,
                                                 rid.ctypes.data_as(C.POINTER(C.c_int64)), _i32ptr(gi), _i32ptr(out)))
    return out


def april_sample_rows_logprobs(ctx, logits_device_ptr: int, n_rows: int, request_ids, gen_index):
    rid = np.ascontiguousarray(request_ids, dtype=np.int64)
    gi = np.ascontiguousarray(gen_index, dtype=np.int32)
    out = np.empty(n_rows, dtype=np.int32)
    lp = np.empty(n_rows, dtype=np.float32)
    _check(ctx, load_library().april_sample_rows_logprobs(ctx, C.c_void_p(logits_device_ptr), n_rows,
                                                          rid.ctypes.data_as(C.POINTER(C.c_int64)), _i32ptr(gi),
                                                          _i32ptr(out), lp.ctypes.data_as(C.POINTER(C.c_float))))
    return out, lp


def april_sample_rows_noalloc(ctx, logits_device_ptr: int, n_rows: int, request_ids, gen_index) -> np.ndarray:
    rid = np.ascontiguousarray(request_ids, dtype=np.int64)
    gi = np.ascontiguousarray(gen_index, dtype=np.int32)
    out = np.empty(n_rows, dtype=np.int32)
    _check(ctx, load_library().april_sample_rows_noalloc(ctx, C.c_void_p(logits_device_ptr), n_rows,
                                                         rid.ctypes.data_as(C.POINTER(C.c_int64)), _i32ptr(gi),
                                                         _i32ptr(out)))
    return out


def april_profile_enable(ctx, every: int):
    _check(ctx, load_library().april_profile_enable(ctx, every))


def april_profile_reset(ctx):
    _check(ctx, load_library().april_profile_reset(ctx))


def april_profile_get(ctx) -> List[dict]:
    arr = (april_kernel_stat * APRIL_KERNEL_CLASSES)()
    n = _check(ctx, load_library().april_profile_get(ctx, arr, APRIL_KERNEL_CLASSES))
    return [dict(name=arr[i].name.decode(), launches=int(arr[i].launches), total_ms=float(arr[i].total_ms),
                 alg_bytes=float(arr[i].alg_bytes), alg_flops=float(arr[i].alg_flops)) for i in range(n)]


def april_get_info(ctx) -> dict:
    info = april_info()
    _check(ctx, load_library().april_get_info(ctx, C.byref(info)))
    return {n: int(getattr(info, n)) for n, _ in april_info._fields_}


# ---------------------------------------------------------------------------
# helpers to build the configuration and weight table from the synthetic inputs
# ---------------------------------------------------------------------------
def make_cfg(shape, *, max_inflight, max_ctx, sampler=APRIL_SAMPLER_GREEDY, top_k=1, temperature=1.0, seed=0,
             eos_token=-1, debug_logits=False, kv_pool_bytes=0, stream=None, top_p=0.0,
             logprobs=False, n_samples_per_prompt=0, pausable=False) -> april_model_cfg:
    return april_model_cfg(
        shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
        shape.vocab, shape.n_experts, shape.experts_per_tok, shape.d_expert_ffn, shape.dtype,
        shape.rope_theta, shape.rms_eps, 16, kv_pool_bytes, max_inflight, max_ctx, sampler, top_k,
        temperature, seed, eos_token, 1 if debug_logits else 0, top_p, 1 if logprobs else 0,
        n_samples_per_prompt, 1 if pausable else 0, stream)


def pack_weights(shape, weights_fp32: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    """fp32-valued arrays -> the element type the library expects: matrices and the
    embedding as bf16 bit patterns for a bf16 model (the values are already exactly
    representable), gains always float32."""
    out = {}
    for name, a in weights_fp32.items():
        is_gain = name.startswith(("attn_norm", "mlp_norm", "final_norm"))
        if shape.dtype == APRIL_DTYPE_BF16 and not is_gain:
            bits = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
            if np.any(bits & np.uint32(0xFFFF)):
                raise ValueError(f"{name}: values are not exactly representable in bf16")
            out[name] = (bits >> np.uint32(16)).astype(np.uint16)
        else:
            out[name] = np.ascontiguousarray(a, dtype=np.float32)
    return out
