"""ctypes binding of the C ABI in include/odb.h: argument marshalling only.

Every function has the name of the C entry point it calls.  Device buffers are
torch CUDA tensors (PyTorch-ROCm is the device allocator and stream provider);
all arithmetic happens inside libodb.so.  There is no fallback: if the library
has not been built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libodb.so")

#: every symbol include/odb.h declares
SYMBOLS = (
    "odb_model_create", "odb_model_destroy", "odb_model_init_random", "odb_model_set_tensor",
    "odb_model_get_tensor", "odb_cache_create", "odb_cache_destroy", "odb_cache_length", "odb_prefill",
    "odb_block_step", "odb_prefill_logits", "odb_block_step_logits", "odb_cache_read", "odb_strerror",
    "odb_last_error", "odb_profile_begin", "odb_profile_end", "odb_set_option", "odb_model_status",
    "odb_predict_length", "odb_accept_jump", "odb_block_step_shared", "odb_block_step_static",
    "odb_block_step_shared_rows", "odb_block_step_shared_logits", "odb_cache_truncate", "odb_generate",
    "odb_speculative_jump",
)

KERNEL_CLASSES = ("gemm_qkv", "attention", "gemm_o", "gemm_gate_up", "gemm_down", "gemm_lm_head", "rmsnorm")
OPT_KSPLIT_REDUCE = 0
STATIC_SCRATCH_BYTES = 32 << 20

T_EMBED, T_WQ, T_WK, T_WV, T_WO, T_WG, T_WU, T_WD, T_LM, T_G1, T_G2, T_GF = range(12)


class OdbError(RuntimeError):
    pass


class odb_config(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int), ("d_model", ctypes.c_int), ("n_heads", ctypes.c_int),
                ("head_dim", ctypes.c_int), ("d_ff", ctypes.c_int), ("vocab", ctypes.c_int),
                ("rope_base", ctypes.c_float), ("rms_eps", ctypes.c_float), ("mask_id", ctypes.c_int)]


_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class odb_allocator(ctypes.Structure):
    _fields_ = [("alloc", _ALLOC_FN), ("free", _FREE_FN), ("user", ctypes.c_void_p)]


class odb_generate_params(ctypes.Structure):
    _fields_ = [("block_len", ctypes.c_int), ("n_drafts", ctypes.c_int), ("tau", ctypes.c_float),
                ("eos_id", ctypes.c_int), ("truncate_thr", ctypes.c_float), ("share_from", ctypes.c_int),
                ("row_budget", ctypes.c_int)]


class odb_generate_event(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("length", ctypes.c_int), ("block_off", ctypes.c_int),
                ("block_len", ctypes.c_int), ("chosen", ctypes.c_int), ("n_masked", ctypes.c_int),
                ("cand_pos", ctypes.c_int * 4), ("cand_tok", ctypes.c_int * 4)]


class odb_generate_stats(ctypes.Structure):
    _fields_ = [("n_refresh", ctypes.c_int), ("n_step", ctypes.c_int), ("n_step_shared", ctypes.c_int),
                ("final_len", ctypes.c_int), ("n_events", ctypes.c_int), ("refresh_positions", ctypes.c_longlong),
                ("step_rows", ctypes.c_longlong), ("refresh_ms", ctypes.c_double), ("step_ms", ctypes.c_double),
                ("total_ms", ctypes.c_double)]


EVENT_KINDS = ("refresh", "step", "shared")

_lib = None


def lib() -> ctypes.CDLL:
    """Loads libodb.so (built by `__graft_entry__.build()` / build.py) once."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise OdbError("%s is missing: build it with `python -m paper_2511_21759_amd.build` "
                       "(there is no fallback path)" % LIB_PATH)
    # PyTorch-ROCm ships its own HIP runtime; import it first so that the library
    # binds to the runtime torch uses (one runtime per process, shared streams).
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    L.odb_model_create.argtypes = [ctypes.POINTER(odb_config), ctypes.POINTER(odb_allocator), ctypes.POINTER(vp)]
    L.odb_model_destroy.argtypes = [vp]
    L.odb_model_destroy.restype = None
    L.odb_model_init_random.argtypes = [vp, ctypes.c_uint64, ctypes.c_double, vp]
    L.odb_model_set_tensor.argtypes = [vp, ci, ci, vp, ctypes.c_size_t]
    L.odb_model_get_tensor.argtypes = [vp, ci, ci, vp, ctypes.c_size_t]
    L.odb_cache_create.argtypes = [vp, ci, ci, ctypes.POINTER(vp)]
    L.odb_cache_destroy.argtypes = [vp]
    L.odb_cache_destroy.restype = None
    L.odb_cache_length.argtypes = [vp]
    L.odb_prefill.argtypes = [vp, vp, vp, ci, ci, vp, vp, vp]
    L.odb_block_step.argtypes = [vp, vp, vp, ci, ci, ci, cf, vp, vp, vp, vp]
    L.odb_prefill_logits.argtypes = [vp, vp, vp, ci, ci, vp, vp]
    L.odb_block_step_logits.argtypes = [vp, vp, vp, ci, ci, ci, vp, vp]
    L.odb_cache_read.argtypes = [vp, ci, ci, ci, ci, ci, vp]
    L.odb_profile_begin.argtypes = [vp, ci, ci]
    L.odb_profile_end.argtypes = [vp, ctypes.POINTER(ci), ctypes.POINTER(cf), ctypes.POINTER(cf)]
    L.odb_predict_length.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, cf, vp, vp]
    L.odb_cache_truncate.argtypes = [vp, ci]
    L.odb_generate.argtypes = [vp, vp, vp, ci, ci, vp, vp, vp, vp, ci, vp]
    L.odb_accept_jump.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, vp, vp, vp, vp, vp]
    L.odb_speculative_jump.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, vp, vp, vp, vp, vp]
    L.odb_block_step_shared.argtypes = [vp, vp, vp, ci, ci, ci, ci, cf, vp, vp, vp, vp]
    L.odb_block_step_shared_rows.argtypes = [ci, ci, ci, ci]
    L.odb_block_step_shared_logits.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp, vp]
    L.odb_set_option.argtypes = [vp, ci, ci]
    L.odb_model_status.argtypes = [vp]
    L.odb_block_step_static.argtypes = [vp, vp, vp, ci, ci, ci, cf, vp, vp, vp, vp]
    L.odb_strerror.argtypes = [ci]
    L.odb_strerror.restype = ctypes.c_char_p
    L.odb_last_error.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != 0:
        L = lib()
        raise OdbError("%s: %s" % (L.odb_strerror(rc).decode(), L.odb_last_error().decode()))


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dev_i32(t):
    import torch
    if not (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise OdbError("expected a contiguous int32 CUDA tensor")
    return t.data_ptr()


# ---- one function per C entry point ---------------------------------------------------------

class _TorchAllocator:
    """odb_allocator backed by torch.empty(dtype=uint8, device="cuda"): PyTorch stays the one owner of device
    memory (weights, caches, scratch and the working buffers of odb_generate all come from its caching allocator).
    The tensors are kept alive here, by address, until the library frees them."""

    def __init__(self):
        import torch
        self.live = {}

        def alloc(nbytes, _user):
            try:
                t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device="cuda")
            except RuntimeError:           # out of memory: the library reports ODB_E_NOMEM
                return None
            self.live[t.data_ptr()] = t    # (torch's blocks are aligned to 512 bytes)
            return t.data_ptr()

        def free(ptr, _user):
            self.live.pop(ptr, None)

        self._alloc, self._free = _ALLOC_FN(alloc), _FREE_FN(free)      # the callbacks must outlive the model
        self.struct = odb_allocator(self._alloc, self._free, None)


_allocators: Dict[int, _TorchAllocator] = {}


def odb_model_create(shape: Dict, torch_allocator: bool = True) -> int:
    """torch_allocator: hand the library an odb_allocator backed by torch (default); False = allocator NULL, the
    library then calls hipMalloc / hipFree itself."""
    cfg = odb_config(**{k: shape[k] for k, _ in odb_config._fields_})
    out = ctypes.c_void_p()
    al = _TorchAllocator() if torch_allocator else None
    _check(lib().odb_model_create(ctypes.byref(cfg), ctypes.byref(al.struct) if al else None, ctypes.byref(out)))
    if al:
        _allocators[out.value] = al
    return out.value


def odb_model_destroy(model: int) -> None:
    lib().odb_model_destroy(model)
    _allocators.pop(model, None)


def odb_model_init_random(model: int, seed: int, std: float) -> None:
    _check(lib().odb_model_init_random(model, seed, std, _stream()))


def odb_model_set_tensor(model: int, tensor_id: int, layer: int, bits: np.ndarray) -> None:
    bits = np.ascontiguousarray(bits, np.uint16)
    _check(lib().odb_model_set_tensor(model, tensor_id, layer, bits.ctypes.data, bits.size))


def odb_model_get_tensor(model: int, tensor_id: int, layer: int, n: int) -> np.ndarray:
    out = np.empty(n, np.uint16)
    _check(lib().odb_model_get_tensor(model, tensor_id, layer, out.ctypes.data, n))
    return out


def odb_cache_create(model: int, batch: int, max_len: int) -> int:
    out = ctypes.c_void_p()
    _check(lib().odb_cache_create(model, batch, max_len, ctypes.byref(out)))
    return out.value


def odb_cache_destroy(cache: int) -> None:
    lib().odb_cache_destroy(cache)


def odb_cache_length(cache: int) -> int:
    return lib().odb_cache_length(cache)


def odb_prefill(model: int, cache: int, tokens, resp_off: int, conf=None, argmax=None):
    """tokens: int32 CUDA tensor [B, L] -> (conf [B, L-resp_off] f32, argmax int32)."""
    import torch
    B, L = tokens.shape
    if conf is None:
        conf = torch.empty((B, L - resp_off), dtype=torch.float32, device=tokens.device)
    if argmax is None:
        argmax = torch.empty((B, L - resp_off), dtype=torch.int32, device=tokens.device)
    _check(lib().odb_prefill(model, cache, _dev_i32(tokens), L, resp_off, conf.data_ptr(), argmax.data_ptr(),
                             _stream()))
    return conf, argmax


def odb_predict_length(model: int, tokens, conf, argmax, resp_off: int, eos_id: int, truncate_thr: float, out=None):
    """tokens int32 [B, L], conf f32 / argmax int32 [B, L-resp_off] (CUDA tensors) -> new lengths int32 [B]."""
    import torch
    B, L = tokens.shape
    if conf.dtype != torch.float32 or argmax.dtype != torch.int32 or not conf.is_contiguous() or not argmax.is_contiguous():
        raise TypeError("conf must be contiguous float32 and argmax contiguous int32")
    if tuple(conf.shape) != (B, L - resp_off) or tuple(argmax.shape) != (B, L - resp_off):
        raise ValueError("conf / argmax must have shape [B, L - resp_off]")
    if out is None:
        out = torch.empty((B,), dtype=torch.int32, device=tokens.device)
    _check(lib().odb_predict_length(model, _dev_i32(tokens), conf.data_ptr(), argmax.data_ptr(), B, L, resp_off, eos_id,
                                    truncate_thr, out.data_ptr(), _stream()))
    return out


def odb_block_step_shared(model: int, cache: int, drafts, block_off: int, n_masked: int, tau: float,
                          conf=None, argmax=None, unmask=None):
    """drafts: int32 CUDA tensor [B, S, b] -> (conf f32, argmax int32, unmask uint8), each [B, S, b]."""
    import torch
    B, S, b = drafts.shape
    if conf is None:
        conf = torch.empty((B, S, b), dtype=torch.float32, device=drafts.device)
    if argmax is None:
        argmax = torch.empty((B, S, b), dtype=torch.int32, device=drafts.device)
    if unmask is None:
        unmask = torch.empty((B, S, b), dtype=torch.uint8, device=drafts.device)
    _check(lib().odb_block_step_shared(model, cache, _dev_i32(drafts), block_off, b, S, n_masked, tau, conf.data_ptr(),
                                       argmax.data_ptr(), unmask.data_ptr(), _stream()))
    return conf, argmax, unmask


def odb_block_step_shared_logits(model: int, cache: int, drafts, block_off: int, n_masked: int, vocab: int):
    """-> (logits f32 [rows, vocab], rowout int32 [rows]: index into [B, S, b] of every row, -1 for padding)."""
    import torch
    B, S, b = drafts.shape
    rows = lib().odb_block_step_shared_rows(B, b, S, n_masked)
    _check(min(rows, 0))
    logits = torch.empty((rows, vocab), dtype=torch.float32, device=drafts.device)
    rowout = torch.empty((rows,), dtype=torch.int32, device=drafts.device)
    _check(lib().odb_block_step_shared_logits(model, cache, _dev_i32(drafts), block_off, b, S, n_masked,
                                              logits.data_ptr(), rowout.data_ptr(), _stream()))
    return logits, rowout


def odb_cache_truncate(cache: int, new_len: int) -> None:
    _check(lib().odb_cache_truncate(cache, new_len))


def odb_generate(model: int, cache: int, tokens, prompt_len: int, block_len: int, n_drafts: int = 1, tau: float = 0.9,
                 eos_id: int = -1, truncate_thr: float = 0.9, share_from: int = -1, row_budget: int = 0,
                 max_events: int = 0, event_tokens: bool = False):
    """tokens: int32 CUDA tensor [prompt_len + resp_len] whose first prompt_len entries hold the prompt; decoded
    in place.  -> (stats dict, events list of dicts, event_tokens int32 CUDA tensor [n, L0] or None).
    An event's cand_pos / cand_tok hold the candidates in use: four with n_drafts = 8, else two."""
    import torch
    if tokens.dtype != torch.int32 or tokens.dim() != 1 or not tokens.is_contiguous() or not tokens.is_cuda:
        raise TypeError("tokens must be a contiguous 1-D int32 CUDA tensor")
    L0 = tokens.shape[0]
    gp = odb_generate_params(block_len, n_drafts, tau, eos_id, truncate_thr, share_from, row_budget)
    st = odb_generate_stats()
    ev = (odb_generate_event * max_events)() if max_events > 0 else None
    snap = torch.empty((max_events, L0), dtype=torch.int32, device=tokens.device) if event_tokens and max_events > 0 else None
    _check(lib().odb_generate(model, cache, tokens.data_ptr(), prompt_len, L0 - prompt_len, ctypes.byref(gp),
                              ctypes.byref(st), ctypes.cast(ev, ctypes.c_void_p) if ev is not None else None,
                              snap.data_ptr() if snap is not None else None, max_events, _stream()))
    stats = {name: getattr(st, name) for name, _ in odb_generate_stats._fields_}
    n = min(st.n_events, max_events)
    nc = 4 if n_drafts == 8 else 2
    events = [dict(kind=EVENT_KINDS[e.kind], L=e.length, block_off=e.block_off, block_len=e.block_len, chosen=e.chosen,
                   n_masked=e.n_masked, cand_pos=np.array(list(e.cand_pos)[:nc], np.int32),
                   cand_tok=np.array(list(e.cand_tok)[:nc], np.int32)) for e in (ev[i] for i in range(n))]
    return stats, events, (snap[:n] if snap is not None else None)


def odb_accept_jump(model: int, drafts, conf, argmax, unmask, cand_pos, cand_tok):
    """drafts/argmax int32, conf f32, unmask uint8: CUDA tensors [B, 4, b]; cand_pos/cand_tok int32 [B, 2]
    -> (chosen int32 [B], new_drafts int32 [B, 4, b], new_cand_pos int32 [B, 2], new_cand_tok int32 [B, 2])."""
    import torch
    B, S, b = drafts.shape
    if S != 4:
        raise ValueError("the accept-jump stage runs on four drafts")
    want = {"drafts": (drafts, torch.int32, (B, 4, b)), "conf": (conf, torch.float32, (B, 4, b)),
            "argmax": (argmax, torch.int32, (B, 4, b)), "unmask": (unmask, torch.uint8, (B, 4, b)),
            "cand_pos": (cand_pos, torch.int32, (B, 2)), "cand_tok": (cand_tok, torch.int32, (B, 2))}
    for name, (t, dt, shp) in want.items():
        if t.dtype != dt or tuple(t.shape) != shp or not t.is_contiguous() or not t.is_cuda:
            raise TypeError("%s must be a contiguous CUDA tensor of dtype %s and shape %s" % (name, dt, shp))
    chosen = torch.empty((B,), dtype=torch.int32, device=drafts.device)
    new_drafts = torch.empty_like(drafts)
    new_pos, new_tok = torch.empty_like(cand_pos), torch.empty_like(cand_tok)
    _check(lib().odb_accept_jump(model, drafts.data_ptr(), conf.data_ptr(), argmax.data_ptr(), unmask.data_ptr(),
                                 cand_pos.data_ptr(), cand_tok.data_ptr(), B, b, chosen.data_ptr(), new_drafts.data_ptr(),
                                 new_pos.data_ptr(), new_tok.data_ptr(), _stream()))
    return chosen, new_drafts, new_pos, new_tok


def odb_speculative_jump(model: int, drafts, conf, argmax, unmask, cand_pos, cand_tok, n_next: int):
    """drafts/argmax int32, conf f32, unmask uint8: CUDA tensors [B, S, b], S = 4 or 8; cand_pos/cand_tok int32 [B, 4]
    -> (chosen int32 [B], new_drafts int32 [B, n_next, b], new_cand_pos int32 [B, 4], new_cand_tok int32 [B, 4])."""
    import torch
    B, S, b = drafts.shape
    want = {"drafts": (drafts, torch.int32, (B, S, b)), "conf": (conf, torch.float32, (B, S, b)),
            "argmax": (argmax, torch.int32, (B, S, b)), "unmask": (unmask, torch.uint8, (B, S, b)),
            "cand_pos": (cand_pos, torch.int32, (B, 4)), "cand_tok": (cand_tok, torch.int32, (B, 4))}
    for name, (t, dt, shp) in want.items():
        if t.dtype != dt or tuple(t.shape) != shp or not t.is_contiguous() or not t.is_cuda:
            raise TypeError("%s must be a contiguous CUDA tensor of dtype %s and shape %s" % (name, dt, shp))
    chosen = torch.empty((B,), dtype=torch.int32, device=drafts.device)
    new_drafts = torch.empty((B, max(int(n_next), 1), b), dtype=torch.int32, device=drafts.device)
    new_pos, new_tok = torch.empty_like(cand_pos), torch.empty_like(cand_tok)
    _check(lib().odb_speculative_jump(model, drafts.data_ptr(), conf.data_ptr(), argmax.data_ptr(), unmask.data_ptr(),
                                      cand_pos.data_ptr(), cand_tok.data_ptr(), B, b, S, n_next, chosen.data_ptr(),
                                      new_drafts.data_ptr(), new_pos.data_ptr(), new_tok.data_ptr(), _stream()))
    return chosen, new_drafts, new_pos, new_tok


def odb_block_step(model: int, cache: int, drafts, block_off: int, tau: float, conf=None, argmax=None, unmask=None):
    """drafts: int32 CUDA tensor [B, S, b] -> (conf f32, argmax int32, unmask uint8), each [B, S, b]."""
    import torch
    B, S, b = drafts.shape
    if conf is None:
        conf = torch.empty((B, S, b), dtype=torch.float32, device=drafts.device)
    if argmax is None:
        argmax = torch.empty((B, S, b), dtype=torch.int32, device=drafts.device)
    if unmask is None:
        unmask = torch.empty((B, S, b), dtype=torch.uint8, device=drafts.device)
    _check(lib().odb_block_step(model, cache, _dev_i32(drafts), block_off, b, S, tau, conf.data_ptr(),
                                argmax.data_ptr(), unmask.data_ptr(), _stream()))
    return conf, argmax, unmask


def odb_block_step_static(model: int, cache: int, drafts, block_off: int, tau: float, conf, argmax, unmask):
    """odb_block_step in the library's fixed scratch area; the caller brings every output tensor (nothing is
    allocated on the way, here or in the library)."""
    B, S, b = drafts.shape
    _check(lib().odb_block_step_static(model, cache, _dev_i32(drafts), block_off, b, S, tau, conf.data_ptr(),
                                       argmax.data_ptr(), unmask.data_ptr(), _stream()))
    return conf, argmax, unmask


def odb_prefill_logits(model: int, cache: int, tokens, resp_off: int, vocab: int):
    import torch
    B, L = tokens.shape
    logits = torch.empty((B, L - resp_off, vocab), dtype=torch.float32, device=tokens.device)
    _check(lib().odb_prefill_logits(model, cache, _dev_i32(tokens), L, resp_off, logits.data_ptr(), _stream()))
    return logits


def odb_block_step_logits(model: int, cache: int, drafts, block_off: int, vocab: int):
    import torch
    B, S, b = drafts.shape
    logits = torch.empty((B, S, b, vocab), dtype=torch.float32, device=drafts.device)
    _check(lib().odb_block_step_logits(model, cache, _dev_i32(drafts), block_off, b, S, logits.data_ptr(),
                                       _stream()))
    return logits


def odb_cache_read(cache: int, layer: int, kv: int, batch_index: int, pos0: int, n: int, n_heads: int,
                   head_dim: int) -> np.ndarray:
    out = np.empty((n, n_heads, head_dim), np.float32)
    _check(lib().odb_cache_read(cache, layer, kv, batch_index, pos0, n, out.ctypes.data))
    return out


def odb_set_option(model: int, option: int, value: int) -> None:
    _check(lib().odb_set_option(model, option, value))


def odb_model_status(model: int) -> None:
    _check(lib().odb_model_status(model))


def odb_profile_begin(model: int, kernel_class: int, max_launches: int) -> None:
    _check(lib().odb_profile_begin(model, kernel_class, max_launches))


def odb_profile_end(model: int) -> Tuple[int, float, float]:
    """-> (timed launches, sum of their event-pair durations in ms, sum of the empty pairs recorded behind them)."""
    n, ms, empty = ctypes.c_int(), ctypes.c_float(), ctypes.c_float()
    _check(lib().odb_profile_end(model, ctypes.byref(n), ctypes.byref(ms), ctypes.byref(empty)))
    return n.value, ms.value, empty.value


def odb_profile_kernel(model: int, run, steps: int, kernel_class: int = 3, max_launches: int = 1 << 16) -> Dict:
    """Average on-stream duration of one kernel class over `steps` calls of run()."""
    odb_profile_begin(model, kernel_class, max_launches)
    try:
        for _ in range(steps):
            run()
    finally:
        n, ms, empty = odb_profile_end(model)
    return {"kernel": KERNEL_CLASSES[kernel_class], "launches": n, "avg_ms": ms / max(n, 1),
            "avg_empty_pair_ms": empty / max(n, 1)}


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widening of bf16 bit patterns (pure reinterpretation, no arithmetic)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
