"""ctypes binding of ``include/pcm.h``: same names, argument marshalling only.

PyTorch provides device memory (tensors) and the stream; nothing is computed here.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Tuple

import torch

PCM_F32, PCM_BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpcm.so")
_MEASURE_LIB_PATH = os.path.join(_HERE, "libpcm_measure.so")
_lib = None
_measure_lib = None


class PcmError(RuntimeError):
    pass


def library_path() -> str:
    return _LIB_PATH


class LossOptions(C.Structure):
    """pcm_loss_options of include/pcm.h."""
    _fields_ = [("eps_low", C.c_float), ("eps_high", C.c_float), ("loss_scale", C.c_float),
                ("entropy_coef", C.c_float), ("normalisation", C.c_int), ("ratio_level", C.c_int),
                ("chunk_weight", C.c_void_p), ("head_evaluation", C.c_int), ("panel_rows", C.c_int),
                ("packed_weights", C.c_void_p), ("dense_backward", C.c_int), ("grad_sumsq_out", C.c_void_p)]


def _sig(fn, res, args):
    fn.restype = res
    fn.argtypes = args


def lib() -> C.CDLL:
    """The loaded C library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise PcmError(f"{_LIB_PATH} is missing: build it with `python -m paper_2605_16154_amd.build` "
                       "(or __graft_entry__.build()); there is no fallback path")
    L = C.CDLL(_LIB_PATH)
    vp, i32, i64, u64, f32, f64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_uint64, C.c_float, C.c_double, C.c_size_t
    _sig(L.pcm_version, C.c_char_p, [])
    _sig(L.pcm_status_string, C.c_char_p, [i32])
    _sig(L.pcm_state_bytes, sz, [i32])
    _sig(L.pcm_state_init, i32, [vp, i32, vp])
    _sig(L.pcm_label_phases, i32, [vp, vp, i32, i32, i32, i32, i32, f32, vp, vp])
    _sig(L.pcm_score_phases_workspace_bytes, sz, [i32] * 5)
    _sig(L.pcm_score_phases, i32, [vp, vp, vp, vp, i32, i32, i32, i32, i32, f64, vp, vp, vp, vp, vp, sz, vp])
    _sig(L.pcm_score_phases_static, i32, [vp, vp, vp, vp, i32, i32, i32, i32, i32, f64, vp, vp, vp, vp, vp])
    _sig(L.pcm_update_keep_probs, i32, [vp, vp, vp, i32, f64, i32, vp, vp])
    _sig(L.pcm_sample_chunks_workspace_bytes, sz, [i32] * 4)
    _sig(L.pcm_sample_chunks, i32, [vp, vp, vp, vp, i32, i32, i32, i32, u64, u64, vp, vp, vp, vp, sz, vp])
    _sig(L.pcm_sample_chunks_ex, i32, [vp, vp, vp, vp, i32, i32, i32, i32, i32, u64, u64, vp, vp, vp, vp, sz, vp])
    _sig(L.pcm_importance_weights, i32, [vp, vp, vp, vp, i32, i32, i32, vp, vp])
    _sig(L.pcm_kept_phase_counts, i32, [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp])
    _sig(L.pcm_packed_head_bytes, sz, [i32] * 3)
    _sig(L.pcm_pack_head_weights, i32, [vp, vp, vp, vp, i32, i32, i32, vp, vp])
    _sig(L.grpo_masked_actor_step_workspace_bytes, sz, [i32] * 7)
    _sig(L.grpo_masked_actor_step_ex_workspace_bytes, sz, [i32] * 7 + [C.POINTER(LossOptions)])
    _sig(L.grpo_masked_actor_step, i32,
         [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, f32, f32, f32,
          vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp])
    _sig(L.grpo_masked_actor_step_ex, i32,
         [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, C.POINTER(LossOptions),
          vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp])
    _sig(L.pcm_adamw_clip_step_workspace_bytes, sz, [i32, C.POINTER(i64)])
    _sig(L.pcm_adamw_clip_step, i32,
         [i32, C.POINTER(i64), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), i64,
          f64, f64, f64, f64, f64, f64, vp, vp, sz, vp])
    _sig(L.pcm_adamw_clip_step_ex, i32,
         [i32, C.POINTER(i64), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), i64,
          f64, f64, f64, f64, f64, f64, vp, vp, vp, sz, vp])
    _sig(L.pcm_profile_enable, i32, [i32])
    _sig(L.pcm_profile_stage_count, i32, [])
    _sig(L.pcm_profile_stage_name, C.c_char_p, [i32])
    _sig(L.pcm_profile_collect, i32, [C.POINTER(f64), C.POINTER(i64)])
    _lib = L
    return L


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise PcmError(f"{what} failed: {lib().pcm_status_string(rc).decode()} ({rc})")


def _ptr(t: Optional[torch.Tensor], dtype=None, name: str = "tensor") -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise PcmError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise PcmError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise PcmError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


_workspaces: Dict[torch.device, torch.Tensor] = {}


def _workspace(nbytes: int, device) -> Tuple[Optional[int], int]:
    """One growing scratch tensor per device, shared by all calls (they are stream-ordered)."""
    if nbytes == 0:
        return None, 0
    dev = torch.device(device)
    ws = _workspaces.get(dev)
    if ws is None or ws.numel() < nbytes:
        _workspaces[dev] = ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    return ws.data_ptr(), ws.numel()


def pcm_version() -> str:
    return lib().pcm_version().decode()


def pcm_state_bytes(K: int) -> int:
    return lib().pcm_state_bytes(K)


def pcm_state_init(K: int, device="cuda") -> torch.Tensor:
    """Allocates and initialises the keep-probability state block (int64 words)."""
    nbytes = pcm_state_bytes(K)
    if nbytes == 0:
        raise PcmError("pcm_state_bytes: K out of range")
    state = torch.empty(nbytes // 8, dtype=torch.int64, device=device)
    _check(lib().pcm_state_init(state.data_ptr(), K, _stream()), "pcm_state_init")
    return state


def pcm_label_phases(actions, n_chunks, L: int, D: int, gripper_dim: Optional[int] = None, close_threshold: float = 0.0,
                     out=None):
    """actions f32 [T, N, L*D] -> phase u8 [T, N] (0 approach, 1 pre-grasp, 2 active-grip, 3 release-ramp, 4 tail)."""
    T, N, A = actions.shape
    if A != L * D:
        raise PcmError("actions must be [T, N, L*D]")
    if out is None:
        out = torch.empty((T, N), dtype=torch.uint8, device=actions.device)
    g = D - 1 if gripper_dim is None else gripper_dim
    rc = lib().pcm_label_phases(_ptr(actions, torch.float32, "actions"), _ptr(n_chunks, torch.int32, "n_chunks"), T, N,
                                L, D, g, close_threshold, _ptr(out, torch.uint8, "phase"), _stream())
    _check(rc, "pcm_label_phases")
    return out


def pcm_score_phases(actions, phase, reward, n_chunks, n_groups: int, G: int, K: int, adv_eps: float = 1e-6,
                     out=None, static_scratch: bool = False):
    """-> (C f64[K], valid u8[K], adv f32[T], active u8[T]).

    static_scratch=True calls pcm_score_phases_static (no workspace; `out` must then be given if the call
    itself is to allocate nothing)."""
    T, N, A = actions.shape
    dev = actions.device
    if out is None:
        out = (torch.empty(K, dtype=torch.float64, device=dev), torch.empty(K, dtype=torch.uint8, device=dev),
               torch.empty(T, dtype=torch.float32, device=dev), torch.empty(T, dtype=torch.uint8, device=dev))
    Cc, valid, adv, active = out
    args = (_ptr(actions, torch.float32, "actions"), _ptr(phase, torch.uint8, "phase"),
            _ptr(reward, torch.uint8, "reward"), _ptr(n_chunks, torch.int32, "n_chunks"),
            n_groups, G, N, A, K, adv_eps, _ptr(Cc, torch.float64, "C_out"),
            _ptr(valid, torch.uint8, "valid_out"), _ptr(adv, torch.float32, "adv_out"),
            _ptr(active, torch.uint8, "active_out"))
    if static_scratch:
        _check(lib().pcm_score_phases_static(*args, _stream()), "pcm_score_phases_static")
        return out
    need = lib().pcm_score_phases_workspace_bytes(n_groups, G, N, A, K)
    ws, ws_bytes = _workspace(need, dev)
    _check(lib().pcm_score_phases(*args, ws, ws_bytes, _stream()), "pcm_score_phases")
    return out


def pcm_update_keep_probs(state, Cc, valid, p_min: float = 0.1, T_rc: int = 5, keep_probs_out=None):
    K = Cc.shape[0]
    if keep_probs_out is None:
        keep_probs_out = torch.empty(K, dtype=torch.float64, device=Cc.device)
    rc = lib().pcm_update_keep_probs(_ptr(state, torch.int64, "state"), _ptr(Cc, torch.float64, "C"),
                                     _ptr(valid, torch.uint8, "valid"), K, p_min, T_rc,
                                     _ptr(keep_probs_out, torch.float64, "keep_probs_out"), _stream())
    _check(rc, "pcm_update_keep_probs")
    return keep_probs_out


SELECTORS = {"pcm": 0, "random": 1, "top_phase": 2, "stratified": 3}


def pcm_sample_chunks(keep_probs, phase, n_chunks, active, B: int, seed: int, step: int, out=None,
                      selector: str = "pcm"):
    """-> (kept_idx i32[T*min(B,N)], kept_offsets i32[T+1], n_kept i32[1]).

    selector "pcm" calls pcm_sample_chunks; "random" and "top_phase" (the ablations) pcm_sample_chunks_ex.
    """
    if selector not in SELECTORS:
        raise PcmError(f"unknown selector {selector!r}")
    T, N = phase.shape
    K = keep_probs.shape[0]
    dev = phase.device
    if out is None:
        out = (torch.empty(T * min(B, N), dtype=torch.int32, device=dev),
               torch.empty(T + 1, dtype=torch.int32, device=dev), torch.empty(1, dtype=torch.int32, device=dev))
    kept_idx, kept_offsets, n_kept = out
    need = lib().pcm_sample_chunks_workspace_bytes(T, N, K, B)
    ws, ws_bytes = _workspace(need, dev)
    head = (_ptr(keep_probs, torch.float64, "keep_probs"), _ptr(phase, torch.uint8, "phase"),
            _ptr(n_chunks, torch.int32, "n_chunks"), _ptr(active, torch.uint8, "active"), T, N, K, B)
    tail = (seed & 0xFFFFFFFFFFFFFFFF, step & 0xFFFFFFFFFFFFFFFF, _ptr(kept_idx, torch.int32, "kept_idx"),
            _ptr(kept_offsets, torch.int32, "kept_offsets"), _ptr(n_kept, torch.int32, "n_kept"), ws, ws_bytes, _stream())
    if selector == "pcm":
        _check(lib().pcm_sample_chunks(*head, *tail), "pcm_sample_chunks")
    else:
        _check(lib().pcm_sample_chunks_ex(*head, SELECTORS[selector], *tail), "pcm_sample_chunks_ex")
    return out


def pcm_importance_weights(phase, n_chunks, kept_idx, kept_offsets, K: int, out=None):
    """-> f32 [len(kept_idx)]: N_c / b_c per kept chunk (entries beyond the kept count are left as they are)."""
    T, N = phase.shape
    if out is None:
        out = torch.zeros(kept_idx.shape[0], dtype=torch.float32, device=phase.device)
    rc = lib().pcm_importance_weights(_ptr(phase, torch.uint8, "phase"), _ptr(n_chunks, torch.int32, "n_chunks"),
                                      _ptr(kept_idx, torch.int32, "kept_idx"),
                                      _ptr(kept_offsets, torch.int32, "kept_offsets"), T, N, K,
                                      _ptr(out, torch.float32, "weights"), _stream())
    _check(rc, "pcm_importance_weights")
    return out


def pcm_kept_phase_counts(phase, n_chunks, active, kept_idx, n_kept, K: int, out=None):
    """-> (kept i32[K], eligible i32[K]): kept chunks per phase and the chunk slots that could have been kept."""
    T, N = phase.shape
    if out is None:
        out = (torch.empty(K, dtype=torch.int32, device=phase.device), torch.empty(K, dtype=torch.int32, device=phase.device))
    rc = lib().pcm_kept_phase_counts(_ptr(phase, torch.uint8, "phase"), _ptr(n_chunks, torch.int32, "n_chunks"),
                                     _ptr(active, torch.uint8, "active"), _ptr(kept_idx, torch.int32, "kept_idx"),
                                     _ptr(n_kept, torch.int32, "n_kept"), kept_idx.shape[0], T, N, K,
                                     _ptr(out[0], torch.int32, "kept_per_phase"), _ptr(out[1], torch.int32, "chunks_per_phase"),
                                     _stream())
    _check(rc, "pcm_kept_phase_counts")
    return out


def pcm_pack_head_weights(Wg, Wu, Wd, Wo, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """bf16 [d, ff], [d, ff], [ff, d], [d, V] -> u8 buffer holding the forward products' operand layouts."""
    d, ff = Wg.shape
    V = Wo.shape[1]
    nbytes = lib().pcm_packed_head_bytes(d, ff, V)
    if nbytes == 0:
        raise PcmError("pcm_pack_head_weights: unsupported head shape")
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=Wg.device)
    rc = lib().pcm_pack_head_weights(_ptr(Wg, torch.bfloat16, "Wg"), _ptr(Wu, torch.bfloat16, "Wu"),
                                     _ptr(Wd, torch.bfloat16, "Wd"), _ptr(Wo, torch.bfloat16, "Wo"), d, ff, V,
                                     _ptr(out, torch.uint8, "packed"), _stream())
    _check(rc, "pcm_pack_head_weights")
    return out


def grpo_masked_actor_step_workspace_bytes(max_kept_chunks, A, d, ff, V, dtype, want_grads) -> int:
    return lib().grpo_masked_actor_step_workspace_bytes(max_kept_chunks, A, d, ff, V, dtype, int(want_grads))


def grpo_masked_actor_step(hidden, tokens, logp_old, adv, kept_idx, n_kept, T: int, N: int, A: int,
                           Wg, Wu, Wd, Wo, eps_low: float = 0.2, eps_high: float = 0.2, loss_scale: float = 1.0,
                           want_grads: bool = True, want_dX: bool = True, max_kept_chunks: Optional[int] = None,
                           out: Optional[Dict[str, torch.Tensor]] = None, token_mean: bool = False,
                           entropy_coef: float = 0.0, chunk_ratio: bool = False,
                           chunk_weight: Optional[torch.Tensor] = None,
                           composed_head: bool = False, panel_rows: int = 0,
                           packed_weights: Optional[torch.Tensor] = None,
                           dense_backward: bool = False, grad_sumsq: bool = False) -> Dict[str, torch.Tensor]:
    """-> dict(loss f32[1], logp f32[max_kept*A], stats f32[5], and if requested dWg, dWu, dWd, dWo, dX).

    `out` may carry preallocated tensors under those names (they are reused, not reallocated).  With none of
    token_mean, entropy_coef, chunk_ratio, chunk_weight, composed_head set this is grpo_masked_actor_step
    (stats[4] stays 0); otherwise grpo_masked_actor_step_ex.  composed_head = PCM_HEAD_COMPOSED (down and logit
    projection applied as one matrix); panel_rows = target height of the row panels of the bf16 path (0: default);
    packed_weights = the operand layouts from pcm_pack_head_weights (the step then skips its own weight re-layout);
    dense_backward = backward products over all kept rows, also those whose gradient is zero (bf16 path);
    grad_sumsq = also return "grad_sumsq" (f64[1]): the sum of the squares of the four weight gradients, for
    pcm_adamw_clip_step(grad_sumsq=...).
    """
    dev = hidden.device
    d, ff = Wg.shape
    V = Wo.shape[1]
    if hidden.dtype == torch.float32:
        dtype = PCM_F32
    elif hidden.dtype == torch.bfloat16:
        dtype = PCM_BF16
    else:
        raise PcmError(f"hidden must be float32 or bfloat16, got {hidden.dtype}")
    for name, w, shape in (("Wg", Wg, (d, ff)), ("Wu", Wu, (d, ff)), ("Wd", Wd, (ff, d)), ("Wo", Wo, (d, V))):
        if tuple(w.shape) != shape or w.dtype != hidden.dtype:
            raise PcmError(f"{name} must be {shape} of {hidden.dtype}")
    if hidden.shape != (T * N * A, d):
        raise PcmError("hidden must be [T*N*A, d]")
    if max_kept_chunks is None:
        max_kept_chunks = kept_idx.shape[0]
    if kept_idx.shape[0] < max_kept_chunks:
        raise PcmError("kept_idx is shorter than max_kept_chunks")
    rows = max_kept_chunks * A
    out = {} if out is None else out

    def buf(name, shape, dt):
        t = out.get(name)
        if t is None:
            out[name] = t = torch.empty(shape, dtype=dt, device=dev)
        elif tuple(t.shape) != tuple(shape):
            raise PcmError(f"out[{name!r}] has shape {tuple(t.shape)}, expected {tuple(shape)}")
        return t

    loss = buf("loss", (1,), torch.float32)
    logp = buf("logp", (rows,), torch.float32)
    if "stats" not in out:
        out["stats"] = torch.zeros(5, dtype=torch.float32, device=dev)
    stats = buf("stats", (5,), torch.float32)
    grads = [None] * 4
    if want_grads:
        grads = [buf("dWg", (d, ff), torch.float32), buf("dWu", (d, ff), torch.float32),
                 buf("dWd", (ff, d), torch.float32), buf("dWo", (d, V), torch.float32)]
    dX = buf("dX", (rows, d), hidden.dtype) if want_dX else None
    extended = (token_mean or entropy_coef != 0.0 or chunk_ratio or chunk_weight is not None or composed_head
                or panel_rows != 0 or packed_weights is not None or dense_backward or grad_sumsq)
    sumsq = buf("grad_sumsq", (1,), torch.float64) if grad_sumsq else None
    opt = None
    if extended:
        if chunk_weight is not None and chunk_weight.shape[0] < max_kept_chunks:
            raise PcmError("chunk_weight is shorter than max_kept_chunks")
        opt = LossOptions(eps_low, eps_high, loss_scale, entropy_coef, int(token_mean), int(chunk_ratio),
                          _ptr(chunk_weight, torch.float32, "chunk_weight"), int(composed_head), int(panel_rows),
                          _ptr(packed_weights, torch.uint8, "packed_weights"), int(dense_backward),
                          _ptr(sumsq, torch.float64, "grad_sumsq"))
        need = lib().grpo_masked_actor_step_ex_workspace_bytes(max_kept_chunks, A, d, ff, V, dtype,
                                                               int(want_grads or want_dX), C.byref(opt))
    else:
        need = grpo_masked_actor_step_workspace_bytes(max_kept_chunks, A, d, ff, V, dtype, want_grads or want_dX)
    if need == 0:
        raise PcmError("grpo_masked_actor_step: unsupported shape or dtype for this path")
    ws, ws_bytes = _workspace(need, dev)
    head = (_ptr(hidden, None, "hidden"), _ptr(tokens, torch.uint8, "tokens"), _ptr(logp_old, torch.float32, "logp_old"),
            _ptr(adv, torch.float32, "adv"), _ptr(kept_idx, torch.int32, "kept_idx"), _ptr(n_kept, torch.int32, "n_kept"),
            max_kept_chunks, T, N, A, d, ff, V, dtype, _ptr(Wg, None, "Wg"), _ptr(Wu, None, "Wu"), _ptr(Wd, None, "Wd"),
            _ptr(Wo, None, "Wo"))
    tail = (_ptr(loss, torch.float32, "loss"), _ptr(logp, torch.float32, "logp"),
            *[_ptr(g, torch.float32, "dW") for g in grads], _ptr(dX, None, "dX"), _ptr(stats, torch.float32, "stats"),
            ws, ws_bytes, _stream())
    if extended:
        rc = lib().grpo_masked_actor_step_ex(*head, C.byref(opt), *tail)
        _check(rc, "grpo_masked_actor_step_ex")
    else:
        rc = lib().grpo_masked_actor_step(*head, eps_low, eps_high, loss_scale, *tail)
        _check(rc, "grpo_masked_actor_step")
    return out


def pcm_adamw_clip_step(grads, weights, m, v, step: int, lr: float = 1e-5, beta1: float = 0.9, beta2: float = 0.999,
                        eps: float = 1e-8, weight_decay: float = 0.0, max_grad_norm: float = 2.0, weights_bf16=None,
                        grad_norm_out: Optional[torch.Tensor] = None,
                        grad_sumsq: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Global-norm clipping + AdamW over lists of fp32 tensors (updated in place); -> grad norm f32[1].

    `weights_bf16`, if given, is a list (entries may be None) of bf16 tensors that receive the new weights.
    `grad_sumsq` (f64[1], as the actor step returns it) is the sum of the squares of all gradient elements: the call
    is then pcm_adamw_clip_step_ex, which reads the gradients once instead of twice.
    """
    n = len(grads)
    if not (len(weights) == len(m) == len(v) == n) or (weights_bf16 is not None and len(weights_bf16) != n):
        raise PcmError("pcm_adamw_clip_step: lists must have equal length")
    dev = grads[0].device
    for g, w, mi, vi in zip(grads, weights, m, v):
        if not (g.numel() == w.numel() == mi.numel() == vi.numel()):
            raise PcmError("pcm_adamw_clip_step: gradient, weight and moment tensors must have equal sizes")
    numel = (C.c_int64 * n)(*[g.numel() for g in grads])
    arr = lambda ts, dt, name: (C.c_void_p * n)(*[_ptr(t, dt, name) for t in ts])
    lowp = None
    if weights_bf16 is not None:
        for w, b in zip(weights, weights_bf16):
            if b is not None and b.numel() != w.numel():
                raise PcmError("pcm_adamw_clip_step: bf16 copy must have the size of its weight tensor")
        lowp = arr(weights_bf16, torch.bfloat16, "weights_bf16")
    if grad_norm_out is None:
        grad_norm_out = torch.empty(1, dtype=torch.float32, device=dev)
    need = lib().pcm_adamw_clip_step_workspace_bytes(n, numel)
    if need == 0:
        raise PcmError("pcm_adamw_clip_step: bad tensor list")
    ws, ws_bytes = _workspace(need, dev)
    head = (n, numel, arr(grads, torch.float32, "grads"), arr(weights, torch.float32, "weights"),
            arr(m, torch.float32, "m"), arr(v, torch.float32, "v"), lowp, step, lr, beta1, beta2, eps, weight_decay,
            max_grad_norm)
    tail = (_ptr(grad_norm_out, torch.float32, "norm"), ws, ws_bytes, _stream())
    if grad_sumsq is not None:
        rc = lib().pcm_adamw_clip_step_ex(*head, _ptr(grad_sumsq, torch.float64, "grad_sumsq"), *tail)
    else:
        rc = lib().pcm_adamw_clip_step(*head, *tail)
    _check(rc, "pcm_adamw_clip_step")
    return grad_norm_out


def pcm_measure_mfma_rate(random_operands: bool = True, milliseconds: int = 100) -> Tuple[float, float]:
    """-> (TFLOP/s, shader clock in GHz) that the bf16 matrix cores sustain on their own, on zeros or random data.

    A measurement aid from its own library (libpcm_measure.so, include/pcm_measure.h), not a step of the path."""
    global _measure_lib
    if _measure_lib is None:
        if not os.path.exists(_MEASURE_LIB_PATH):
            raise PcmError(f"{_MEASURE_LIB_PATH} is missing: build it with `python -m paper_2605_16154_amd.build`")
        _measure_lib = C.CDLL(_MEASURE_LIB_PATH)
        _sig(_measure_lib.pcm_measure_mfma_rate, C.c_int, [C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)])
    tf, clk = C.c_double(0.0), C.c_double(0.0)
    _check(_measure_lib.pcm_measure_mfma_rate(int(random_operands), milliseconds, C.byref(tf), C.byref(clk)),
           "pcm_measure_mfma_rate")
    return tf.value, clk.value


def pcm_profile_enable(on: bool) -> None:
    _check(lib().pcm_profile_enable(int(on)), "pcm_profile_enable")


def pcm_profile_collect() -> Dict[str, Tuple[float, int]]:
    """-> {stage name: (total milliseconds, launches)} accumulated since profiling was enabled."""
    n = lib().pcm_profile_stage_count()
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(lib().pcm_profile_collect(ms, cnt), "pcm_profile_collect")
    return {lib().pcm_profile_stage_name(i).decode(): (ms[i], cnt[i]) for i in range(n)}
