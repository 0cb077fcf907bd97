"""Thin ctypes binding over libsapo.so (the C ABI declared in include/sapo.h).

Argument marshalling only: every step of rollout generation and scoring runs in
the HIP kernels of the library.  torch is used for device memory and streams.
There is no CPU fallback: if the library has not been built, or there is no
GPU, the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsapo.so")

SAPO_OK, SAPO_EINVAL, SAPO_ESHAPE, SAPO_EWORKSPACE, SAPO_EHIP = 0, -1, -2, -3, -4
SAPO_DTYPE_F32, SAPO_DTYPE_BF16 = 0, 1


class SapoError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("libsapo error %d: %s" % (code, msg))
        self.code = code


class sapo_model_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ff", C.c_int32),
                ("vocab", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float),
                ("tied_embeddings", C.c_int32), ("dtype", C.c_int32), ("kv_page_tokens", C.c_int32),
                ("max_seq", C.c_int32)]


class sapo_adam_config(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float)]


_lib = None


def load_library() -> C.CDLL:
    """Load libsapo.so built in-tree; raise if it is missing (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libsapo.so is not built: run `python -m paper_2509_08721_amd.build` "
                           "(expected at %s)" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i32, u64, u32, sz, f32 = C.c_void_p, C.c_int, C.c_uint64, C.c_uint32, C.c_size_t, C.c_float
    lib.sapo_weights_create.argtypes = [C.POINTER(sapo_model_config), C.POINTER(vp), i32, vp, C.POINTER(vp)]
    lib.sapo_weights_create.restype = i32
    lib.sapo_weights_destroy.argtypes = [vp]
    lib.sapo_weights_destroy.restype = None
    lib.sapo_weights_set_qkv_bias.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.sapo_weights_set_qkv_bias.restype = i32
    lib.sapo_weights_uses_mfma.argtypes = [vp]
    lib.sapo_weights_uses_mfma.restype = i32
    lib.sapo_rollout_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    lib.sapo_rollout_workspace_bytes.restype = sz
    lib.sapo_score_workspace_bytes.argtypes = [vp, i32, i32]
    lib.sapo_score_workspace_bytes.restype = sz
    lib.sapo_debug_logits_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.sapo_debug_logits_workspace_bytes.restype = sz
    lib.sapo_rollout_generate.argtypes = [vp, vp, i32, i32, i32, i32, f32, u64, vp, vp, vp, sz, vp]
    lib.sapo_rollout_generate.restype = i32
    lib.sapo_rollout_generate_stop.argtypes = [vp, vp, i32, i32, i32, i32, f32, u64, i32, vp, vp, vp, vp, sz, vp]
    lib.sapo_rollout_generate_stop.restype = i32
    lib.sapo_device_info.argtypes = [vp]
    lib.sapo_device_info.restype = i32
    lib.sapo_debug_read_probe.argtypes = [vp, sz, vp, vp]
    lib.sapo_debug_read_probe.restype = i32
    lib.sapo_debug_mfma_probe.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.sapo_debug_mfma_probe.restype = i32
    lib.sapo_weights_update.argtypes = [vp, C.POINTER(vp), i32, vp]
    lib.sapo_weights_update.restype = i32
    lib.sapo_rollout_last_stats.argtypes = [vp, vp]
    lib.sapo_rollout_last_stats.restype = i32
    lib.sapo_rollout_generate_ragged.argtypes = [vp, vp, vp, i32, i32, i32, i32, f32, u64, i32, vp, vp, vp, vp, sz, vp]
    lib.sapo_rollout_generate_ragged.restype = i32
    lib.sapo_score_logprobs.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.sapo_score_logprobs.restype = i32
    lib.sapo_score_logprobs_at.argtypes = [vp, vp, vp, vp, i32, i32, i32, f32, vp, vp, vp, sz, vp]
    lib.sapo_score_logprobs_at.restype = i32
    lib.sapo_assemble_workspace_bytes.argtypes = [i32, i32]
    lib.sapo_assemble_workspace_bytes.restype = sz
    lib.sapo_assemble_training_set.argtypes = [vp, vp, i32, vp, vp, i32, i32, i32, i32, i32, u64, vp, vp, vp, vp, vp, sz, vp]
    lib.sapo_assemble_training_set.restype = i32
    lib.sapo_surrogate_workspace_bytes.argtypes = []
    lib.sapo_surrogate_workspace_bytes.restype = sz
    lib.sapo_clipped_surrogate.argtypes = [vp, vp, vp, vp, i32, i32, f32, f32, vp, vp, vp, sz, vp]
    lib.sapo_clipped_surrogate.restype = i32
    lib.sapo_clipped_surrogate_noalloc.argtypes = [vp, vp, vp, vp, i32, i32, f32, f32, vp, vp, vp]
    lib.sapo_clipped_surrogate_noalloc.restype = i32
    lib.sapo_trainer_create.argtypes = [C.POINTER(sapo_model_config), C.POINTER(vp), i32, C.POINTER(sapo_adam_config), vp,
                                        C.POINTER(vp)]
    lib.sapo_trainer_create.restype = i32
    lib.sapo_trainer_destroy.argtypes = [vp]
    lib.sapo_trainer_destroy.restype = None
    lib.sapo_trainer_workspace_bytes.argtypes = [vp, i32, i32]
    lib.sapo_trainer_workspace_bytes.restype = sz
    lib.sapo_trainer_workspace_bytes_for.argtypes = [vp, i32, i32, i32]
    lib.sapo_trainer_workspace_bytes_for.restype = sz
    lib.sapo_policy_update.argtypes = [vp, vp, vp, vp, vp, i32, i32, f32, f32, vp, vp, vp, sz, vp]
    lib.sapo_policy_update.restype = i32
    lib.sapo_trainer_export.argtypes = [vp, C.POINTER(vp), i32, vp]
    lib.sapo_trainer_export.restype = i32
    lib.sapo_trainer_set_matmul_pieces.argtypes = [vp, i32]
    lib.sapo_trainer_set_matmul_pieces.restype = i32
    lib.sapo_trainer_set_qkv_bias.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.sapo_trainer_set_qkv_bias.restype = i32
    lib.sapo_trainer_get_qkv_bias.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.sapo_trainer_get_qkv_bias.restype = i32
    lib.sapo_trainer_steps.argtypes = [vp]
    lib.sapo_trainer_steps.restype = i32
    lib.sapo_trainer_read.argtypes = [vp, i32, i32, vp, sz, vp]
    lib.sapo_trainer_read.restype = i32
    lib.sapo_debug_logits.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp, sz, vp]
    lib.sapo_debug_logits.restype = i32
    lib.sapo_debug_half_clamped.argtypes = [vp, vp, i32, i32, vp, vp, sz, vp]
    lib.sapo_debug_half_clamped.restype = i32
    lib.sapo_weights_half_stats.argtypes = [vp, vp]
    lib.sapo_weights_half_stats.restype = i32
    lib.sapo_debug_gumbel.argtypes = [u64, u32, u32, u32, i32, vp, vp]
    lib.sapo_debug_gumbel.restype = i32
    lib.sapo_profile_kernel_count.argtypes = []
    lib.sapo_profile_kernel_count.restype = i32
    lib.sapo_profile_kernel_name.argtypes = [i32]
    lib.sapo_profile_kernel_name.restype = C.c_char_p
    lib.sapo_profile_start.argtypes = []
    lib.sapo_profile_start.restype = i32
    lib.sapo_profile_stop.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64), i32]
    lib.sapo_profile_stop.restype = i32
    lib.sapo_last_error.argtypes = []
    lib.sapo_last_error.restype = C.c_char_p
    _lib = lib
    return lib


EXPORTED = ["sapo_weights_create", "sapo_weights_update", "sapo_weights_destroy", "sapo_weights_uses_mfma", "sapo_weights_set_qkv_bias",
            "sapo_rollout_workspace_bytes", "sapo_score_workspace_bytes",
            "sapo_debug_logits_workspace_bytes", "sapo_rollout_generate", "sapo_rollout_generate_stop", "sapo_rollout_last_stats",
            "sapo_rollout_generate_ragged",
            "sapo_score_logprobs", "sapo_score_logprobs_at",
            "sapo_surrogate_workspace_bytes", "sapo_clipped_surrogate", "sapo_clipped_surrogate_noalloc",
            "sapo_assemble_workspace_bytes", "sapo_assemble_training_set",
            "sapo_trainer_create", "sapo_trainer_destroy", "sapo_trainer_workspace_bytes", "sapo_trainer_workspace_bytes_for",
            "sapo_policy_update",
            "sapo_trainer_export", "sapo_trainer_steps", "sapo_trainer_read", "sapo_trainer_set_matmul_pieces",
            "sapo_trainer_set_qkv_bias", "sapo_trainer_get_qkv_bias",
            "sapo_debug_logits", "sapo_debug_half_clamped", "sapo_weights_half_stats", "sapo_debug_gumbel", "sapo_debug_read_probe", "sapo_debug_mfma_probe", "sapo_device_info", "sapo_last_error", "sapo_profile_kernel_count",
            "sapo_profile_kernel_name", "sapo_profile_start", "sapo_profile_stop"]


def _check(rc: int):
    if rc != SAPO_OK:
        raise SapoError(rc, load_library().sapo_last_error().decode())


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: libsapo has no CPU path")
    return torch


def _stream_ptr(stream=None) -> int:
    torch = _torch()
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def make_config(shape) -> sapo_model_config:
    """workloads.ModelShape -> sapo_model_config."""
    return sapo_model_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                             shape.d_ff, shape.vocab, shape.rms_eps, shape.rope_theta,
                             1 if shape.tied_embeddings else 0,
                             SAPO_DTYPE_F32 if shape.dtype == "f32" else SAPO_DTYPE_BF16,
                             shape.kv_page_tokens, shape.max_seq)


class Weights:
    """Owner of a sapo_weights handle."""

    def __init__(self, handle: int, cfg: sapo_model_config):
        self.handle = handle
        self.cfg = cfg

    @property
    def uses_mfma(self) -> bool:
        return bool(load_library().sapo_weights_uses_mfma(self.handle))

    def close(self):
        if self.handle:
            load_library().sapo_weights_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _to_device(a: np.ndarray):
    """numpy array (float32, or uint16 holding bf16 bits) -> device tensor with the same bytes."""
    torch = _torch()
    t = torch.from_numpy(np.ascontiguousarray(a))
    if a.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def sapo_weights_create(shape, weights: dict, stream=None) -> Weights:
    """Upload the tensors of workloads.make_weights() and build the library's packed copy."""
    torch = _torch()
    lib = load_library()
    cfg = make_config(shape)
    order: List[Optional[np.ndarray]] = [weights["embed"]]
    for lw in weights["layers"]:
        order += [lw[k] for k in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]
    order += [weights["final_norm"], weights.get("lm_head")]
    dev = [None if a is None else _to_device(a) for a in order]
    ptrs = (C.c_void_p * len(dev))(*[None if t is None else t.data_ptr() for t in dev])
    out = C.c_void_p()
    _check(lib.sapo_weights_create(C.byref(cfg), ptrs, len(dev), _stream_ptr(stream), C.byref(out)))
    wts = Weights(out.value, cfg)
    for l, lw in enumerate(weights["layers"]):
        if "bq" in lw:
            sapo_weights_set_qkv_bias(wts, l, _to_device(lw["bq"]), _to_device(lw["bk"]), _to_device(lw["bv"]), stream)
    torch.cuda.synchronize()          # the originals in `dev` may be freed after this
    return wts


def sapo_weights_update(w: Weights, weights: dict, stream=None):
    """New values (a dict as for sapo_weights_create, same shapes) into an existing handle, in place."""
    torch = _torch()
    order: List[Optional[np.ndarray]] = [weights["embed"]]
    for lw in weights["layers"]:
        order += [lw[k] for k in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]
    order += [weights["final_norm"], weights.get("lm_head")]
    dev = [None if a is None else _to_device(a) for a in order]
    ptrs = (C.c_void_p * len(dev))(*[None if t is None else t.data_ptr() for t in dev])
    _check(load_library().sapo_weights_update(w.handle, ptrs, len(dev), _stream_ptr(stream)))
    for l, lw in enumerate(weights["layers"]):
        if "bq" in lw:
            sapo_weights_set_qkv_bias(w, l, _to_device(lw["bq"]), _to_device(lw["bk"]), _to_device(lw["bv"]), stream)
    torch.cuda.synchronize()          # the originals in `dev` may be freed after this


def sapo_weights_set_qkv_bias(w: Weights, layer: int, bq, bk, bv, stream=None):
    """bq float32 [Hq*hd], bk / bv float32 [Hkv*hd] device tensors."""
    torch = _torch()
    for t in (bq, bk, bv):
        assert t.dtype == torch.float32 and t.is_cuda and t.is_contiguous()
    _check(load_library().sapo_weights_set_qkv_bias(w.handle, layer, bq.data_ptr(), bk.data_ptr(), bv.data_ptr(),
                                                    _stream_ptr(stream)))
    torch.cuda.synchronize()


def sapo_weights_destroy(w: Weights):
    w.close()


def _workspace(nbytes: int):
    torch = _torch()
    if nbytes == 0:
        raise SapoError(SAPO_EINVAL, load_library().sapo_last_error().decode())
    return torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")


def _aligned_ptr(t) -> int:
    return (t.data_ptr() + 255) & ~255


def _ws_args(t):
    """(256-byte aligned pointer into a workspace tensor, bytes available from there)."""
    p = _aligned_ptr(t)
    return p, max(0, t.numel() * t.element_size() - (p - t.data_ptr()))


def sapo_rollout_workspace_bytes(w: Weights, P: int, Lp: int, G: int, max_new: int) -> int:
    return int(load_library().sapo_rollout_workspace_bytes(w.handle, P, Lp, G, max_new))


def sapo_score_workspace_bytes(w: Weights, S: int, T: int) -> int:
    return int(load_library().sapo_score_workspace_bytes(w.handle, S, T))


def sapo_rollout_generate(w: Weights, prompts, G: int, max_new: int, temperature: float, seed: int,
                          workspace=None, stream=None, out_tokens=None, out_logprobs=None):
    """prompts: int32 device tensor [P, Lp].  Returns (tokens int32 [P*G, max_new],
    logprobs float32 [P*G, max_new]) device tensors; work is enqueued on the stream."""
    torch = _torch()
    lib = load_library()
    P, Lp = int(prompts.shape[0]), int(prompts.shape[1])
    assert prompts.dtype == torch.int32 and prompts.is_cuda and prompts.is_contiguous()
    if out_tokens is None:
        out_tokens = torch.empty((P * G, max_new), dtype=torch.int32, device="cuda")
    if out_logprobs is None:
        out_logprobs = torch.empty((P * G, max_new), dtype=torch.float32, device="cuda")
    nbytes = sapo_rollout_workspace_bytes(w, P, Lp, G, max_new)
    if workspace is None:
        workspace = _workspace(nbytes)
    _check(lib.sapo_rollout_generate(w.handle, prompts.data_ptr(), P, Lp, G, max_new, float(temperature),
                                     int(seed), out_tokens.data_ptr(), out_logprobs.data_ptr(),
                                     *_ws_args(workspace), _stream_ptr(stream)))
    return out_tokens, out_logprobs


def sapo_rollout_generate_stop(w: Weights, prompts, G: int, max_new: int, temperature: float, seed: int,
                               stop_token: int, workspace=None, stream=None, out=None):
    """As sapo_rollout_generate with a stop token.  Returns (tokens, logprobs, lengths int32 [P*G]); `out`, if
    given, is such a triple of device tensors to write into (the captured decode step is reused between calls
    that pass the same buffers)."""
    torch = _torch()
    lib = load_library()
    P, Lp = int(prompts.shape[0]), int(prompts.shape[1])
    assert prompts.dtype == torch.int32 and prompts.is_cuda and prompts.is_contiguous()
    if out is not None:
        out_tokens, out_logprobs, out_lengths = out
        assert out_tokens.shape == (P * G, max_new) and out_tokens.dtype == torch.int32 and out_tokens.is_contiguous()
        assert out_logprobs.shape == (P * G, max_new) and out_logprobs.dtype == torch.float32 and out_logprobs.is_contiguous()
        assert out_lengths.shape == (P * G,) and out_lengths.dtype == torch.int32
    else:
        out_tokens = torch.empty((P * G, max_new), dtype=torch.int32, device="cuda")
        out_logprobs = torch.empty((P * G, max_new), dtype=torch.float32, device="cuda")
        out_lengths = torch.empty((P * G,), dtype=torch.int32, device="cuda")
    nbytes = sapo_rollout_workspace_bytes(w, P, Lp, G, max_new)
    if workspace is None:
        workspace = _workspace(nbytes)
    _check(lib.sapo_rollout_generate_stop(w.handle, prompts.data_ptr(), P, Lp, G, max_new, float(temperature),
                                          int(seed), int(stop_token), out_tokens.data_ptr(), out_logprobs.data_ptr(),
                                          out_lengths.data_ptr(), *_ws_args(workspace), _stream_ptr(stream)))
    return out_tokens, out_logprobs, out_lengths


def sapo_rollout_last_stats(w: Weights) -> dict:
    """Figures of the last rollout call on this handle: decode steps enqueued, compactions of the batch, rows per
    step at the end, ended sequences at the last look."""
    out = (C.c_int32 * 4)()
    _check(load_library().sapo_rollout_last_stats(w.handle, out))
    return {"steps": out[0], "compactions": out[1], "rows": out[2], "ended": out[3]}


def sapo_rollout_generate_ragged(w: Weights, prompts, prompt_lens, G: int, max_new: int, temperature: float, seed: int,
                                 stop_token: int = -1, workspace=None, stream=None):
    """prompts int32 device tensor [P, Lp_max] (rows padded), prompt_lens a host sequence of P lengths.
    Returns (tokens, logprobs, lengths or None)."""
    torch = _torch()
    lib = load_library()
    P, Lp = int(prompts.shape[0]), int(prompts.shape[1])
    assert prompts.dtype == torch.int32 and prompts.is_cuda and prompts.is_contiguous()
    lens = np.ascontiguousarray(np.asarray(prompt_lens, dtype=np.int32))
    assert lens.shape == (P,)
    out_tokens = torch.empty((P * G, max_new), dtype=torch.int32, device="cuda")
    out_logprobs = torch.empty((P * G, max_new), dtype=torch.float32, device="cuda")
    out_lengths = torch.empty((P * G,), dtype=torch.int32, device="cuda") if stop_token >= 0 else None
    nbytes = sapo_rollout_workspace_bytes(w, P, Lp, G, max_new)
    if workspace is None:
        workspace = _workspace(nbytes)
    _check(lib.sapo_rollout_generate_ragged(w.handle, prompts.data_ptr(), lens.ctypes.data, P, Lp, G, max_new,
                                            float(temperature), int(seed), int(stop_token), out_tokens.data_ptr(),
                                            out_logprobs.data_ptr(), None if out_lengths is None else out_lengths.data_ptr(),
                                            *_ws_args(workspace), _stream_ptr(stream)))
    return out_tokens, out_logprobs, out_lengths


def sapo_score_logprobs_at(w: Weights, tokens, completion_mask, rewards, G: int, temperature: float, workspace=None,
                           stream=None):
    """sapo_score_logprobs at a temperature: log softmax(z / temperature)[token]."""
    torch = _torch()
    lib = load_library()
    S, T = int(tokens.shape[0]), int(tokens.shape[1])
    assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.is_contiguous()
    assert completion_mask.dtype == torch.uint8 and completion_mask.is_cuda and completion_mask.is_contiguous()
    assert rewards.dtype == torch.float32 and rewards.is_cuda and rewards.is_contiguous()
    out_logprobs = torch.empty((S, T), dtype=torch.float32, device="cuda")
    out_advantages = torch.empty((S,), dtype=torch.float32, device="cuda")
    nbytes = sapo_score_workspace_bytes(w, S, T)
    if workspace is None:
        workspace = _workspace(nbytes)
    _check(lib.sapo_score_logprobs_at(w.handle, tokens.data_ptr(), completion_mask.data_ptr(), rewards.data_ptr(),
                                      S, T, G, float(temperature), out_logprobs.data_ptr(), out_advantages.data_ptr(),
                                      *_ws_args(workspace), _stream_ptr(stream)))
    return out_logprobs, out_advantages


def sapo_score_logprobs(w: Weights, tokens, completion_mask, rewards, G: int, workspace=None, stream=None,
                        out_logprobs=None, out_advantages=None):
    """tokens int32 [S, T], completion_mask uint8 [S, T], rewards float32 [S] (device tensors).
    Returns (logprobs float32 [S, T], advantages float32 [S])."""
    torch = _torch()
    lib = load_library()
    S, T = int(tokens.shape[0]), int(tokens.shape[1])
    assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.is_contiguous()
    assert completion_mask.dtype == torch.uint8 and completion_mask.is_cuda and completion_mask.is_contiguous()
    assert rewards.dtype == torch.float32 and rewards.is_cuda and rewards.is_contiguous()
    if out_logprobs is None:
        out_logprobs = torch.empty((S, T), dtype=torch.float32, device="cuda")
    if out_advantages is None:
        out_advantages = torch.empty((S,), dtype=torch.float32, device="cuda")
    nbytes = sapo_score_workspace_bytes(w, S, T)
    if workspace is None:
        workspace = _workspace(nbytes)
    _check(lib.sapo_score_logprobs(w.handle, tokens.data_ptr(), completion_mask.data_ptr(), rewards.data_ptr(),
                                   S, T, G, out_logprobs.data_ptr(), out_advantages.data_ptr(),
                                   *_ws_args(workspace), _stream_ptr(stream)))
    return out_logprobs, out_advantages


def sapo_assemble_workspace_bytes(n_local_pool: int, n_ext_pool: int) -> int:
    return int(load_library().sapo_assemble_workspace_bytes(n_local_pool, n_ext_pool))


def sapo_assemble_training_set(local_tokens, local_rewards, ext_tokens, ext_rewards, G: int, n_local: int, n_ext: int,
                               seed: int, workspace=None, stream=None):
    """Pools: tokens int32 [n_pool * G, T] and rewards float32 [n_pool * G] (device tensors; a pool may have 0 rows).
    Returns (tokens int32 [(n_local + n_ext) * G, T], rewards float32, source int32 [n_local + n_ext], counts int32 [2])."""
    torch = _torch()
    lib = load_library()
    T = int(local_tokens.shape[1]) if local_tokens.shape[0] else int(ext_tokens.shape[1])
    for tk, rw in ((local_tokens, local_rewards), (ext_tokens, ext_rewards)):
        assert tk.dtype == torch.int32 and tk.is_cuda and tk.is_contiguous() and rw.dtype == torch.float32 and rw.is_cuda
        assert tk.shape[0] % G == 0 and rw.numel() == tk.shape[0] and (tk.shape[0] == 0 or tk.shape[1] == T)
    pl, pe = int(local_tokens.shape[0]) // G, int(ext_tokens.shape[0]) // G
    n = n_local + n_ext
    out_t = torch.empty((n * G, T), dtype=torch.int32, device="cuda")
    out_r = torch.empty((n * G,), dtype=torch.float32, device="cuda")
    out_s = torch.empty((n,), dtype=torch.int32, device="cuda")
    out_c = torch.empty((2,), dtype=torch.int32, device="cuda")
    nbytes = sapo_assemble_workspace_bytes(pl, pe)
    if workspace is None:
        workspace = _workspace(max(nbytes, 256))
    _check(lib.sapo_assemble_training_set(local_tokens.data_ptr() if pl else None, local_rewards.data_ptr() if pl else None, pl,
                                          ext_tokens.data_ptr() if pe else None, ext_rewards.data_ptr() if pe else None, pe,
                                          G, T, n_local, n_ext, int(seed), out_t.data_ptr() if n else None,
                                          out_r.data_ptr() if n else None, out_s.data_ptr() if n else None, out_c.data_ptr(),
                                          *_ws_args(workspace), _stream_ptr(stream)))
    return out_t, out_r, out_s, out_c


def sapo_surrogate_workspace_bytes() -> int:
    return int(load_library().sapo_surrogate_workspace_bytes())


def sapo_clipped_surrogate(logp_new, logp_old, completion_mask, advantages, eps_low: float = 0.2,
                           eps_high: float = 0.28, want_grad: bool = True, workspace=None, stream=None):
    """logp_new / logp_old float32 [S, T], completion_mask uint8 [S, T], advantages float32 [S] (device).
    Returns (loss float32 [1], d loss / d logp_new float32 [S, T] or None)."""
    torch = _torch()
    lib = load_library()
    S, T = int(logp_new.shape[0]), int(logp_new.shape[1])
    for t in (logp_new, logp_old):
        assert t.dtype == torch.float32 and t.is_cuda and t.is_contiguous() and tuple(t.shape) == (S, T)
    assert completion_mask.dtype == torch.uint8 and completion_mask.is_cuda and completion_mask.is_contiguous()
    assert tuple(completion_mask.shape) == (S, T)
    assert advantages.dtype == torch.float32 and advantages.is_cuda and advantages.is_contiguous() and advantages.numel() == S
    loss = torch.empty((1,), dtype=torch.float32, device="cuda")
    grad = torch.empty((S, T), dtype=torch.float32, device="cuda") if want_grad else None
    nbytes = sapo_surrogate_workspace_bytes()
    if workspace is None:
        workspace = _workspace(nbytes)
    _check(lib.sapo_clipped_surrogate(logp_new.data_ptr(), logp_old.data_ptr(), completion_mask.data_ptr(),
                                      advantages.data_ptr(), S, T, eps_low, eps_high, loss.data_ptr(),
                                      grad.data_ptr() if want_grad else None, *_ws_args(workspace),
                                      _stream_ptr(stream)))
    return loss, grad


def sapo_clipped_surrogate_noalloc(logp_new, logp_old, completion_mask, advantages, out_loss, out_dlogp=None,
                                   eps_low: float = 0.2, eps_high: float = 0.28, stream=None):
    """sapo_clipped_surrogate without a workspace and without any allocation: the caller passes the outputs
    (out_loss float32 [1], out_dlogp float32 [S, T] or None); the library's scratch is a device array of its own."""
    torch = _torch()
    S, T = int(logp_new.shape[0]), int(logp_new.shape[1])
    for t in (logp_new, logp_old) + ((out_dlogp,) if out_dlogp is not None else ()):
        assert t.dtype == torch.float32 and t.is_cuda and t.is_contiguous() and tuple(t.shape) == (S, T)
    assert completion_mask.dtype == torch.uint8 and completion_mask.is_cuda and completion_mask.is_contiguous()
    assert tuple(completion_mask.shape) == (S, T)
    assert advantages.dtype == torch.float32 and advantages.is_cuda and advantages.is_contiguous() and advantages.numel() == S
    assert out_loss.dtype == torch.float32 and out_loss.is_cuda and out_loss.numel() >= 1
    _check(load_library().sapo_clipped_surrogate_noalloc(logp_new.data_ptr(), logp_old.data_ptr(), completion_mask.data_ptr(),
                                                         advantages.data_ptr(), S, T, eps_low, eps_high, out_loss.data_ptr(),
                                                         out_dlogp.data_ptr() if out_dlogp is not None else None,
                                                         _stream_ptr(stream)))
    return out_loss, out_dlogp


# --------------------------------------------------------------------------- #
# the local policy update
# --------------------------------------------------------------------------- #
LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def _tensor_order(weights: dict) -> list:
    order = [weights["embed"]]
    for lw in weights["layers"]:
        order += [lw[k] for k in LAYER_TENSORS]
    order.append(weights["final_norm"])
    if weights.get("lm_head") is not None:
        order.append(weights["lm_head"])
    return order


class Trainer:
    """Owner of a sapo_trainer handle."""

    def __init__(self, handle: int, cfg: sapo_model_config, shape, tensor_shapes):
        self.handle = handle
        self.cfg = cfg
        self.shape = shape
        self.tensor_shapes = tensor_shapes     # per tensor of the list: (shape tuple, is fp32 gain), then the bias vectors
        self.n_in = len(tensor_shapes)
        self.has_bias = False

    @property
    def steps(self) -> int:
        return int(load_library().sapo_trainer_steps(self.handle))

    def close(self):
        if self.handle:
            load_library().sapo_trainer_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def sapo_trainer_create(shape, weights: dict, lr: float = 1e-3, beta1: float = 0.9, beta2: float = 0.999,
                        eps: float = 1e-8, stream=None) -> Trainer:
    """Upload the tensors of workloads.make_weights() as the trainer's fp32 masters."""
    torch = _torch()
    lib = load_library()
    cfg = make_config(shape)
    order = _tensor_order(weights)
    dev = [_to_device(a) for a in order]
    ptrs = (C.c_void_p * len(dev))(*[t.data_ptr() for t in dev])
    opt = sapo_adam_config(lr, beta1, beta2, eps)
    out = C.c_void_p()
    _check(lib.sapo_trainer_create(C.byref(cfg), ptrs, len(dev), C.byref(opt), _stream_ptr(stream), C.byref(out)))
    shapes = [(tuple(a.shape), a.ndim == 1) for a in order]
    nqkv = shape.q_dim + 2 * shape.kv_dim
    shapes += [((nqkv,), True)] * shape.n_layers        # the bias vectors [bq | bk | bv] (sapo_trainer_read)
    tr = Trainer(out.value, cfg, shape, shapes)
    tr.n_in = len(order)
    for l, lw in enumerate(weights["layers"]):
        if "bq" in lw:
            sapo_trainer_set_qkv_bias(tr, l, _to_device(lw["bq"]), _to_device(lw["bk"]), _to_device(lw["bv"]), stream)
    torch.cuda.synchronize()          # the originals in `dev` may be freed after this
    return tr


def sapo_trainer_set_qkv_bias(tr: Trainer, layer: int, bq, bk, bv, stream=None):
    """bq float32 [Hq*hd], bk / bv float32 [Hkv*hd] device tensors."""
    torch = _torch()
    for t in (bq, bk, bv):
        assert t.dtype == torch.float32 and t.is_cuda and t.is_contiguous()
    _check(load_library().sapo_trainer_set_qkv_bias(tr.handle, layer, bq.data_ptr(), bk.data_ptr(), bv.data_ptr(),
                                                    _stream_ptr(stream)))
    tr.has_bias = True
    torch.cuda.synchronize()


def sapo_trainer_get_qkv_bias(tr: Trainer, layer: int, stream=None):
    """(bq, bk, bv) float32 device tensors: the masters of one layer's projection biases."""
    torch = _torch()
    q, kv = tr.shape.q_dim, tr.shape.kv_dim
    bq = torch.empty((q,), dtype=torch.float32, device="cuda")
    bk = torch.empty((kv,), dtype=torch.float32, device="cuda")
    bv = torch.empty((kv,), dtype=torch.float32, device="cuda")
    _check(load_library().sapo_trainer_get_qkv_bias(tr.handle, layer, bq.data_ptr(), bk.data_ptr(), bv.data_ptr(),
                                                    _stream_ptr(stream)))
    return bq, bk, bv


def sapo_trainer_destroy(tr: Trainer):
    tr.close()


def sapo_trainer_set_matmul_pieces(tr: Trainer, pieces: int):
    """3: fp32-accurate matrix products (default); 1: bf16 operands."""
    _check(load_library().sapo_trainer_set_matmul_pieces(tr.handle, pieces))


def sapo_trainer_steps(tr: Trainer) -> int:
    return tr.steps


def sapo_trainer_workspace_bytes(tr: Trainer, S: int, T: int) -> int:
    return int(load_library().sapo_trainer_workspace_bytes(tr.handle, S, T))


def sapo_trainer_workspace_bytes_for(tr: Trainer, S: int, T: int, S_micro: int) -> int:
    return int(load_library().sapo_trainer_workspace_bytes_for(tr.handle, S, T, S_micro))


def sapo_policy_update(tr: Trainer, tokens, completion_mask, logp_old, advantages, eps_low: float = 0.2,
                       eps_high: float = 0.28, want_logp: bool = True, workspace=None, stream=None):
    """tokens int32 [S, T], completion_mask uint8 [S, T], logp_old float32 [S, T], advantages float32 [S]
    (device).  Returns (loss before the step float32 [1], logp_new float32 [S, T] or None)."""
    torch = _torch()
    lib = load_library()
    S, T = int(tokens.shape[0]), int(tokens.shape[1])
    assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.is_contiguous()
    assert completion_mask.dtype == torch.uint8 and completion_mask.is_cuda and completion_mask.is_contiguous()
    assert tuple(completion_mask.shape) == (S, T)
    assert logp_old.dtype == torch.float32 and logp_old.is_cuda and logp_old.is_contiguous() and tuple(logp_old.shape) == (S, T)
    assert advantages.dtype == torch.float32 and advantages.is_cuda and advantages.is_contiguous() and advantages.numel() == S
    nbytes = sapo_trainer_workspace_bytes(tr, S, T)
    if workspace is None:
        workspace = _workspace(nbytes)
    loss = torch.empty((1,), dtype=torch.float32, device="cuda")
    logp = torch.empty((S, T), dtype=torch.float32, device="cuda") if want_logp else None
    _check(lib.sapo_policy_update(tr.handle, tokens.data_ptr(), completion_mask.data_ptr(), logp_old.data_ptr(),
                                  advantages.data_ptr(), S, T, eps_low, eps_high, loss.data_ptr(),
                                  logp.data_ptr() if want_logp else None, *_ws_args(workspace),
                                  _stream_ptr(stream)))
    return loss, logp


def sapo_trainer_read(tr: Trainer, what: int, tensor: int, stream=None):
    """One tensor of the trainer's state as a float32 device tensor (what: 0 masters, 1 gradient, 2 / 3 moments)."""
    torch = _torch()
    shp = tr.tensor_shapes[tensor][0]
    out = torch.empty(shp, dtype=torch.float32, device="cuda")
    _check(load_library().sapo_trainer_read(tr.handle, what, tensor, out.data_ptr(), out.numel(), _stream_ptr(stream)))
    return out


def sapo_trainer_export(tr: Trainer, stream=None) -> dict:
    """The masters in the model's storage type as a weights dict of numpy arrays (the layout of
    workloads.make_weights(): uint16 bf16 bit patterns for a bf16 model), ready for sapo_weights_create."""
    torch = _torch()
    bf16 = tr.cfg.dtype == SAPO_DTYPE_BF16
    dev = [torch.empty(shp, dtype=torch.float32 if (gain or not bf16) else torch.bfloat16, device="cuda")
           for shp, gain in tr.tensor_shapes[:tr.n_in]]
    ptrs = (C.c_void_p * len(dev))(*[t.data_ptr() for t in dev])
    _check(load_library().sapo_trainer_export(tr.handle, ptrs, len(dev), _stream_ptr(stream)))
    torch.cuda.synchronize()
    host = [(t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.cpu().numpy()) for t in dev]
    it = iter(host)
    w = {"embed": next(it), "layers": []}
    for _ in range(tr.cfg.n_layers):
        w["layers"].append({k: next(it) for k in LAYER_TENSORS})
    w["final_norm"] = next(it)
    w["lm_head"] = None if tr.cfg.tied_embeddings else next(it)
    if tr.has_bias:
        for l, lw in enumerate(w["layers"]):
            lw["bq"], lw["bk"], lw["bv"] = (t.cpu().numpy() for t in sapo_trainer_get_qkv_bias(tr, l, stream))
    return w


def sapo_trainer_export_weights(tr: Trainer, stream=None) -> Weights:
    """The trainer's masters as a new policy handle (sapo_trainer_export into device buffers, then
    sapo_weights_create and, for a model with projection biases, sapo_weights_set_qkv_bias), without a
    trip through host memory."""
    torch = _torch()
    lib = load_library()
    bf16 = tr.cfg.dtype == SAPO_DTYPE_BF16
    dev = [torch.empty(shp, dtype=torch.float32 if (gain or not bf16) else torch.bfloat16, device="cuda")
           for shp, gain in tr.tensor_shapes[:tr.n_in]]
    ptrs = (C.c_void_p * len(dev))(*[t.data_ptr() for t in dev])
    _check(lib.sapo_trainer_export(tr.handle, ptrs, len(dev), _stream_ptr(stream)))
    full = list(dev) + ([None] if tr.cfg.tied_embeddings else [])     # sapo_weights_create's list has a head slot
    wptrs = (C.c_void_p * len(full))(*[None if t is None else t.data_ptr() for t in full])
    out = C.c_void_p()
    _check(lib.sapo_weights_create(C.byref(tr.cfg), wptrs, len(full), _stream_ptr(stream), C.byref(out)))
    w = Weights(out.value, tr.cfg)
    if tr.has_bias:
        for l in range(tr.cfg.n_layers):
            bq, bk, bv = sapo_trainer_get_qkv_bias(tr, l, stream)
            sapo_weights_set_qkv_bias(w, l, bq, bk, bv, stream)
    torch.cuda.synchronize()          # `dev` may be freed after this
    return w


def sapo_trainer_export_into(tr: Trainer, w: Weights, buffers=None, stream=None):
    """The trainer's masters into an existing policy handle of the same configuration, in place
    (sapo_trainer_export into device buffers, then sapo_weights_update; biases through
    sapo_weights_set_qkv_bias).  `buffers`: the list this call returned earlier, to reuse its device tensors.
    Returns the buffers."""
    torch = _torch()
    lib = load_library()
    bf16 = tr.cfg.dtype == SAPO_DTYPE_BF16
    if buffers is None:
        buffers = [torch.empty(shp, dtype=torch.float32 if (gain or not bf16) else torch.bfloat16, device="cuda")
                   for shp, gain in tr.tensor_shapes[:tr.n_in]]
    ptrs = (C.c_void_p * len(buffers))(*[t.data_ptr() for t in buffers])
    _check(lib.sapo_trainer_export(tr.handle, ptrs, len(buffers), _stream_ptr(stream)))
    full = list(buffers) + ([None] if tr.cfg.tied_embeddings else [])
    wptrs = (C.c_void_p * len(full))(*[None if t is None else t.data_ptr() for t in full])
    _check(lib.sapo_weights_update(w.handle, wptrs, len(full), _stream_ptr(stream)))
    if tr.has_bias:
        for l in range(tr.cfg.n_layers):
            bq, bk, bv = sapo_trainer_get_qkv_bias(tr, l, stream)
            sapo_weights_set_qkv_bias(w, l, bq, bk, bv, stream)
    return buffers


def sapo_device_info() -> dict:
    out = (C.c_int32 * 4)()
    _check(load_library().sapo_device_info(out))
    return {"compute_units": out[0], "max_clock_MHz": out[1], "memory_clock_MHz": out[2], "memory_bus_bits": out[3]}


def sapo_debug_read_probe(nbytes: int = 1 << 31, repeats: int = 5) -> float:
    """Streaming read bandwidth in GB/s of a kernel that only reads: median of `repeats` timed launches over a
    buffer of `nbytes` (larger than the memory-side cache)."""
    torch = _torch()
    lib = load_library()
    buf = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ms = []
    for i in range(repeats + 1):
        ev[0].record()
        _check(lib.sapo_debug_read_probe(buf.data_ptr(), nbytes, sink.data_ptr(), _stream_ptr(None)))
        ev[1].record()
        torch.cuda.synchronize()
        if i > 0:
            ms.append(ev[0].elapsed_time(ev[1]))
    return nbytes / (float(np.median(ms)) * 1e-3) / 1e9


def sapo_debug_mfma_probe(std: float = 1.0, iters: int = 4096, repeats: int = 5, seed: int = 7) -> float:
    """TFLOP/s of a kernel that only issues half-precision MFMAs on registers (operands N(0, std^2)): median of
    `repeats` timed launches of 4096 workgroups."""
    torch = _torch()
    lib = load_library()
    ops = torch.from_numpy((np.random.default_rng(seed).standard_normal(6 * 64 * 8) * std).astype(np.float16)).cuda()
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    flops = C.c_double(0.0)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ms = []
    for i in range(repeats + 1):
        ev[0].record()
        _check(lib.sapo_debug_mfma_probe(ops.data_ptr(), 4096, iters, C.byref(flops), sink.data_ptr(), _stream_ptr(None)))
        ev[1].record()
        torch.cuda.synchronize()
        if i > 0:
            ms.append(ev[0].elapsed_time(ev[1]))
    return flops.value / (float(np.median(ms)) * 1e-3) / 1e12


def sapo_debug_logits(w: Weights, tokens, positions: Sequence[Sequence[int]], stream=None):
    """Teacher-forced logits after consuming tokens[s, 0..t] for each (s, t) in positions.
    Returns float32 [n, vocab] device tensor."""
    torch = _torch()
    lib = load_library()
    S, T = int(tokens.shape[0]), int(tokens.shape[1])
    pos = torch.tensor(np.asarray(positions, dtype=np.int32).reshape(-1, 2), dtype=torch.int32, device="cuda")
    n = int(pos.shape[0])
    assert int(pos[:, 0].min()) >= 0 and int(pos[:, 0].max()) < S and int(pos[:, 1].min()) >= 0 and int(pos[:, 1].max()) < T
    out = torch.empty((n, w.cfg.vocab), dtype=torch.float32, device="cuda")
    nbytes = int(lib.sapo_debug_logits_workspace_bytes(w.handle, S, T, n))
    ws = _workspace(nbytes)
    _check(lib.sapo_debug_logits(w.handle, tokens.data_ptr(), S, T, pos.data_ptr(), n, out.data_ptr(),
                                 _aligned_ptr(ws), nbytes, _stream_ptr(stream)))
    torch.cuda.synchronize()
    return out


def sapo_debug_half_clamped(w: Weights, tokens, stream=None) -> int:
    """Half-precision activation values at the clamp (+-65504) in a teacher-forced forward pass over tokens [S, T]."""
    lib = load_library()
    S, T = int(tokens.shape[0]), int(tokens.shape[1])
    nbytes = int(lib.sapo_debug_logits_workspace_bytes(w.handle, S, T, 1))
    ws = _workspace(nbytes)
    out = C.c_int64(0)
    _check(lib.sapo_debug_half_clamped(w.handle, tokens.data_ptr(), S, T, C.byref(out), _aligned_ptr(ws), nbytes,
                                       _stream_ptr(stream)))
    return int(out.value)


def sapo_weights_half_stats(w: Weights) -> dict:
    """{"half_path": the handle runs on the 16-bit matrix-core path, "below_normal_range": non-zero weight values
    under 2^-14 at the last create / update}."""
    out = (C.c_int64 * 2)()
    _check(load_library().sapo_weights_half_stats(w.handle, out))
    return {"half_path": bool(out[0]), "below_normal_range": int(out[1])}


def sapo_debug_gumbel(seed: int, seq: int, step: int, v0: int, n: int, stream=None):
    """The sampler's noise g for vocab entries v0 .. v0+n-1 of (seed, seq, step): float32 [n]."""
    torch = _torch()
    out = torch.empty((n,), dtype=torch.float32, device="cuda")
    _check(load_library().sapo_debug_gumbel(int(seed), seq, step, v0, n, out.data_ptr(), _stream_ptr(stream)))
    return out


def sapo_profile_start():
    """Start bracketing every kernel launch of the library with HIP events."""
    _check(load_library().sapo_profile_start())


def sapo_profile_stop() -> dict:
    """Stop and return {kernel symbol: (total_ms, launches)} for the kernels that ran."""
    lib = load_library()
    n = lib.sapo_profile_kernel_count()
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(lib.sapo_profile_stop(ms, cnt, n))
    return {lib.sapo_profile_kernel_name(i).decode(): (ms[i], int(cnt[i])) for i in range(n) if cnt[i] > 0}

