"""ctypes binding of libflexdenoise.so: argument marshalling only.

Every function has the name and argument order of its C counterpart in
include/flexdenoise.h.  Device buffers are torch tensors (PyTorch supplies device
memory and streams, nothing else); a negative status raises FlexDenoiseError.
There is no fallback: if the native library is missing, importing this module
raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

from . import synth

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflexdenoise.so")

FC_F32, FC_BF16 = 0, 1
FC_ATTN_FACTORIZED_CROSS, FC_ATTN_FULL3D_CONCAT = 0, 1


class FlexDenoiseError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.fc_last_error().decode() if _lib is not None else ""
        super().__init__(f"{where}: {_lib.fc_status_string(status).decode()} ({status}): {msg}")


class fc_model_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("frames", "height", "width", "channels", "patch", "hidden", "heads",
                                         "mlp_dim", "depth", "text_len", "text_dim", "t_embed_dim",
                                         "attn_mode", "dtype")] + [("ln_eps", C.c_float), ("text_adaln", C.c_int32)]


class fc_schedule(C.Structure):
    _fields_ = [("train_steps", C.c_int32), ("beta_start", C.c_float), ("beta_end", C.c_float),
                ("num_steps", C.c_int32), ("guidance_scale", C.c_float), ("eta", C.c_float),
                ("sampler", C.c_int32), ("seed", C.c_uint64)]


EXPORTS = {
    "fc_model_create": [C.POINTER(fc_model_config), C.POINTER(C.c_void_p)],
    "fc_model_weight_count": [C.c_void_p, C.POINTER(C.c_size_t)],
    "fc_model_set_weights": [C.c_void_p, C.c_void_p, C.c_size_t],
    "fc_model_destroy": [C.c_void_p],
    "fc_workspace_bytes": [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)],
    "fc_denoise_step": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(fc_schedule), C.c_int32,
                        C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p],
    "fc_denoise_resume": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(fc_schedule), C.c_int32,
                          C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p],
    "fc_denoise_resume_ex": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(fc_schedule), C.c_int32,
                             C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_void_p), C.c_void_p, C.c_size_t,
                             C.c_void_p],
    "fc_schedule_coefficients": [C.POINTER(fc_schedule), C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_int32)],
    "fc_cache_stitch": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p],
    "fc_cache_decompress": [C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_void_p, C.c_int32,
                            C.POINTER(C.c_int32), C.c_int32, C.c_int64, C.c_void_p, C.c_void_p],
    "fc_cache_alpha": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_size_t,
                       C.c_void_p],
    "fc_cache_frame_similarity": [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p],
    "fc_cache_frame_similarity_noalloc": [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p],
    "fc_cache_select_key_frames": [C.POINTER(C.c_float), C.c_int32, C.c_float, C.POINTER(C.c_int32)],
    "fc_profile_enable": [C.c_void_p, C.c_int32],
    "fc_profile_select": [C.c_void_p, C.c_int32],
    "fc_profile_categories": [],
    "fc_profile_read": [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64)],
    "fc_op_linear": [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                     C.c_int32, C.c_int32, C.c_void_p],
    "fc_op_linear_scratch": [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                             C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p],
    "fc_op_attention": [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                        C.c_int32, C.c_int32, C.c_void_p],
    "fc_op_attention_bounded": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                C.c_int32, C.c_void_p, C.c_void_p],
    "fc_op_layernorm_modulate": [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                 C.c_int32, C.c_float, C.c_void_p],
    "fc_op_layernorm_residual2": [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_int32, C.c_void_p],
    "fc_op_patch_embed": [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                          C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                          C.c_int32, C.c_void_p],
    "fc_bench_pipe_rates": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p],
    "fc_op_cfg_ddim": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_float,
                       C.POINTER(C.c_float), C.c_void_p],
}
_STRING_EXPORTS = {"fc_status_string": [C.c_int], "fc_last_error": [], "fc_profile_category_name": [C.c_int32]}
_SIZE_EXPORTS = {"fc_cache_workspace_bytes": [C.c_int32]}


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2501_04012_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    for name, argtypes in EXPORTS.items():
        fn = getattr(lib, name)
        fn.argtypes, fn.restype = argtypes, C.c_int
    for name, argtypes in _STRING_EXPORTS.items():
        fn = getattr(lib, name)
        fn.argtypes, fn.restype = argtypes, C.c_char_p
    for name, argtypes in _SIZE_EXPORTS.items():
        fn = getattr(lib, name)
        fn.argtypes, fn.restype = argtypes, C.c_size_t
    return lib


_lib = None
_lib = _load()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise FlexDenoiseError(status, where)


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor / numpy array / None."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    return getattr(stream, "cuda_stream", stream) or None


def _cfg_struct(cfg: synth.ModelConfig) -> fc_model_config:
    return fc_model_config(cfg.frames, cfg.height, cfg.width, cfg.channels, cfg.patch, cfg.hidden, cfg.heads,
                           cfg.mlp_dim, cfg.depth, cfg.text_len, cfg.text_dim, cfg.t_embed_dim, cfg.attn_mode,
                           cfg.dtype, cfg.ln_eps, cfg.text_adaln)


def _sched_struct(s: synth.Schedule) -> fc_schedule:
    return fc_schedule(s.train_steps, s.beta_start, s.beta_end, s.num_steps, s.guidance_scale, s.eta, s.sampler, s.seed)


# ------------------------------------------------------------------ the C calls, one to one

def fc_model_create(cfg: synth.ModelConfig) -> int:
    h = C.c_void_p()
    st = _cfg_struct(cfg)
    _check(_lib.fc_model_create(C.byref(st), C.byref(h)), "fc_model_create")
    return h.value


def fc_model_weight_count(model: int) -> int:
    n = C.c_size_t()
    _check(_lib.fc_model_weight_count(model, C.byref(n)), "fc_model_weight_count")
    return n.value


def fc_model_set_weights(model: int, host_blob: np.ndarray) -> None:
    blob = np.ascontiguousarray(host_blob, dtype=np.float32)
    _check(_lib.fc_model_set_weights(model, blob.ctypes.data, blob.size), "fc_model_set_weights")


def fc_model_destroy(model: int) -> None:
    _check(_lib.fc_model_destroy(model), "fc_model_destroy")


def fc_workspace_bytes(model: int, batch_requests: int, use_cfg: bool) -> int:
    n = C.c_size_t()
    _check(_lib.fc_workspace_bytes(model, batch_requests, int(use_cfg), C.byref(n)), "fc_workspace_bytes")
    return n.value


def fc_denoise_step(model, latent, cond, null_cond, sched: synth.Schedule, step: int, batch_requests: int,
                    eps_out, workspace, stream=None) -> None:
    s = _sched_struct(sched)
    _check(_lib.fc_denoise_step(model, _ptr(latent), _ptr(cond), _ptr(null_cond), C.byref(s), step, batch_requests,
                                _ptr(eps_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                _stream(stream)), "fc_denoise_step")


def fc_denoise_resume(model, latent, cond, null_cond, sched: synth.Schedule, k: int, batch_requests: int,
                      workspace, stream=None) -> None:
    s = _sched_struct(sched)
    _check(_lib.fc_denoise_resume(model, _ptr(latent), _ptr(cond), _ptr(null_cond), C.byref(s), k, batch_requests,
                                  _ptr(workspace), workspace.numel() * workspace.element_size(),
                                  _stream(stream)), "fc_denoise_resume")


def fc_denoise_resume_ex(model, latent, cond, null_cond, sched: synth.Schedule, k: int, batch_requests: int,
                         export_steps, export_dst, workspace, stream=None) -> None:
    """export_steps: ascending step numbers; export_dst: device tensors of the latent's size."""
    s = _sched_struct(sched)
    n = len(export_steps)
    steps = (C.c_int32 * max(n, 1))(*[int(v) for v in export_steps])
    dsts = (C.c_void_p * max(n, 1))(*[_ptr(t) for t in export_dst])
    _check(_lib.fc_denoise_resume_ex(model, _ptr(latent), _ptr(cond), _ptr(null_cond), C.byref(s), k, batch_requests,
                                     n, steps, dsts, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream(stream)), "fc_denoise_resume_ex")


def fc_cache_stitch(x_obj, x_bg, m_obj, m_bg, out, pixels: int, channels: int, stream=None) -> None:
    _check(_lib.fc_cache_stitch(_ptr(x_obj), _ptr(x_bg), _ptr(m_obj), _ptr(m_bg), _ptr(out), pixels, channels,
                                _stream(stream)), "fc_cache_stitch")


def fc_cache_decompress(first, diff_base, n_base: int, alpha: float, extra, n_extra: int, src, frames: int,
                        frame_elems: int, out, stream=None) -> None:
    codes = (C.c_int32 * max(frames, 1))(*[int(v) for v in src])
    _check(_lib.fc_cache_decompress(_ptr(first), _ptr(diff_base), n_base, alpha, _ptr(extra), n_extra, codes, frames,
                                    frame_elems, _ptr(out), _stream(stream)), "fc_cache_decompress")


def fc_cache_workspace_bytes(frames: int) -> int:
    return int(_lib.fc_cache_workspace_bytes(frames))


def fc_cache_alpha(first_s, keys_s, diff_base, n_base: int, frame_elems: int, alpha_out, workspace,
                   stream=None) -> None:
    _check(_lib.fc_cache_alpha(_ptr(first_s), _ptr(keys_s), _ptr(diff_base), n_base, frame_elems, _ptr(alpha_out),
                               _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "fc_cache_alpha")


def fc_cache_frame_similarity(frames_dev, frames: int, frame_elems: int, sim, workspace, stream=None) -> None:
    _check(_lib.fc_cache_frame_similarity(_ptr(frames_dev), frames, frame_elems, _ptr(sim), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)),
           "fc_cache_frame_similarity")


def fc_cache_frame_similarity_noalloc(frames_dev, frames: int, frame_elems: int, sim, stream=None) -> None:
    _check(_lib.fc_cache_frame_similarity_noalloc(_ptr(frames_dev), frames, frame_elems, _ptr(sim), _stream(stream)),
           "fc_cache_frame_similarity_noalloc")


def fc_bench_pipe_rates(operands, iters: int, mode_first: int, mode_second: int, blocks: int, sink, clocks,
                        stream=None) -> None:
    _check(_lib.fc_bench_pipe_rates(_ptr(operands), iters, mode_first, mode_second, blocks, _ptr(sink), _ptr(clocks),
                                    _stream(stream)), "fc_bench_pipe_rates")


def fc_cache_select_key_frames(sim_host: np.ndarray, threshold: float = 0.99) -> np.ndarray:
    sim_host = np.ascontiguousarray(sim_host, dtype=np.float32)
    T = sim_host.shape[0]
    out = (C.c_int32 * max(T, 1))()
    _check(_lib.fc_cache_select_key_frames(sim_host.ctypes.data_as(C.POINTER(C.c_float)), T, threshold, out),
           "fc_cache_select_key_frames")
    return np.array(out[:T], dtype=np.int64)


def fc_schedule_coefficients(sched: synth.Schedule, step: int):
    s = _sched_struct(sched)
    out = (C.c_float * 4)()
    t = C.c_int32()
    _check(_lib.fc_schedule_coefficients(C.byref(s), step, out, C.byref(t)), "fc_schedule_coefficients")
    return np.array(list(out), dtype=np.float32), t.value


def fc_profile_enable(model: int, enable: bool) -> None:
    _check(_lib.fc_profile_enable(model, int(enable)), "fc_profile_enable")


def fc_profile_select(model: int, category) -> None:
    """Restrict the event brackets to one category (name or index); None or -1 = all."""
    if category is None:
        category = -1
    if isinstance(category, str):
        names = [fc_profile_category_name(i) for i in range(fc_profile_categories())]
        category = names.index(category)
    _check(_lib.fc_profile_select(model, int(category)), "fc_profile_select")


def fc_profile_categories() -> int:
    return _lib.fc_profile_categories()


def fc_profile_category_name(i: int) -> str:
    return _lib.fc_profile_category_name(i).decode()


def fc_profile_read(model: int):
    """{category: (milliseconds, brackets)} since the last read."""
    n = fc_profile_categories()
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(_lib.fc_profile_read(model, n, ms, cnt), "fc_profile_read")
    return {fc_profile_category_name(i): (ms[i], cnt[i]) for i in range(n)}


def fc_op_linear(dtype, A, Wt, bias, gate, out, M, N, K, epilogue, stream=None) -> None:
    _check(_lib.fc_op_linear(dtype, _ptr(A), _ptr(Wt), _ptr(bias), _ptr(gate), _ptr(out), M, N, K, epilogue,
                             _stream(stream)), "fc_op_linear")


def fc_op_linear_scratch(dtype, A, Wt, bias, gate, out, M, N, K, epilogue, scratch, stream=None) -> None:
    nbytes = 0 if scratch is None else scratch.numel() * scratch.element_size()
    _check(_lib.fc_op_linear_scratch(dtype, _ptr(A), _ptr(Wt), _ptr(bias), _ptr(gate), _ptr(out), M, N, K, epilogue,
                                     _ptr(scratch), nbytes, _stream(stream)), "fc_op_linear_scratch")


def fc_op_attention(dtype, q, k, v, out, G, nq, nk, d, impl=0, stream=None) -> None:
    _check(_lib.fc_op_attention(dtype, _ptr(q), _ptr(k), _ptr(v), _ptr(out), G, nq, nk, d, impl, _stream(stream)),
           "fc_op_attention")


def fc_op_attention_bounded(q, k, v, out, G, nq, nk, d, key_norm_scratch, stream=None) -> None:
    _check(_lib.fc_op_attention_bounded(_ptr(q), _ptr(k), _ptr(v), _ptr(out), G, nq, nk, d, _ptr(key_norm_scratch),
                                        _stream(stream)), "fc_op_attention_bounded")


def fc_op_layernorm_modulate(dtype, x, y, shift, scale, out, M, D, eps, stream=None) -> None:
    _check(_lib.fc_op_layernorm_modulate(dtype, _ptr(x), _ptr(y), _ptr(shift), _ptr(scale), _ptr(out), M, D, eps,
                                         _stream(stream)), "fc_op_layernorm_modulate")


def fc_op_layernorm_residual2(dtype, x, y, gate, y2, gate2, shift, scale, out, M, D, eps, write_x, stream=None) -> None:
    _check(_lib.fc_op_layernorm_residual2(dtype, _ptr(x), _ptr(y), _ptr(gate), _ptr(y2), _ptr(gate2), _ptr(shift),
                                          _ptr(scale), _ptr(out), M, D, eps, int(write_x), _stream(stream)),
           "fc_op_layernorm_residual2")


def fc_op_patch_embed(latent, R, B, Wp, bp, pos_sp, pos_t, x, T, H, W, Cc, p, D, rows_per_b, row_off, impl=0,
                      stream=None) -> None:
    _check(_lib.fc_op_patch_embed(_ptr(latent), R, B, _ptr(Wp), _ptr(bp), _ptr(pos_sp), _ptr(pos_t), _ptr(x), T, H, W,
                                  Cc, p, D, rows_per_b, row_off, impl, _stream(stream)), "fc_op_patch_embed")


def fc_op_cfg_ddim(x, eps_c, eps_u, eps_out, n_total, guidance_scale, coef4, stream=None) -> None:
    c = (C.c_float * 4)(*[float(v) for v in coef4])
    _check(_lib.fc_op_cfg_ddim(_ptr(x), _ptr(eps_c), _ptr(eps_u), _ptr(eps_out), n_total, guidance_scale, c,
                               _stream(stream)), "fc_op_cfg_ddim")


# ------------------------------------------------------------------ a thin convenience holder

class Denoiser:
    """Owns an fc_model and a torch workspace tensor for a fixed batch."""

    def __init__(self, cfg: synth.ModelConfig, weights, batch_requests: int, use_cfg: bool, device="cuda:0"):
        import torch
        self.cfg, self.R, self.use_cfg = cfg, batch_requests, use_cfg
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.model = fc_model_create(cfg)
        blob = weights if isinstance(weights, np.ndarray) else synth.pack_weights(cfg, weights)
        if blob.size != fc_model_weight_count(self.model):
            raise ValueError("weight blob size mismatch")
        fc_model_set_weights(self.model, blob)
        self.workspace = torch.empty(fc_workspace_bytes(self.model, batch_requests, use_cfg), dtype=torch.uint8,
                                     device=self.device)

    def step(self, latent, cond, null_cond, sched, step, eps_out=None, stream=None):
        fc_denoise_step(self.model, latent, cond, null_cond if self.use_cfg else None, sched, step, self.R,
                        eps_out, self.workspace, stream)

    def resume(self, latent, cond, null_cond, sched, k, stream=None):
        fc_denoise_resume(self.model, latent, cond, null_cond if self.use_cfg else None, sched, k, self.R,
                          self.workspace, stream)

    def resume_ex(self, latent, cond, null_cond, sched, k, export_steps, export_dst, stream=None):
        fc_denoise_resume_ex(self.model, latent, cond, null_cond if self.use_cfg else None, sched, k, self.R,
                             export_steps, export_dst, self.workspace, stream)

    def close(self):
        if self.model:
            fc_model_destroy(self.model)
            self.model = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
