"""ctypes binding of libmorlax.so: the same entry points as include/morlax.h.

Argument marshalling only.  Tensors are torch CUDA tensors used as device memory (data_ptr) and the
current torch stream is passed as the hipStream_t; every computation runs in the library's kernels.
Loading fails loudly when the library has not been built (`python -m paper_2603_09237_amd.build`).
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmorlax.so")

ACTOR, CRITIC = 0, 1
OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4, -5


class Dims(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("K", "P", "N", "T", "obs_dim", "act_dim", "n_hidden", "width",
                                         "act", "rank", "hyper_width", "wdtype", "mean_tanh", "sigma_state")]


class Rows(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("t0", "t_cnt", "j0", "j_cnt")]


class MorlaxError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"morlax error {code}: {msg}")
        self.code = code


_lib = None

EXPORTS = ("morlax_create", "morlax_destroy", "morlax_last_error", "morlax_hparam_count",
           "morlax_theta_mat_len", "morlax_theta_vec_len", "morlax_saved_bytes", "morlax_workspace_bytes",
           "morlax_env_pref_index", "morlax_hypernet_fwd", "morlax_hypernet_bwd", "morlax_hypernet_bwd_kept",
           "morlax_policy_fwd",
           "morlax_policy_bwd", "morlax_vec_gae", "morlax_vec_gae_trunc", "morlax_adam_step",
           "morlax_sample_preferences", "morlax_scalarize_normalized", "morlax_ppo_loss_grad",
           "morlax_ppo_loss_grad_static", "morlax_eval_returns",
           "morlax_hypervolume_workspace_bytes", "morlax_pareto_hypervolume", "morlax_profile_begin",
           "morlax_profile_end")

GEMM_KINDS = ("fwd_first", "fwd_hidden", "dx_hidden", "dw_hidden", "dw_first", "fwd_fused")


def load():
    """dlopen the library (once) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_09237_amd.build` "
                          "(there is no CPU fallback)")
    # torch provides the device memory and the streams, so the library must bind to the HIP runtime
    # torch has loaded (two runtimes in one process do not share devices): import torch first.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    lib.morlax_create.argtypes = [C.POINTER(Dims), C.POINTER(vp)]
    lib.morlax_create.restype = C.c_int
    lib.morlax_destroy.argtypes = [vp]
    lib.morlax_destroy.restype = None
    lib.morlax_last_error.argtypes = []
    lib.morlax_last_error.restype = C.c_char_p
    for name in ("morlax_hparam_count", "morlax_theta_mat_len", "morlax_theta_vec_len"):
        getattr(lib, name).argtypes = [vp, C.c_int]
        getattr(lib, name).restype = i64
    lib.morlax_saved_bytes.argtypes = [vp, C.c_int, C.POINTER(Rows)]
    lib.morlax_saved_bytes.restype = i64
    lib.morlax_workspace_bytes.argtypes = [vp, C.POINTER(Rows)]
    lib.morlax_workspace_bytes.restype = i64
    lib.morlax_env_pref_index.argtypes = [vp, vp, vp]
    lib.morlax_hypernet_fwd.argtypes = [vp, C.c_int, vp, vp, vp, vp, vp, i64, vp]
    lib.morlax_hypernet_bwd.argtypes = [vp, C.c_int, vp, vp, vp, vp, vp, vp, i64, vp]
    lib.morlax_hypernet_bwd_kept.argtypes = [vp, C.c_int, vp, vp, vp, vp, vp, vp, i64, vp]
    lib.morlax_policy_fwd.argtypes = [vp, C.c_int, vp, vp, vp, C.POINTER(Rows), vp, vp, vp, vp, vp, vp, i64, vp]
    lib.morlax_policy_bwd.argtypes = [vp, C.c_int, vp, vp, vp, C.POINTER(Rows), vp, vp, vp, vp, vp, vp, i64, vp]
    lib.morlax_vec_gae.argtypes = [vp, vp, vp, vp, vp, f32, f32, vp, vp, vp, vp]
    lib.morlax_vec_gae_trunc.argtypes = [vp, vp, vp, vp, vp, vp, f32, f32, vp, vp, vp, vp]
    lib.morlax_adam_step.argtypes = [vp, C.c_int, vp, vp, vp, vp, f32, f32, f32, f32, i32, vp]
    lib.morlax_sample_preferences.argtypes = [vp, vp, i32, vp, vp]
    lib.morlax_scalarize_normalized.argtypes = [vp, C.POINTER(Rows), vp, vp, vp, vp, i64, vp]
    lib.morlax_ppo_loss_grad.argtypes = [vp, C.POINTER(Rows), vp, vp, i32, vp, vp, vp, vp, vp, f32, i32,
                                         vp, vp, vp, vp, vp, i64, vp]
    lib.morlax_ppo_loss_grad_static.argtypes = [vp, C.POINTER(Rows), vp, vp, i32, vp, vp, vp, vp, vp, f32, i32,
                                                vp, vp, vp, vp, vp]
    lib.morlax_ppo_loss_grad_static.restype = C.c_int
    lib.morlax_eval_returns.argtypes = [vp, vp, vp, f32, vp, vp]
    lib.morlax_eval_returns.restype = C.c_int
    lib.morlax_hypervolume_workspace_bytes.argtypes = [i32, i32]
    lib.morlax_hypervolume_workspace_bytes.restype = i64
    lib.morlax_pareto_hypervolume.argtypes = [vp, vp, i32, i32, vp, vp, vp, i64, vp]
    lib.morlax_pareto_hypervolume.restype = C.c_int
    lib.morlax_profile_begin.argtypes = [vp]
    lib.morlax_profile_begin.restype = C.c_int
    lib.morlax_profile_end.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64), C.POINTER(C.c_double)]
    lib.morlax_profile_end.restype = C.c_int
    for name in ("morlax_env_pref_index", "morlax_hypernet_fwd", "morlax_hypernet_bwd", "morlax_hypernet_bwd_kept",
           "morlax_policy_fwd",
                 "morlax_policy_bwd", "morlax_vec_gae", "morlax_vec_gae_trunc", "morlax_adam_step",
                 "morlax_sample_preferences", "morlax_scalarize_normalized", "morlax_ppo_loss_grad"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, tuple):      # (address, bytes): a workspace given as a raw address
        return t[0]
    return t.data_ptr()


def _nbytes(t):
    """Size of a workspace: a tensor's own, or -- for a raw address -- whatever the caller vouches for."""
    if t is None:
        return 0
    if isinstance(t, int):
        return 1 << 62
    if isinstance(t, tuple):
        return int(t[1])
    return t.numel() * t.element_size()


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _rows(rows):
    if rows is None:
        return None
    if isinstance(rows, Rows):
        return C.byref(rows)
    return C.byref(Rows(*[int(v) for v in rows]))


class Context:
    """Owns a morlax_ctx.  Methods mirror the C entry points and raise MorlaxError on failure."""

    def __init__(self, **dims):
        self.lib = load()
        self.dims = Dims(**{k: int(v) for k, v in dims.items()})
        h = C.c_void_p()
        rc = self.lib.morlax_create(C.byref(self.dims), C.byref(h))
        if rc != OK:
            raise MorlaxError(rc, self.lib.morlax_last_error().decode())
        self.h = h

    @classmethod
    def from_config(cls, cfg):
        return cls(**cfg.dims_dict())

    def close(self):
        if getattr(self, "h", None):
            self.lib.morlax_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != OK:
            raise MorlaxError(rc, self.lib.morlax_last_error().decode())

    # ---- queries
    def hparam_count(self, net):
        return self.lib.morlax_hparam_count(self.h, net)

    def theta_mat_len(self, net):
        return self.lib.morlax_theta_mat_len(self.h, net)

    def theta_vec_len(self, net):
        return self.lib.morlax_theta_vec_len(self.h, net)

    def saved_bytes(self, net, rows=None):
        return self.lib.morlax_saved_bytes(self.h, net, _rows(rows))

    def workspace_bytes(self, rows=None):
        return self.lib.morlax_workspace_bytes(self.h, _rows(rows))

    def profile_begin(self):
        self._check(self.lib.morlax_profile_begin(self.h))

    def profile_end(self):
        """-> {kind: (total_ms, launches, total_flops)} for the grouped-GEMM launches since profile_begin."""
        n = len(GEMM_KINDS)
        ms, cnt, fl = (C.c_double * n)(), (C.c_int64 * n)(), (C.c_double * n)()
        self._check(self.lib.morlax_profile_end(self.h, ms, cnt, fl))
        return {k: (ms[i], cnt[i], fl[i]) for i, k in enumerate(GEMM_KINDS)}

    # ---- ops
    def env_pref_index(self, out, stream=None):
        self._check(self.lib.morlax_env_pref_index(self.h, _ptr(out), stream if stream is not None else _stream()))

    def hypernet_fwd(self, net, hparams, w, theta_mat, theta_vec, ws, stream=None):
        self._check(self.lib.morlax_hypernet_fwd(self.h, net, _ptr(hparams), _ptr(w), _ptr(theta_mat),
                                                 _ptr(theta_vec), _ptr(ws), _nbytes(ws),
                                                 stream if stream is not None else _stream()))

    def hypernet_bwd_kept(self, net, hparams, w, dtheta_mat, dtheta_vec, dhparams, ws_fwd, stream=None):
        self._check(self.lib.morlax_hypernet_bwd_kept(self.h, net, _ptr(hparams), _ptr(w), _ptr(dtheta_mat),
                                                      _ptr(dtheta_vec), _ptr(dhparams), _ptr(ws_fwd), _nbytes(ws_fwd),
                                                      stream if stream is not None else _stream()))

    def hypernet_bwd(self, net, hparams, w, dtheta_mat, dtheta_vec, dhparams, ws, stream=None):
        self._check(self.lib.morlax_hypernet_bwd(self.h, net, _ptr(hparams), _ptr(w), _ptr(dtheta_mat),
                                                 _ptr(dtheta_vec), _ptr(dhparams), _ptr(ws), _nbytes(ws),
                                                 stream if stream is not None else _stream()))

    def policy_fwd(self, net, theta_mat, theta_vec, x, rows, out, eps=None, act=None, logp=None, saved=None,
                   ws=None, stream=None):
        self._check(self.lib.morlax_policy_fwd(self.h, net, _ptr(theta_mat), _ptr(theta_vec), _ptr(x), _rows(rows),
                                               _ptr(out), _ptr(eps), _ptr(act), _ptr(logp), _ptr(saved), _ptr(ws),
                                               _nbytes(ws), stream if stream is not None else _stream()))

    def policy_bwd(self, net, theta_mat, theta_vec, x, rows, saved, dout, dlogsig, dtheta_mat, dtheta_vec, ws,
                   stream=None):
        self._check(self.lib.morlax_policy_bwd(self.h, net, _ptr(theta_mat), _ptr(theta_vec), _ptr(x), _rows(rows),
                                               _ptr(saved), _ptr(dout), _ptr(dlogsig), _ptr(dtheta_mat),
                                               _ptr(dtheta_vec), _ptr(ws), _nbytes(ws),
                                               stream if stream is not None else _stream()))

    def vec_gae(self, r, v, done, w, gamma, lam, adv_vec, vtarg, adv_s, stream=None):
        self._check(self.lib.morlax_vec_gae(self.h, _ptr(r), _ptr(v), _ptr(done), _ptr(w), float(gamma), float(lam),
                                            _ptr(adv_vec), _ptr(vtarg), _ptr(adv_s),
                                            stream if stream is not None else _stream()))

    def vec_gae_trunc(self, r, v, done, trunc, w, gamma, lam, adv_vec, vtarg, adv_s, stream=None):
        self._check(self.lib.morlax_vec_gae_trunc(self.h, _ptr(r), _ptr(v), _ptr(done), _ptr(trunc), _ptr(w),
                                                  float(gamma), float(lam), _ptr(adv_vec), _ptr(vtarg), _ptr(adv_s),
                                                  stream if stream is not None else _stream()))

    def sample_preferences(self, u, kappa, w, stream=None):
        self._check(self.lib.morlax_sample_preferences(self.h, _ptr(u), int(kappa), _ptr(w),
                                                       stream if stream is not None else _stream()))

    def eval_returns(self, r, done, gamma, J, stream=None):
        self._check(self.lib.morlax_eval_returns(self.h, _ptr(r), _ptr(done), float(gamma), _ptr(J),
                                                 stream if stream is not None else _stream()))

    def adam_step(self, net, hparams, dhparams, m, v, lr, beta1, beta2, eps, step, stream=None):
        self._check(self.lib.morlax_adam_step(self.h, net, _ptr(hparams), _ptr(dhparams), _ptr(m), _ptr(v),
                                              float(lr), float(beta1), float(beta2), float(eps), int(step),
                                              stream if stream is not None else _stream()))

    def scalarize_normalized(self, rows, adv_vec, w, adv_out, ws, stream=None):
        self._check(self.lib.morlax_scalarize_normalized(self.h, _rows(rows), _ptr(adv_vec), _ptr(w), _ptr(adv_out),
                                                         _ptr(ws), _nbytes(ws),
                                                         stream if stream is not None else _stream()))

    def ppo_loss_grad_static(self, rows, mu, logsig, logsig_stride, act, logp_old, adv_s, v, vtarg, clip_eps, norm_adv,
                             dmu, dlogsig, dv, stats, stream=None):
        """The loss call on the library's static scratch array (no workspace argument, nothing allocated)."""
        self._check(self.lib.morlax_ppo_loss_grad_static(self.h, _rows(rows), _ptr(mu), _ptr(logsig), int(logsig_stride),
                                                         _ptr(act), _ptr(logp_old), _ptr(adv_s), _ptr(v), _ptr(vtarg),
                                                         float(clip_eps), int(norm_adv), _ptr(dmu), _ptr(dlogsig),
                                                         _ptr(dv), _ptr(stats),
                                                         stream if stream is not None else _stream()))

    def ppo_loss_grad(self, rows, mu, logsig, logsig_stride, act, logp_old, adv_s, v, vtarg, clip_eps, norm_adv,
                      dmu, dlogsig, dv, stats, ws, stream=None):
        self._check(self.lib.morlax_ppo_loss_grad(self.h, _rows(rows), _ptr(mu), _ptr(logsig), int(logsig_stride),
                                                  _ptr(act), _ptr(logp_old), _ptr(adv_s), _ptr(v), _ptr(vtarg),
                                                  float(clip_eps), int(norm_adv), _ptr(dmu), _ptr(dlogsig),
                                                  _ptr(dv), _ptr(stats), _ptr(ws), _nbytes(ws),
                                                  stream if stream is not None else _stream()))


STATIC_SCRATCH_BYTES = 2 * 1024 * 1024


def hypervolume_workspace_bytes(n, K):
    """Bytes of device scratch morlax_pareto_hypervolume needs for n points in K objectives (-1: sizes not served)."""
    return int(load().morlax_hypervolume_workspace_bytes(int(n), int(K)))


def pareto_hypervolume(J, ref, n, K, front, hv, ws, stream=None):
    """morlax_pareto_hypervolume: needs no context; raises MorlaxError on failure."""
    lib = load()
    rc = lib.morlax_pareto_hypervolume(_ptr(J), _ptr(ref), int(n), int(K), _ptr(front), _ptr(hv), _ptr(ws),
                                       _nbytes(ws), stream if stream is not None else _stream())
    if rc != OK:
        raise MorlaxError(rc, lib.morlax_last_error().decode())
