"""FdaMonitor: owns the device buffers one FDA context needs (workspace, state, result
struct) as torch tensors and forwards to the C ABI.  No arithmetic happens here."""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import binding as B

_EST_OFFSETS = {"linear": B.FdaEstimate.sync_linear.offset, "sketch": B.FdaEstimate.sync_sketch.offset}


class FdaMonitor:
    def __init__(self, K, d, dtype, variants, l=0, m=0, eps=0.0, hash_coef=None,
                 row_stride=None, device="cuda:0", flags=0):
        if not torch.cuda.is_available():
            raise RuntimeError("FdaMonitor needs a HIP device (no CPU fallback exists)")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.K, self.d = int(K), int(d)
        self.dtype = {"f32": B.FDA_F32, "bf16": B.FDA_BF16}.get(dtype, dtype)
        self.variants = int(variants)
        self.desc, self._keep = B.make_desc(K, d, self.dtype, variants, l, m, eps, hash_coef, row_stride, flags)
        nbytes = B.fda_workspace_bytes(self.desc)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.ctx = B.fda_create(self.desc, self.workspace.data_ptr(), nbytes)
        self.S = B.fda_state_floats(self.ctx)
        self.plan = B.fda_get_plan(self.ctx).as_dict()
        self.state = torch.empty((self.K, self.S), dtype=torch.float32, device=self.device)
        self.mean = torch.empty((self.S,), dtype=torch.float32, device=self.device)
        self.est_dev = torch.zeros(C.sizeof(B.FdaEstimate), dtype=torch.uint8, device=self.device)

    def close(self):
        if getattr(self, "ctx", None):
            B.fda_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _stream():
        return torch.cuda.current_stream().cuda_stream

    def pred_ptr(self, which):
        """Device address of the sync decision of a variant inside the result struct."""
        return None if which is None else self.est_dev.data_ptr() + _EST_OFFSETS[which]

    def local_state(self, w, w_t0, xi=None):
        B.fda_local_state(self.ctx, w.data_ptr(), w_t0.data_ptr(),
                          None if xi is None else xi.data_ptr(), self.state.data_ptr(), self._stream())
        return self.state

    def estimate_variance(self, theta, tie_tol=1e-5, want_host=True, state=None):
        st = self.state if state is None else state
        return B.fda_estimate_variance(self.ctx, st.data_ptr(), float(theta), float(tie_tol),
                                       self.est_dev.data_ptr(), want_host, self._stream())

    def mean_state(self, w, w_t0, xi=None, w_bar=None):
        B.fda_mean_state(self.ctx, w.data_ptr(), w_t0.data_ptr(),
                         None if xi is None else xi.data_ptr(), self.mean.data_ptr(),
                         None if w_bar is None else w_bar.data_ptr(), self._stream())
        return self.mean

    def sync_from_mean(self, w, w_t0, w_bar, w_prev=None, xi=None, pred=None):
        B.fda_sync_from_mean(self.ctx, w.data_ptr(), w_t0.data_ptr(),
                             None if w_prev is None else w_prev.data_ptr(),
                             None if xi is None else xi.data_ptr(), w_bar.data_ptr(),
                             self.pred_ptr(pred), self._stream())

    def estimate_variance_mean(self, theta, tie_tol=1e-5, want_host=True, mean_state=None):
        st = self.mean if mean_state is None else mean_state
        return B.fda_estimate_variance_mean(self.ctx, st.data_ptr(), float(theta), float(tie_tol),
                                            self.est_dev.data_ptr(), want_host, self._stream())

    def sync(self, w, w_t0, w_prev=None, pred=None):
        B.fda_sync(self.ctx, w.data_ptr(), w_t0.data_ptr(),
                   None if w_prev is None else w_prev.data_ptr(), self.pred_ptr(pred), self._stream())

    def sync_xi(self, w, w_t0, w_prev, xi, pred=None):
        """sync followed by update_xi, with the norm taken inside the synchronization pass."""
        B.fda_sync_xi(self.ctx, w.data_ptr(), w_t0.data_ptr(), w_prev.data_ptr(), xi.data_ptr(),
                      self.pred_ptr(pred), self._stream())

    def update_xi(self, w_t0, w_prev, xi, pred=None):
        B.fda_update_xi(self.ctx, w_t0.data_ptr(), w_prev.data_ptr(), xi.data_ptr(),
                        self.pred_ptr(pred), self._stream())

    def step(self, w, w_t0, w_prev, xi, theta, decide_by="sketch", mean=False, w_bar=None,
             tie_tol=1e-5, want_host=False):
        """Algorithm 1 lines 6-9 in one call (fda_step)."""
        ptr = lambda t: None if t is None else t.data_ptr()
        by = B.FDA_VARIANT_SKETCH if decide_by == "sketch" else B.FDA_VARIANT_LINEAR
        st = self.mean if mean else self.state
        return B.fda_step(self.ctx, w.data_ptr(), w_t0.data_ptr(), ptr(w_prev), ptr(xi), st.data_ptr(),
                          ptr(w_bar), float(theta), float(tie_tol), by,
                          B.FDA_STEP_MEAN_STATE if mean else 0, self.est_dev.data_ptr(), want_host,
                          self._stream())

    def last_state_path(self):
        return B.fda_last_state_path(self.ctx, self._stream())

    def last_mean_state_path(self):
        return B.fda_last_mean_state_path(self.ctx, self._stream())

    def mean_numpy(self):
        """(n_bar, p_bar, sk(u_bar)[l,m] or None) as float32 host values."""
        s = self.mean.cpu().numpy()
        sk = None
        if self.variants & B.FDA_VARIANT_SKETCH:
            sk = s[2:].reshape(self.desc.l, self.desc.m).copy()
        return float(s[0]), float(s[1]), sk

    def state_numpy(self):
        """(n[K], p[K], sk[K,l,m] or None) as float32 host arrays."""
        s = self.state.cpu().numpy()
        sk = None
        if self.variants & B.FDA_VARIANT_SKETCH:
            sk = s[:, 2:].reshape(self.K, self.desc.l, self.desc.m)
        return s[:, 0].copy(), s[:, 1].copy(), sk
