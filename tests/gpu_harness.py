"""Plumbing for the GPU parity tests: upload seeded inputs, call the C ABI through the binding, download.

No arithmetic of the method happens here; comparisons use the error norms below.
"""
from __future__ import annotations

import numpy as np
import torch

from paper_2407_01445_amd import binding as fc

DEV = "cuda:0"
RECORD_FILL = 7.5      # what the unused fields of a state record hold
CANONICAL_FIELDS = dict(u_img=0, tau_img=1, m_img=2, v_img=3, u_txt=4, tau_txt=5, m_txt=6, v_txt=7)


def to_dev_matrix(x32: np.ndarray, dtype: str, ld: int | None = None) -> torch.Tensor:
    """float32 host matrix -> device matrix in the path's storage type, optionally with row stride ld > d."""
    t = torch.from_numpy(np.ascontiguousarray(x32))
    t = t.to(torch.bfloat16) if dtype == "bf16" else t.to(torch.float32)
    rows, d = t.shape
    if ld is None or ld == d:
        return t.to(DEV).contiguous()
    full = torch.full((rows, ld), float("nan"), dtype=t.dtype)      # padding must never be read
    full[:, :d] = t
    return full.to(DEV)


class GpuStep:
    """Device-resident state and buffers for repeated fastclip_step calls on one workload shape."""

    def __init__(self, *, B, b, off, d, N, dtype, version, eps, rho=0.0, tau=0.07, tau_grad_scale=1.0,
                 ld_img=None, ld_txt=None, u_img0=None, u_txt0=None, tau_img0=None, tau_txt0=None, gathered=None,
                 norms=None, state_stride=1, canonical_records=False, fine_tiles=False, single_pass=False, tiles=256):
        """tiles: 256 / 128 ask for that tile size on the bf16 path (FASTCLIP_TILES_256 / FASTCLIP_TILES_128), None leaves
        the choice to the library; the default keeps the tests of the large-tile kernels on them whatever the batch size.
        gathered: None, or dict(u_img=[B], u_txt=[B], tau_img=[B] or None, tau_txt=[B] or None) = the state
        gathered from all workers (the step then runs with FASTCLIP_GATHERED_STATE)."""
        self.B, self.b, self.off, self.d, self.N = B, b, off, d, N
        self.dtype, self.version = dtype, version
        self.eps, self.rho, self.scale = eps, rho, tau_grad_scale
        self.ld_img, self.ld_txt = ld_img or d, ld_txt or d
        f32 = dict(dtype=torch.float32, device=DEV)
        self.u_img = torch.zeros(N, **f32) if u_img0 is None else torch.from_numpy(np.asarray(u_img0, np.float32)).to(DEV)
        self.u_txt = torch.zeros(N, **f32) if u_txt0 is None else torch.from_numpy(np.asarray(u_txt0, np.float32)).to(DEV)
        self.tau = torch.full((1,), tau, **f32)
        self.tau_img = self.tau_txt = None
        if version == fc.V2:
            self.tau_img = torch.full((N,), tau, **f32) if tau_img0 is None else torch.from_numpy(np.asarray(tau_img0, np.float32)).to(DEV)
            self.tau_txt = torch.full((N,), tau, **f32) if tau_txt0 is None else torch.from_numpy(np.asarray(tau_txt0, np.float32)).to(DEV)
        self.state_stride = state_stride
        self.records = None
        # columns of the record that hold u_1, u_2, tau_1, tau_2; canonical_records: the order {u_1, tau_1, m_1, v_1,
        # u_2, tau_2, m_2, v_2} that the library moves as two 16-byte words (CANONICAL_FIELDS names all eight columns)
        cu1, cu2, ct1, ct2 = (0, 4, 1, 5) if canonical_records else (0, 1, 2, 3)
        if state_stride > 1:
            assert state_stride >= (8 if canonical_records else 4)
            self.records = torch.full((N, state_stride), RECORD_FILL, **f32)
            self.records[:, cu1], self.records[:, cu2] = self.u_img, self.u_txt
            self.u_img, self.u_txt = self.records[:, cu1], self.records[:, cu2]
            if version == fc.V2:
                self.records[:, ct1], self.records[:, ct2] = self.tau_img, self.tau_txt
                self.tau_img, self.tau_txt = self.records[:, ct1], self.records[:, ct2]
        nan = float("nan")
        self.d_img = torch.full((b, d), nan, **f32)
        self.d_txt = torch.full((b, d), nan, **f32)
        self.loss = torch.full((1,), nan, **f32)
        self.d_tau = torch.full((1,), nan, **f32)
        self.d_tau_img = torch.full((b,), nan, **f32)
        self.d_tau_txt = torch.full((b,), nan, **f32)
        self.g_img = torch.full((b,), nan, **f32)
        self.g_txt = torch.full((b,), nan, **f32)
        self.u_new_img = torch.full((b,), nan, **f32)
        self.u_new_txt = torch.full((b,), nan, **f32)
        self.cfg = None
        self.ws = None
        self.flags = (fc.FINE_TILES if fine_tiles else 0) | (fc.SINGLE_PASS if single_pass else 0)
        if dtype == "bf16" and not fine_tiles:
            self.flags |= {256: fc.TILES_256, 128: fc.TILES_128, None: 0}[tiles]
        self.u_glob_img = self.u_glob_txt = self.tau_glob_img = self.tau_glob_txt = None
        self.norm_img = self.norm_txt = None
        if norms is not None:       # (norm_img [b], norm_txt [b]): gradients through the L2 normalisation
            self.norm_img = torch.from_numpy(np.asarray(norms[0], np.float32)).to(DEV)
            self.norm_txt = torch.from_numpy(np.asarray(norms[1], np.float32)).to(DEV)
        if gathered is not None:
            self.flags |= fc.GATHERED_STATE
            up = lambda a: None if a is None else torch.from_numpy(np.asarray(a, np.float32)).to(DEV)
            self.u_glob_img, self.u_glob_txt = up(gathered["u_img"]), up(gathered["u_txt"])
            self.tau_glob_img, self.tau_glob_txt = up(gathered.get("tau_img")), up(gathered.get("tau_txt"))

    def config(self, gamma):
        return fc.make_config(version=self.version, emb_dtype=fc.BF16 if self.dtype == "bf16" else fc.F32,
                              B=self.B, b=self.b, off=self.off, d=self.d, N=self.N, gamma=gamma, eps=self.eps,
                              rho=self.rho, tau_grad_scale=self.scale, ld_img=self.ld_img, ld_txt=self.ld_txt,
                              flags=self.flags, state_stride=self.state_stride)

    def set_inputs(self, img32, txt32, idx):
        self.img = to_dev_matrix(img32, self.dtype, self.ld_img)
        self.txt = to_dev_matrix(txt32, self.dtype, self.ld_txt)
        self.idx = torch.from_numpy(np.asarray(idx, np.int64)).to(DEV)

    def buffers(self):
        return fc.make_buffers(img_glob=self.img, txt_glob=self.txt, idx=self.idx, u_img=self.u_img, u_txt=self.u_txt,
                               tau=self.tau, tau_img=self.tau_img, tau_txt=self.tau_txt, d_img=self.d_img,
                               d_txt=self.d_txt, loss=self.loss, d_tau=self.d_tau, d_tau_img=self.d_tau_img,
                               d_tau_txt=self.d_tau_txt, g_img=self.g_img, g_txt=self.g_txt,
                               u_new_img=self.u_new_img, u_new_txt=self.u_new_txt, u_glob_img=self.u_glob_img,
                               u_glob_txt=self.u_glob_txt, tau_glob_img=self.tau_glob_img,
                               tau_glob_txt=self.tau_glob_txt, norm_img=self.norm_img, norm_txt=self.norm_txt)

    def step(self, gamma, timed=False):
        cfg = self.config(gamma)
        need = fc.fastclip_workspace_bytes(cfg)
        assert need > 0
        if self.ws is None or self.ws.numel() < need:
            # poison the workspace so that any read of unwritten memory shows up as NaN
            self.ws = torch.full((need // 4 + 64,), float("nan"), dtype=torch.float32, device=DEV).view(torch.uint8)[:need]
        bufs = self.buffers()
        if timed:
            out = fc.fastclip_step_timed(cfg, bufs, self.ws)
        else:
            fc.fastclip_step(cfg, bufs, self.ws)
            out = None
        torch.cuda.synchronize()
        return out

    def step_update_tau(self, gamma, upd, state):
        """fastclip_step_update_tau with this object's buffers."""
        cfg = self.config(gamma)
        need = fc.fastclip_workspace_bytes(cfg)
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.full((need // 4 + 64,), float("nan"), dtype=torch.float32, device=DEV).view(torch.uint8)[:need]
        fc.fastclip_step_update_tau(cfg, self.buffers(), upd, state, self.ws)
        torch.cuda.synchronize()

    def outputs(self):
        o = {k: getattr(self, k).cpu().numpy().astype(np.float64) for k in
             ("d_img", "d_txt", "g_img", "g_txt", "u_new_img", "u_new_txt", "d_tau_img", "d_tau_txt")}
        o["loss"] = float(self.loss.item())
        o["d_tau"] = float(self.d_tau.item())
        return o


def rel_inf(x, ref):
    x, ref = np.asarray(x, np.float64), np.asarray(ref, np.float64)
    return float(np.max(np.abs(x - ref)) / max(np.max(np.abs(ref)), 1e-300))


def rel_l2(x, ref):
    x, ref = np.asarray(x, np.float64), np.asarray(ref, np.float64)
    return float(np.linalg.norm((x - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-300))


def rel_each(x, ref):
    x, ref = np.asarray(x, np.float64), np.asarray(ref, np.float64)
    return float(np.max(np.abs(x - ref) / np.abs(ref)))


def compare(got: dict, want: dict, version: int, tol: float, label: str = "", tol_measured: float | None = None):
    """u, g: per element relative (all > 0).  Gradients and per-sample tau gradients: max-norm and 2-norm
    relative.  The scalars (loss, d_tau) are sums of terms of both signs that can cancel to nearly nothing, so their
    error is taken relative to the same sum with every term replaced by its absolute value (the oracle's loss_abs /
    d_tau_abs): that is what the arithmetic can be held to whatever the draw; where nothing cancels it is the plain
    relative error.  Returns the worst error seen; asserts all <= tol, and all <= tol_measured if that is given
    (a guard at the level the path really reaches, next to the contractual tolerance)."""
    errs = {}
    errs["loss"] = abs(got["loss"] - want["loss"]) / want["loss_abs"]
    for k in ("g_img", "g_txt", "u_new_img", "u_new_txt"):
        errs[k] = rel_each(got[k], want[k])
    for k in ("d_img", "d_txt"):
        errs[k + "_inf"] = rel_inf(got[k], want[k])
        errs[k + "_l2"] = rel_l2(got[k], want[k])
    if version in (fc.V0, fc.V3):
        errs["d_tau"] = abs(got["d_tau"] - want["d_tau"]) / want["d_tau_abs"]
    if version == fc.V2:
        for k in ("d_tau_img", "d_tau_txt"):
            errs[k + "_inf"] = rel_inf(got[k], want[k])
    worst = max(errs.values())
    plain = abs(got["loss"] - want["loss"]) / max(abs(want["loss"]), 1e-300)
    print("[parity %s] tol %.1e worst %.3e :: %s (loss relative to itself %.2e)" % (label, tol, worst,
          " ".join("%s=%.2e" % kv for kv in sorted(errs.items())), plain), flush=True)
    bad = {k: v for k, v in errs.items() if not (v <= tol)}
    assert not bad, "parity failed %s: %s" % (label, bad)
    if tol_measured is not None:
        bad = {k: v for k, v in errs.items() if not (v <= tol_measured)}
        assert not bad, "parity worse than this path has measured %s: %s" % (label, bad)
    return worst
