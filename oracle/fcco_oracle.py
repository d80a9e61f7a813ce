"""CPU oracle for one worker's FCCO global-contrastive-loss step (FastCLIP v0-v3).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP
library is checked against.  It may be imported by tests/, by
__graft_entry__.smoke() and by bench.py's cpu_baseline leg, and by nothing
else; it imports nothing from the GPU package and shares no code with it.

Everything is float64 numpy.  One call = Alg. 1 lines 6, 7 and 9 of the paper
plus the gradient half of line 12, for one worker k that owns the local rows
[off, off+b) of an already gathered global batch of B image/text embedding
pairs, with the encoders removed: "gradient" means the gradient with respect
to the local embedding rows themselves (the factor "nabla e" of Eqs. 2-7 is
the identity).

Notation (paper, Sec. 3 and Appendix A):
    s_ij           dot product of image row i and text row j
    l1(i, j, tau)  exp((s_ij - s_ii) / tau)           contrast: text j
    l2(i, j, tau)  exp((s_ji - s_ii) / tau)           contrast: image j
    g1_i, g2_i     mean of l1 / l2 over the batch without i   (Proc. 1)
    u1_i, u2_i     per-sample moving-average estimators       (Eq. 1)
    f(g)           log(eps + g)

Readings taken where the paper is silent (each one is listed in the design
notes of this repository):
  * the inner average runs over the GLOBAL batch without the anchor and is
    divided by M = B - 1 (Proc. 1, Eq. 1, Eqs. 2-3 all use B_{i-});
  * similarities are plain dot products of the rows as given (inputs are
    already L2-normalised by the caller); if the caller also hands over the
    norms that the local rows had before normalisation, the gradients are taken
    through the normalisation, with respect to the raw rows;
  * u^0 = 0 marks "never visited": a stored value that is exactly zero is
    replaced by g whatever gamma is;
  * the estimator uses u^{t+1} as a constant (no gradient through u) and the
    temperature(s) of the current call;
  * one worker's estimator is normalised by its local batch size b; only
    gradients of local rows are produced.  Without gathered state only the
    loss terms of the local anchors enter (Eq. 2 in full and the i-in-B_k part
    of Eq. 3).  With the gathered u^{t+1} of every global anchor (u_glob_*;
    Alg. 1 line 8) Eq. 3 / 5 / 7 enters in full: every global anchor i, local
    or not, has the local rows among its contrasts.  For individual
    temperatures the remote anchors' tau_1, tau_2 are gathered the same way
    (the paper's Eq. 7 uses tau_{1,i}, tau_{2,i} of the anchor i);
  * the scalar "loss" is the objective (GCL, RGCL, RGCL-g, or GCL without its
    leading tau for v0) with g(S_{i-}) replaced by u^{t+1} and the dataset
    average replaced by the local-batch average;
  * Eq. 9's factor 1/|S| is the argument tau_grad_scale.

Pins (tests/test_oracle_pins.py): gamma = 1 definition check against an
independent scalar evaluation, central finite differences of losses written
straight from GCL / RGCL / RGCL-g, reduction to softmax cross-entropy
(MBCL with eps = 1/M), hand-expanded B = 2 and B = 3 cases, invariants
(u > 0, untouched state, permutation, image/text swap, Euler identity),
the two-visit recurrence of Eq. 1, the closed-form values of the gamma
schedule, and for the gathered-state mode the agreement of the workers' shares
with the single-worker gradient of the same global batch plus finite
differences of the all-anchor frozen-u surrogate.  Nothing here is "parity
unpinned".
"""
from __future__ import annotations

import math

import numpy as np

V0, V1, V2, V3 = 0, 1, 2, 3


def gamma_cosine(t: int, iters_per_epoch: int, decay_epochs: int, gamma_min: float) -> float:
    """Inner learning rate of Sec. 4 "The Inner LR Schedule".

    epoch = floor(t / iters_per_epoch); gamma = 0.5 (1 + cos(pi epoch / E)) (1 - gamma_min)
    + gamma_min while epoch < E, and gamma_min from epoch E on.
    """
    epoch = t // iters_per_epoch
    if epoch >= decay_epochs:
        return float(gamma_min)
    return 0.5 * (1.0 + math.cos(math.pi * epoch / decay_epochs)) * (1.0 - gamma_min) + gamma_min


def check_indices(idx, n_state: int) -> bool:
    """True iff every index lies in [0, n_state) and no index repeats."""
    idx = np.asarray(idx, dtype=np.int64)
    if idx.size == 0:
        return True
    if idx.min() < 0 or idx.max() >= n_state:
        return False
    return np.unique(idx).size == idx.size


def ema_update(u_arr, idx, g, gamma):
    """Eq. 1 at positions idx of the state array u_arr (modified in place); returns the new values.

    A stored value of exactly zero means "never visited" and is replaced by g whatever gamma is.
    """
    idx = np.asarray(idx, dtype=np.int64)
    g = np.asarray(g, dtype=np.float64)
    old = np.asarray(u_arr[idx], dtype=np.float64)
    new = np.where(old == 0.0, g, (1.0 - gamma) * old + gamma * g)
    u_arr[idx] = new
    return new


def fcco_step(img, txt, off, b, idx, u_img, u_txt, *, version, gamma, eps, rho=0.0,
              tau=None, tau_img=None, tau_txt=None, tau_grad_scale=1.0,
              u_glob_img=None, u_glob_txt=None, tau_glob_img=None, tau_glob_txt=None,
              norm_img=None, norm_txt=None, contrast_side=True):
    """One FCCO step of worker k.  Updates u_img / u_txt IN PLACE at idx.

    img, txt   [B, d] global image / text embeddings (any float dtype; used as float64)
    off, b     local anchors are global rows off .. off+b-1
    idx        [b] dataset index of each local anchor (distinct)
    u_img/txt  [N] state arrays (numpy, modified in place)
    version    V0 (GCL without leading tau, learnable global tau; Eqs. 4, 5, 8)
               V1 (GCL, constant tau; Eqs. 2, 3)
               V2 (RGCL, per-sample tau_img/tau_txt [N]; Eqs. 6, 7, 9)
               V3 (RGCL-g, learnable global tau; Eqs. 2, 3, 10)
    u_glob_img/txt  optional [B]: u^{t+1} of every row of the global batch as gathered from
               all workers (Alg. 1 line 8); the entries of the local rows are ignored (this
               call's own new values are used).  When given, the contrast-side estimator of
               Eq. 3 / 5 / 7 runs over every global anchor instead of the local ones only.
    tau_glob_img/txt  [B], V2 with u_glob_* only: tau_1, tau_2 of every row of the global
               batch (entries of the local rows ignored).
    norm_img/txt  optional [b]: the rows of img / txt are the L2-normalised encoder outputs (cosine
               similarity, Sec. 3) and these are the norms the local rows had before; d_img / d_txt
               are then gradients with respect to the rows BEFORE normalisation.
    contrast_side  False leaves the estimator of Eq. 3 / 5 / 7 out (only Eq. 2 / 4 / 6 remains).  Not a mode
               of the method: tests use it to learn how large that term is in a given gradient.
    Returns a dict with g_img, g_txt, h_img, h_txt, u_new_img, u_new_txt, d_img,
    d_txt ([b, d]), loss, and d_tau (v0, v3) or d_tau_img, d_tau_txt ([b], v2).
    """
    img = np.asarray(img, dtype=np.float64)
    txt = np.asarray(txt, dtype=np.float64)
    idx = np.asarray(idx, dtype=np.int64)
    B, d = img.shape
    assert txt.shape == (B, d) and B >= 2 and 1 <= b and 0 <= off and off + b <= B
    assert idx.shape == (b,) and 0.0 < gamma <= 1.0 and eps >= 0.0
    M = B - 1                                    # |B_{i-}|
    rows = off + np.arange(b)                    # global row p of local anchor r
    I_loc, T_loc = img[rows], txt[rows]

    # temperatures entering l1 / l2 of each anchor (Proc. 1: global or individual)
    if version == V2:
        tau1 = np.asarray(tau_img, dtype=np.float64)[idx]
        tau2 = np.asarray(tau_txt, dtype=np.float64)[idx]
    else:
        tau1 = np.full(b, float(tau))
        tau2 = np.full(b, float(tau))

    # similarities: image anchors against every text, text anchors against every image
    S1 = I_loc @ txt.T                           # S1[r, j] = s_{p j}
    S2 = T_loc @ img.T                           # S2[r, j] = s_{j p}
    s_pp = np.einsum("rk,rk->r", I_loc, T_loc)   # s_ii of each anchor

    # Proc. 1: l1, l2 over the batch without the anchor itself, and their means
    X1 = S1 - s_pp[:, None]
    X2 = S2 - s_pp[:, None]
    E1 = np.exp(X1 / tau1[:, None])
    E2 = np.exp(X2 / tau2[:, None])
    E1[np.arange(b), rows] = 0.0                 # j = i is not in B_{i-}
    E2[np.arange(b), rows] = 0.0
    g1 = E1.sum(axis=1) / M
    g2 = E2.sum(axis=1) / M
    # h = mean of (s - s_ii) * l, so that d g / d tau = -h / tau^2  (nabla_3 l of Eqs. 8-10)
    h1 = (X1 * E1).sum(axis=1) / M
    h2 = (X2 * E2).sum(axis=1) / M

    # Eq. 1: moving average at the batch positions, everything else untouched
    u1 = ema_update(u_img, idx, g1, gamma)
    u2 = ema_update(u_txt, idx, g2, gamma)

    # outer derivative f'(u) = 1/(eps+u), times the 1/|B_k| and 1/|B_{i-}| of Eqs. 2-7,
    # times the leading factor (tau, 1, or tau_i) and the 1/tau that d l / d s brings
    if version == V0:
        c1 = 1.0 / (tau1 * b * M * (eps + u1))
        c2 = 1.0 / (tau2 * b * M * (eps + u2))
    else:                                        # leading tau (or tau_i) cancels the 1/tau
        c1 = 1.0 / (b * M * (eps + u1))
        c2 = 1.0 / (b * M * (eps + u2))

    # Eq. 2 / 4 / 6: anchor side.  d l1(i,j)/d e_{1,i} = l1 (e_{2,j} - e_{2,i}) / tau,
    # d l2(i,j)/d e_{1,i} = -l2 e_{2,i} / tau, and the mirror images for e_{2,i}.
    d_img = c1[:, None] * (E1 @ txt - (M * g1)[:, None] * T_loc) - (c2 * M * g2)[:, None] * T_loc
    d_txt = c2[:, None] * (E2 @ img - (M * g2)[:, None] * I_loc) - (c1 * M * g1)[:, None] * I_loc
    if not contrast_side:
        pass
    elif u_glob_img is None and u_glob_txt is None:
        # Eq. 3 / 5 / 7 restricted to local anchors i: local row p is a contrast of the
        # other local anchors r'.  l2(r', p) = exp((s_{p p'} - s_{p'p'}) / tau2_{r'}) moves image
        # row p, l1(r', p) = exp((s_{p'p} - s_{p'p'}) / tau1_{r'}) moves text row p.
        L2 = np.exp((S1[:, rows] - s_pp[None, :]) / tau2[None, :]) * c2[None, :]
        L1 = np.exp((S2[:, rows] - s_pp[None, :]) / tau1[None, :]) * c1[None, :]
        np.fill_diagonal(L2, 0.0)
        np.fill_diagonal(L1, 0.0)
        d_img += L2 @ T_loc
        d_txt += L1 @ I_loc
    else:
        # Eq. 3 / 5 / 7 in full.  Anchor i runs over the whole global batch; its coefficient is
        # kappa_i / (|B_k| |B_{i-}| (eps + u_i^{t+1})) with the u^{t+1} gathered from its worker
        # (this call's own values for the local rows).  l2(i, p) = exp((s_{p i} - s_ii) / tau2_i)
        # moves image row p towards/away from text row i; l1(i, p) = exp((s_{i p} - s_ii) / tau1_i)
        # moves text row p along image row i.  The anchor itself is not among its contrasts.
        s_all = np.einsum("ik,ik->i", img, txt)
        u1_all = np.array(u_glob_img, dtype=np.float64)
        u2_all = np.array(u_glob_txt, dtype=np.float64)
        assert u1_all.shape == (B,) and u2_all.shape == (B,)
        u1_all[rows], u2_all[rows] = u1, u2
        if version == V2:
            t1_all = np.array(tau_glob_img, dtype=np.float64)
            t2_all = np.array(tau_glob_txt, dtype=np.float64)
            assert t1_all.shape == (B,) and t2_all.shape == (B,)
            t1_all[rows], t2_all[rows] = tau1, tau2
        else:
            t1_all = np.full(B, float(tau))
            t2_all = np.full(B, float(tau))
        c1_all = 1.0 / (b * M * (eps + u1_all))
        c2_all = 1.0 / (b * M * (eps + u2_all))
        if version == V0:
            c1_all, c2_all = c1_all / t1_all, c2_all / t2_all
        for r in range(b):
            p = rows[r]
            w2 = c2_all * np.exp((S1[r] - s_all) / t2_all)       # over anchors i: S1[r, i] = s_{p i}
            w1 = c1_all * np.exp((S2[r] - s_all) / t1_all)       # S2[r, i] = s_{i p}
            w2[p] = 0.0
            w1[p] = 0.0
            d_img[r] += w2 @ txt
            d_txt[r] += w1 @ img

    if norm_img is not None or norm_txt is not None:
        # e^ = e / |e|:  d e^ / d e = (Id - e^ e^T) / |e|, applied to the gradient with respect to e^
        n1 = np.asarray(norm_img, dtype=np.float64)
        n2 = np.asarray(norm_txt, dtype=np.float64)
        assert n1.shape == (b,) and n2.shape == (b,)
        d_img = (d_img - I_loc * np.einsum("rk,rk->r", I_loc, d_img)[:, None]) / n1[:, None]
        d_txt = (d_txt - T_loc * np.einsum("rk,rk->r", T_loc, d_txt)[:, None]) / n2[:, None]

    out = dict(g_img=g1, g_txt=g2, h_img=h1, h_txt=h2, u_new_img=u1, u_new_txt=u2,
               d_img=d_img, d_txt=d_txt)
    log1, log2 = np.log(eps + u1), np.log(eps + u2)
    # loss_abs / d_tau_abs: the same sums with every term replaced by its absolute value.  They are no
    # outputs of the method but the scale against which an error of the scalar is judged: the scalars are
    # sums of terms of both signs (logarithms of values around 1, tau log against 2 rho tau) and can
    # cancel to nearly nothing, and then an error relative to the scalar itself says nothing about the
    # arithmetic that produced it.
    mean_abs_log = np.mean(np.abs(log1) + np.abs(log2))
    mean_abs_h = np.mean(np.abs(h1) / (eps + u1) + np.abs(h2) / (eps + u2))
    if version == V1:
        out["loss"] = float(tau) * np.mean(log1 + log2)
        out["loss_abs"] = abs(float(tau)) * mean_abs_log
    elif version == V0:                          # Eq. 8
        out["loss"] = np.mean(log1 + log2)
        out["loss_abs"] = mean_abs_log
        out["d_tau"] = -np.mean(h1 / (eps + u1) + h2 / (eps + u2)) / float(tau) ** 2
        out["d_tau_abs"] = mean_abs_h / float(tau) ** 2
    elif version == V3:                          # Eq. 10
        out["loss"] = float(tau) * np.mean(log1 + log2) + 2.0 * rho * float(tau)
        out["loss_abs"] = abs(float(tau)) * mean_abs_log + abs(2.0 * rho * float(tau))
        out["d_tau"] = (np.mean(log1 + log2) + 2.0 * rho
                        - np.mean(h1 / (eps + u1) + h2 / (eps + u2)) / float(tau))
        out["d_tau_abs"] = mean_abs_log + abs(2.0 * rho) + mean_abs_h / abs(float(tau))
    elif version == V2:                          # Eq. 9
        out["loss"] = np.mean(tau1 * (log1 + rho) + tau2 * (log2 + rho))
        out["loss_abs"] = np.mean(np.abs(tau1) * (np.abs(log1) + abs(rho)) + np.abs(tau2) * (np.abs(log2) + abs(rho)))
        out["d_tau_img"] = tau_grad_scale * (log1 + rho - h1 / (tau1 * (eps + u1)))
        out["d_tau_txt"] = tau_grad_scale * (log2 + rho - h2 / (tau2 * (eps + u2)))
    else:
        raise ValueError("unknown version")
    return out


def normalize_rows(raw):
    """Cosine similarity of Sec. 3 at the boundary: the unit rows e / |e| that fcco_step takes, and the norms |e|.

    raw: [b, d] encoder outputs (any float dtype; used as float64), no row all zero.
    Returns (unit [b, d], norm [b]) in float64.
    """
    raw = np.asarray(raw, dtype=np.float64)
    norm = np.sqrt(np.einsum("rk,rk->r", raw, raw))
    return raw / norm[:, None], norm


# ----------------------------------------------------------------------------------------------
# Temperature update (Alg. 1 line 12, Proc. "temperature_update" with Proc. "parameter_update")
SGDM, LAMB, LION, ADAMW = 1, 2, 3, 4


def parameter_update(theta, grad, m, v, *, optimizer, lr, step, beta1, beta2, eps=1e-8, weight_decay=0.0):
    """One step of Proc. "parameter_update" on an array (or scalar) theta with gradient estimator grad.

    m, v are the optimizer states before the step (v is ignored by SGD with momentum and Lion);
    `step` is t + 1, the 1-based count that the bias corrections of AdamW / LAMB use.  For SGD with
    momentum beta1 plays the role of the momentum parameter mu.  LAMB is taken with the layer factor
    alpha = 1, which the paper prescribes for the temperature and which makes it AdamW.
    Returns (theta_new, m_new, v_new) as float64 arrays.
    """
    theta = np.asarray(theta, dtype=np.float64)
    grad = np.asarray(grad, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    if optimizer == SGDM:
        m_new = beta1 * m + grad + weight_decay * theta
        return theta - lr * m_new, m_new, v
    if optimizer == LION:
        c = beta1 * m + (1.0 - beta1) * grad
        m_new = beta2 * m + (1.0 - beta2) * grad
        return theta - lr * (np.sign(c) + weight_decay * theta), m_new, v
    if optimizer in (ADAMW, LAMB):
        m_new = beta1 * m + (1.0 - beta1) * grad
        v_new = beta2 * v + (1.0 - beta2) * grad * grad
        m_hat = m_new / (1.0 - beta1 ** step)
        v_hat = v_new / (1.0 - beta2 ** step)
        r = m_hat / (np.sqrt(v_hat) + eps)
        return theta - lr * (r + weight_decay * theta), m_new, v_new
    raise ValueError("unknown optimizer")


def temperature_update(version, grads, *, optimizer, lr, step, beta1, beta2, eps=1e-8, tau_min=0.0,
                       lr_drop_below=0.0, lr_drop_factor=1.0, tau=None, m=None, v=None,
                       tau_img=None, tau_txt=None, idx=None, m_img=None, v_img=None, m_txt=None, v_txt=None):
    """Proc. "temperature_update" for one worker, weight decay 0.

    V1: nothing changes.  V0 / V3: the scalar tau is stepped with grads["d_tau"] (Eq. 8 / Eq. 10; with
    several workers the caller averages it first) and returned as (tau_new, m_new, v_new).  V2: the
    entries idx of tau_img / tau_txt (and of their optimizer states, all length-N arrays) are stepped IN
    PLACE with grads["d_tau_img"], grads["d_tau_txt"] (Eq. 9); all other entries are untouched.
    Readings: the constraint tau >= tau_0 of GCL / RGCL / RGCL-g is kept by projecting after the step
    (max(tau, tau_min)); the rule "the learning rate of tau drops to a third once tau is below 0.03" is
    applied to the value of tau before the step (lr * lr_drop_factor when tau < lr_drop_below)."""
    kw = dict(optimizer=optimizer, step=step, beta1=beta1, beta2=beta2, eps=eps)
    if version == V1:
        return None
    if version in (V0, V3):
        lr_now = lr * lr_drop_factor if float(tau) < lr_drop_below else lr
        t_new, m_new, v_new = parameter_update(tau, grads["d_tau"], m, v, lr=lr_now, **kw)
        return float(max(t_new, tau_min)), float(m_new), float(v_new)
    idx = np.asarray(idx, dtype=np.int64)
    for t_arr, m_arr, v_arr, g in ((tau_img, m_img, v_img, grads["d_tau_img"]),
                                   (tau_txt, m_txt, v_txt, grads["d_tau_txt"])):
        old = np.asarray(t_arr[idx], dtype=np.float64)
        lr_now = np.where(old < lr_drop_below, lr * lr_drop_factor, lr)
        t_new, m_new, v_new = parameter_update(old, g, m_arr[idx], v_arr[idx], lr=lr_now, **kw)
        t_arr[idx] = np.maximum(t_new, tau_min)
        m_arr[idx] = m_new
        v_arr[idx] = v_new
    return None
