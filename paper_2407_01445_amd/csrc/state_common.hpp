// The per-anchor arithmetic of the state phase, shared by the kernels that run it: k_state (fp32 path) and the fold
// kernels of the MFMA path, whose blocks on the diagonal finish the anchors of their rows.
#pragma once
#include "fc_internal.hpp"

namespace fc {

// Proc. "parameter_update" for one temperature with weight decay 0, then the projection onto tau >= tau_0.
// g: gradient estimator (Eqs. 8-10).  m, v: the optimizer's state (v only for AdamW / LAMB, pv may be NULL otherwise).
__device__ inline void tau_step(const TauUpd& u, float* ptau, float* pm, float* pv, float g) {
  const float tau = *ptau;
  float m = *pm;
  const float lr = tau < u.drop_below ? u.lr * u.drop_factor : u.lr;
  float next;
  if (u.optimizer == FASTCLIP_TAU_SGDM) {
    m = fmaf(u.beta1, m, g);
    next = tau - lr * m;
  } else if (u.optimizer == FASTCLIP_TAU_LION) {
    const float c = fmaf(u.beta1, m, (1.0f - u.beta1) * g);
    m = fmaf(u.beta2, m, (1.0f - u.beta2) * g);
    next = tau - lr * (c > 0.f ? 1.f : (c < 0.f ? -1.f : 0.f));
  } else {                                             // AdamW; LAMB with layer factor 1
    float v = *pv;
    m = fmaf(u.beta1, m, (1.0f - u.beta1) * g);
    v = fmaf(u.beta2, v, (1.0f - u.beta2) * g * g);
    *pv = v;
    next = tau - lr * ((m * u.corr1) / (sqrtf(v * u.corr2) + u.eps));
  }
  *pm = m;
  *ptau = fmaxf(next, u.tau_min);
}

// State phase.  Eq. 1 at the batch positions (first visit: stored 0 -> g), the coefficient
// 1/(|B_k| |B_i-| (eps+u)) of Eqs. 2-7 (with the extra 1/tau of Eqs. 4-5 for V0), Eq. 9 per anchor,
// and per-block partial sums of the two scalars that Eqs. 8 and 10 and the loss need.
struct StateArgs {
  const int64_t* idx;
  float *u_img, *u_txt;
  const float *tau1, *tau2;
  const float *uold1, *uold2;   // u^t at the batch positions, gathered by the prep kernel
  const float* sums;   // [4][nparts][bstride]
  int nparts;
  int fused;           // fold kernels: 1 = form the coefficients and finish the anchors there, 0 = k_state has run
  int64_t bstride, b;
  int64_t stride;      // elements between consecutive samples in u_img / u_txt (and the temperature arrays)
  float M, gamma, eps, rho, tau_scale;
  int version;
  float *c1, *c2, *dcoef;
  double* red;        // [blocks][2]: per-block sums of the anchors' loss terms and h terms
  float *d_tau_img, *d_tau_txt, *g_img, *g_txt, *u_new_img, *u_new_txt;
  // V2 with the temperature update in the same pass (optimizer != 0): the temperatures and their moments at idx
  TauUpd tau_upd;
  float *tau_img, *tau_txt, *m_img, *v_img, *m_txt, *v_txt;
};
StateArgs make_state_args(const StepCtx& c);

__device__ inline double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ inline float ema_update(float u_old, float g, float gamma) {
  return u_old == 0.0f ? g : fmaf(gamma, g, (1.0f - gamma) * u_old);
}

// One side of one anchor: the sum of its exponentials over the contrasts (M g), u^t and the temperature give
// u^{t+1} (Eq. 1) and the coefficient of Eqs. 2-7.  Every kernel that needs a coefficient forms it here.
__device__ inline float anchor_coefficient(const StateArgs& a, float sum_e, float u_old, float tau, float* u_new) {
  const float u = ema_update(u_old, sum_e * (1.0f / a.M), a.gamma);
  *u_new = u;
  float c = 1.0f / (((float)a.b * a.M) * (a.eps + u));
  if (a.version == FASTCLIP_V0) c /= tau;
  return c;
}

// Everything the state phase does for local anchor r once its four sums s = (sum e1, sum x1 e1, sum e2, sum x2 e2)
// are known: scatter of u^{t+1}, coefficients, Eq. 9 (and the temperature step if asked for), optional outputs.
// Returns the anchor's terms of the loss and of the h sums of Eqs. 8 / 10, as doubles: the scalars are sums of terms
// of both signs and are accumulated in fp64 on every path.  PRECISE (fp32-storage accuracy path): the logarithms, the
// h terms and Eq. 9 are evaluated in fp64 as well, so that the only fp32 roundings behind the scalars are those of the
// stored sums and of u^{t+1} itself; the MFMA path keeps them in fp32.
template <bool PRECISE>
__device__ inline void state_finish_anchor(const StateArgs& a, int64_t r, const float (&s)[4], float uo1, float uo2,
                                           float t1, float t2, float* c1_out, float* c2_out, double* lsum,
                                           double* hsum) {
  const float invM = 1.0f / a.M;
  const float g1 = s[0] * invM, g2 = s[2] * invM;
  const int64_t n = a.idx[r] * a.stride;
  float u1, u2;
  const float c1 = anchor_coefficient(a, s[0], uo1, t1, &u1);
  const float c2 = anchor_coefficient(a, s[2], uo2, t2, &u2);
  a.u_img[n] = u1;
  a.u_txt[n] = u2;
  a.c1[r] = c1;
  a.c2[r] = c2;
  a.dcoef[r] = c1 * s[0] + c2 * s[2];          // c1 M g1 + c2 M g2
  float gt1, gt2;
  if (PRECISE) {
    const double e1 = (double)a.eps + (double)u1, e2 = (double)a.eps + (double)u2;
    const double h1 = (double)s[1] / (double)a.M, h2 = (double)s[3] / (double)a.M;
    const double l1 = log(e1), l2 = log(e2);
    if (a.version == FASTCLIP_V2) {
      gt1 = (float)((double)a.tau_scale * (l1 + (double)a.rho - h1 / ((double)t1 * e1)));
      gt2 = (float)((double)a.tau_scale * (l2 + (double)a.rho - h2 / ((double)t2 * e2)));
      *lsum = (double)t1 * (l1 + (double)a.rho) + (double)t2 * (l2 + (double)a.rho);
    } else {
      *lsum = l1 + l2;
    }
    *hsum = h1 / e1 + h2 / e2;
  } else {
    const float e1 = a.eps + u1, e2 = a.eps + u2;
    const float h1 = s[1] * invM, h2 = s[3] * invM;
    const float l1 = logf(e1), l2 = logf(e2);
    if (a.version == FASTCLIP_V2) {
      gt1 = a.tau_scale * (l1 + a.rho - h1 / (t1 * e1));
      gt2 = a.tau_scale * (l2 + a.rho - h2 / (t2 * e2));
      *lsum = (double)(t1 * (l1 + a.rho)) + (double)(t2 * (l2 + a.rho));
    } else {
      *lsum = (double)l1 + (double)l2;
    }
    *hsum = (double)(h1 / e1) + (double)(h2 / e2);
  }
  if (a.version == FASTCLIP_V2) {
    a.d_tau_img[r] = gt1;
    a.d_tau_txt[r] = gt2;
    if (a.tau_upd.optimizer) {   // Proc. "temperature_update" for sample n, same gather/scatter as u
      tau_step(a.tau_upd, a.tau_img + n, a.m_img + n, a.v_img ? a.v_img + n : nullptr, gt1);
      tau_step(a.tau_upd, a.tau_txt + n, a.m_txt + n, a.v_txt ? a.v_txt + n : nullptr, gt2);
    }
  }
  if (a.g_img) a.g_img[r] = g1;
  if (a.g_txt) a.g_txt[r] = g2;
  if (a.u_new_img) a.u_new_img[r] = u1;
  if (a.u_new_txt) a.u_new_txt[r] = u2;
  *c1_out = c1;
  *c2_out = c2;
}

}  // namespace fc
