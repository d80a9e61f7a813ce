// The per-anchor arithmetic of the state phase, shared by the kernels that run it: k_state (both paths, and on its own
// behind fastclip_state_phase) and the fold kernels of the MFMA path, whose blocks on the diagonal finish the anchors of
// their rows when the batch is small.
#pragma once
#include "fc_internal.hpp"

namespace fc {

// Proc. "parameter_update" for one temperature with weight decay 0, then the projection onto tau >= tau_0.
// g: gradient estimator (Eqs. 8-10).  m, v: the optimizer's state (v only for AdamW / LAMB, untouched otherwise).
__device__ inline void tau_step_values(const TauUpd& u, float& tau, float& m, float& v, float g) {
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
    m = fmaf(u.beta1, m, (1.0f - u.beta1) * g);
    v = fmaf(u.beta2, v, (1.0f - u.beta2) * g * g);
    next = tau - lr * ((m * u.corr1) / (sqrtf(v * u.corr2) + u.eps));
  }
  tau = fmaxf(next, u.tau_min);
}
// The same on memory (pv may be NULL for SGDM / LION).
__device__ inline void tau_step(const TauUpd& u, float* ptau, float* pm, float* pv, float g) {
  const bool two = u.optimizer == FASTCLIP_TAU_ADAMW || u.optimizer == FASTCLIP_TAU_LAMB;
  float tau = *ptau, m = *pm, v = two ? *pv : 0.f;
  tau_step_values(u, tau, m, v, g);
  if (two) *pv = v;
  *pm = m;
  *ptau = tau;
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
  // k_state only.  gather: the kernel reads u^t and the temperatures from the state arrays itself (uold / tau1 / tau2
  // are not used; tau_glob is the global temperature of V0, V1, V3 for that case).  records: the per-sample arrays are
  // the fields {u_1, tau_1, m_1, v_1, u_2, tau_2, m_2, v_2} of 32-byte aligned records (state_records_are_canonical):
  // a lane moves its side's four fields as one 16-byte word.  lanes: threads per anchor side over the partial sums.
  int gather, records, lanes;
  int64_t ntiles;     // tiles of 128 / lanes anchors; a block takes the tiles blockIdx.x, blockIdx.x + gridDim.x, ..
  const float* tau_glob;
};
StateArgs make_state_args(const StepCtx& c);

__device__ inline double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Scalars (called by one whole wavefront): loss of the local batch with g replaced by u^{t+1}; Eq. 8 (V0), Eq. 10 (V3).
// red: the state phase's per-block sums of the anchors' loss terms and h terms.
// Written as values chosen per version and then ONE store per output through the pointer it was given: with a return
// per version, each ending in its own stores, the compiler merged the versions' last stores into one whose address
// register the V3 path never set (it held the flag output of a v_div_scale_f64), so that V3 stored d_tau to a stray
// address wherever this function was inlined behind other code.
__device__ inline void write_scalars(const double* red, int nblocks, int64_t b, int version, const float* tau, float rho,
                                     float* loss, float* d_tau) {
  const int lane = threadIdx.x & 63;
  double A = 0.0, H = 0.0;
  for (int i = lane; i < nblocks; i += 64) { A += red[2 * i]; H += red[2 * i + 1]; }
  A = wave_sum_f64(A) / (double)b;
  H = wave_sum_f64(H) / (double)b;
  const bool has_tau = version != FASTCLIP_V2;                         // V2 has no global temperature (tau may be NULL)
  const bool has_dtau = version == FASTCLIP_V0 || version == FASTCLIP_V3;
  const double t = has_tau ? (double)tau[0] : 1.0;
  const double r2 = 2.0 * (double)rho;
  double L = A, D = 0.0;                                               // V2: the temperatures are inside the anchors' terms
  if (version == FASTCLIP_V1) L = t * A;
  if (version == FASTCLIP_V0) D = -H / (t * t);
  if (version == FASTCLIP_V3) { L = t * A + r2 * t; D = A + r2 - H / t; }
  if (lane == 0) {
    loss[0] = (float)L;
    if (has_dtau) d_tau[0] = (float)D;
  }
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

// Everything the state phase computes for ONE SIDE (image or text) of one anchor from that side's two sums
// (sum_e = sum of l, sum_xe = sum of (s - s_ii) l over the contrasts), u^t and the temperature: u^{t+1} (Eq. 1), the
// coefficient, the side's term of Eq. 9 (V2), and its terms of the loss and of the h sums of Eqs. 8 / 10, as doubles
// (the scalars are sums of terms of both signs and are accumulated in fp64 on every path).  PRECISE (fp32-storage
// accuracy path): the logarithm, the h term and Eq. 9 are evaluated in fp64 as well, so that the only fp32 roundings
// behind the scalars are those of the stored sums and of u^{t+1} itself; the MFMA path keeps them in fp32.
struct SideResult {
  float u, c, ce;       // u^{t+1}, coefficient, coefficient x sum_e (the side's share of the diagonal factor)
  float gt;             // V2: the side's Eq. 9
  double lterm, hterm;
};
template <bool PRECISE>
__device__ inline SideResult state_side(const StateArgs& a, float sum_e, float sum_xe, float u_old, float tau) {
  SideResult o;
  o.c = anchor_coefficient(a, sum_e, u_old, tau, &o.u);
  o.ce = __fmul_rn(o.c, sum_e);
  o.gt = 0.f;
  if (PRECISE) {
    const double e = (double)a.eps + (double)o.u;
    const double h = (double)sum_xe / (double)a.M;
    const double l = log(e);
    if (a.version == FASTCLIP_V2) {
      o.gt = (float)((double)a.tau_scale * (l + (double)a.rho - h / ((double)tau * e)));
      o.lterm = (double)tau * (l + (double)a.rho);
    } else {
      o.lterm = l;
    }
    o.hterm = h / e;
  } else {
    const float e = a.eps + o.u;
    const float h = sum_xe * (1.0f / a.M);
    const float l = logf(e);
    if (a.version == FASTCLIP_V2) {
      o.gt = a.tau_scale * (l + a.rho - h / (tau * e));
      o.lterm = (double)(tau * (l + a.rho));
    } else {
      o.lterm = (double)l;
    }
    o.hterm = (double)(h / e);
  }
  return o;
}

// Both sides of local anchor r by one thread (the fold kernels' diagonal blocks): scatter of u^{t+1}, coefficients,
// Eq. 9 (and the temperature step if asked for), optional outputs.  s = (sum e1, sum x1 e1, sum e2, sum x2 e2).
template <bool PRECISE>
__device__ inline void state_finish_anchor(const StateArgs& a, int64_t r, const float (&s)[4], float uo1, float uo2,
                                           float t1, float t2, float* c1_out, float* c2_out, double* lsum,
                                           double* hsum) {
  const int64_t n = a.idx[r] * a.stride;
  const SideResult o1 = state_side<PRECISE>(a, s[0], s[1], uo1, t1);
  const SideResult o2 = state_side<PRECISE>(a, s[2], s[3], uo2, t2);
  a.u_img[n] = o1.u;
  a.u_txt[n] = o2.u;
  a.c1[r] = o1.c;
  a.c2[r] = o2.c;
  a.dcoef[r] = o1.ce + o2.ce;                  // c1 M g1 + c2 M g2
  if (a.version == FASTCLIP_V2) {
    a.d_tau_img[r] = o1.gt;
    a.d_tau_txt[r] = o2.gt;
    if (a.tau_upd.optimizer) {   // Proc. "temperature_update" for sample n, same gather/scatter as u
      tau_step(a.tau_upd, a.tau_img + n, a.m_img + n, a.v_img ? a.v_img + n : nullptr, o1.gt);
      tau_step(a.tau_upd, a.tau_txt + n, a.m_txt + n, a.v_txt ? a.v_txt + n : nullptr, o2.gt);
    }
  }
  const float invM = 1.0f / a.M;
  if (a.g_img) a.g_img[r] = s[0] * invM;
  if (a.g_txt) a.g_txt[r] = s[2] * invM;
  if (a.u_new_img) a.u_new_img[r] = o1.u;
  if (a.u_new_txt) a.u_new_txt[r] = o2.u;
  *lsum = o1.lterm + o2.lterm;
  *hsum = o1.hterm + o2.hterm;
  *c1_out = o1.c;
  *c2_out = o2.c;
}

}  // namespace fc
