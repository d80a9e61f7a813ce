// Small kernels of the FCCO step: s_ii and temperature gather, the state update of Eq. 1 with
// the per-anchor coefficients, the fp32-storage accuracy path (strips and gradients in
// plain loops with fp64 accumulation), the scalar outputs, and the index checker.
#include <string.h>

#include "fc_internal.hpp"
#include "state_common.hpp"

namespace fc {

constexpr float kLog2e = 1.4426950408889634f;

__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ inline float load_elem(const float* p) { return *p; }
__device__ inline float load_elem(const bf16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }

// ------------------------------------------------------------------------------------------
// prep: one wavefront per local anchor r.  s_pp = <img_p, txt_p> (the s_ii of Sec. 3), the
// temperatures that enter l1 / l2 of this anchor (Proc. 1: global tau, or tau_1[idx], tau_2[idx]),
// and k = log2(e) / tau for the exp2-based evaluation in the MFMA path.
__device__ inline double row_dot(const float* pi, const float* pt, int64_t d, int lane) {
  double acc = 0.0;
  for (int64_t k = lane; k < d; k += 64) acc += (double)pi[k] * (double)pt[k];
  return acc;
}
// bf16 rows: d and the row strides are multiples of 8 and the bases 16-byte aligned, so 8 elements per load
__device__ inline double row_dot(const bf16_t* pi, const bf16_t* pt, int64_t d, int lane) {
  double acc = 0.0;
  for (int64_t k = (int64_t)lane * 8; k < d; k += 512) {
    const uint4 a = *(const uint4*)(pi + k), b = *(const uint4*)(pt + k);
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
    float part = 0.f;   // 8 exact bf16 x bf16 products
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      part = fmaf(__uint_as_float(aw[w] << 16), __uint_as_float(bw[w] << 16), part);
      part = fmaf(__uint_as_float(aw[w] & 0xffff0000u), __uint_as_float(bw[w] & 0xffff0000u), part);
    }
    acc += (double)part;
  }
  return acc;
}

template <typename T>
__global__ void __launch_bounds__(256) k_prep(const T* __restrict__ img, const T* __restrict__ txt, int64_t ld_img,
                                              int64_t ld_txt, int64_t off, int64_t b, int64_t d,
                                              const int64_t* __restrict__ idx, const float* __restrict__ tau,
                                              const float* __restrict__ tau_img, const float* __restrict__ tau_txt,
                                              const float* __restrict__ u_img, const float* __restrict__ u_txt,
                                              int64_t stride, int version, float* __restrict__ diag,
                                              float* __restrict__ tau1,
                                              float* __restrict__ tau2, float* __restrict__ k1, float* __restrict__ k2,
                                              float* __restrict__ uold1, float* __restrict__ uold2) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= b) return;
  float t1 = 0.f, t2 = 0.f, u1 = 0.f, u2 = 0.f;
  if (lane == 0) {        // issue the gathers by dataset index before the dot product so that the latencies overlap:
    const int64_t n = idx[r] * stride;   // the temperatures, and u^t of Eq. 1 for the state phase (nothing writes u
    u1 = u_img[n];                       // before that phase)
    u2 = u_txt[n];
    if (version == FASTCLIP_V2) {
      t1 = tau_img[n];
      t2 = tau_txt[n];
    } else {
      t1 = t2 = tau[0];
    }
  }
  const double acc = wave_sum(row_dot(img + (off + r) * ld_img, txt + (off + r) * ld_txt, d, lane));
  if (lane == 0) {
    diag[r] = (float)acc;
    tau1[r] = t1;
    tau2[r] = t2;
    k1[r] = kLog2e / t1;
    k2[r] = kLog2e / t2;
    uold1[r] = u1;
    uold2[r] = u2;
  }
}

void launch_prep(const StepCtx& c) {
  const Layout& L = c.L;
  float* diag = (float*)(c.ws + L.diag);
  float* tau1 = (float*)(c.ws + L.tau1);
  float* tau2 = (float*)(c.ws + L.tau2);
  float* k1 = (float*)(c.ws + L.k1);
  float* k2 = (float*)(c.ws + L.k2);
  float* uold1 = (float*)(c.ws + L.uold1);
  float* uold2 = (float*)(c.ws + L.uold2);
  dim3 grid((unsigned)((L.b + 3) / 4)), block(256);
  if (L.bf16)
    hipLaunchKernelGGL(k_prep<bf16_t>, grid, block, 0, c.s, (const bf16_t*)c.buf.img_glob, (const bf16_t*)c.buf.txt_glob,
                       c.cfg.ld_img, c.cfg.ld_txt, L.off, L.b, L.d, c.buf.idx, c.buf.tau, c.buf.tau_img,
                       c.buf.tau_txt, c.buf.u_img, c.buf.u_txt, c.cfg.state_stride, c.cfg.version, diag, tau1, tau2, k1, k2,
                       uold1, uold2);
  else
    hipLaunchKernelGGL(k_prep<float>, grid, block, 0, c.s, (const float*)c.buf.img_glob, (const float*)c.buf.txt_glob,
                       c.cfg.ld_img, c.cfg.ld_txt, L.off, L.b, L.d, c.buf.idx, c.buf.tau, c.buf.tau_img,
                       c.buf.tau_txt, c.buf.u_img, c.buf.u_txt, c.cfg.state_stride, c.cfg.version, diag, tau1, tau2, k1, k2,
                       uold1, uold2);
}

// ------------------------------------------------------------------------------------------
// Cosine similarity at the boundary (Sec. 3): one wavefront per raw encoder row e: |e| with the squares summed in fp64,
// then e / |e| rounded once to the storage type of the step.  A row of zeros gives a row of zeros and norm 0.
__device__ inline void store_elem(float* p, float x) { *p = x; }
__device__ inline void store_elem(bf16_t* p, float x) { *p = __builtin_bit_cast(uint16_t, (__bf16)x); }

template <typename TI, typename TO>
__global__ void __launch_bounds__(256) k_normalize_rows(const TI* __restrict__ raw, int64_t ld_raw, int64_t b, int64_t d,
                                                        TO* __restrict__ unit, int64_t ld_unit, float* __restrict__ norm) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= b) return;
  const TI* src = raw + r * ld_raw;
  double acc = 0.0;
  for (int64_t k = lane; k < d; k += 64) {
    const double x = (double)load_elem(src + k);
    acc += x * x;
  }
  const double n = sqrt(wave_sum(acc));
  const float inv = n > 0.0 ? (float)(1.0 / n) : 0.f;
  TO* dst = unit + r * ld_unit;
  for (int64_t k = lane; k < d; k += 64) store_elem(dst + k, load_elem(src + k) * inv);
  if (lane == 0) norm[r] = (float)n;
}

void launch_normalize_rows(const void* raw, int raw_bf16, int64_t ld_raw, int64_t b, int64_t d, void* unit, int unit_bf16,
                           int64_t ld_unit, float* norm, hipStream_t s) {
  const dim3 grid((unsigned)((b + 3) / 4)), block(256);
  if (raw_bf16 && unit_bf16)
    hipLaunchKernelGGL((k_normalize_rows<bf16_t, bf16_t>), grid, block, 0, s, (const bf16_t*)raw, ld_raw, b, d, (bf16_t*)unit, ld_unit, norm);
  else if (raw_bf16)
    hipLaunchKernelGGL((k_normalize_rows<bf16_t, float>), grid, block, 0, s, (const bf16_t*)raw, ld_raw, b, d, (float*)unit, ld_unit, norm);
  else if (unit_bf16)
    hipLaunchKernelGGL((k_normalize_rows<float, bf16_t>), grid, block, 0, s, (const float*)raw, ld_raw, b, d, (bf16_t*)unit, ld_unit, norm);
  else
    hipLaunchKernelGGL((k_normalize_rows<float, float>), grid, block, 0, s, (const float*)raw, ld_raw, b, d, (float*)unit, ld_unit, norm);
}

// ------------------------------------------------------------------------------------------
// Gathered state (Alg. 1 line 8; Eqs. 3 / 5 / 7 over every global anchor): one wavefront per global row j.
// Anchor j contributes c_j l2(j, p) txt_j to the image gradient of a local row p and c_j l1(j, p) img_j to its text
// gradient, with l2(j, p) = exp((s_pj - s_jj) / tau2_j), l1(j, p) = exp((s_jp - s_jj) / tau1_j) and
// c_j = kappa_j / (|B_k| |B_j-| (eps + u_j^{t+1})): the strips already form s_pj and s_jp, so all they need per
// column j is log2(e)/tau_j, s_jj log2(e)/tau_j and c_j.  Local rows get c = 0 (their u^{t+1} is only known after
// the state phase; the fold after the state phase handles them), and so do the padding columns beyond B.
template <typename T>
__global__ void __launch_bounds__(256) k_prep_cols(const T* __restrict__ img, const T* __restrict__ txt, int64_t ld_img,
                                                   int64_t ld_txt, int64_t B, int64_t ncol, int64_t off, int64_t b,
                                                   int64_t d, const float* __restrict__ tau,
                                                   const float* __restrict__ tau_glob_img,
                                                   const float* __restrict__ tau_glob_txt,
                                                   const float* __restrict__ u_glob_img,
                                                   const float* __restrict__ u_glob_txt, int version, float eps,
                                                   float bm, float* __restrict__ colp) {
  const int lane = threadIdx.x & 63;
  const int64_t j = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= ncol) return;
  float k1 = 0.f, k2 = 0.f, d1 = 0.f, d2 = 0.f, c1 = 0.f, c2 = 0.f;
  const bool remote = j < B && (j < off || j >= off + b);
  if (remote) {                                  // wave-uniform
    float t1 = 0.f, t2 = 0.f, u1 = 0.f, u2 = 0.f;
    if (lane == 0) {
      if (version == FASTCLIP_V2) { t1 = tau_glob_img[j]; t2 = tau_glob_txt[j]; }
      else t1 = t2 = tau[0];
      u1 = u_glob_img[j];
      u2 = u_glob_txt[j];
    }
    const double s_jj = wave_sum(row_dot(img + j * ld_img, txt + j * ld_txt, d, lane));
    if (lane == 0) {
      k1 = kLog2e / t1;
      k2 = kLog2e / t2;
      d1 = (float)(s_jj * (double)k1);
      d2 = (float)(s_jj * (double)k2);
      c1 = 1.0f / (bm * (eps + u1));
      c2 = 1.0f / (bm * (eps + u2));
      if (version == FASTCLIP_V0) { c1 /= t1; c2 /= t2; }
    }
  }
  if (lane == 0) {
    const int64_t ntile = ncol >> 8, tile = j >> 8, in = j & 255;
    float* p0 = colp + ((0 * ntile + tile) * 4) * 256 + in;   // side 0: text anchors (tau_2, u_2)
    float* p1 = colp + ((1 * ntile + tile) * 4) * 256 + in;   // side 1: image anchors (tau_1, u_1)
    p0[0] = k2; p0[256] = d2; p0[512] = c2; p0[768] = 0.f;
    p1[0] = k1; p1[256] = d1; p1[512] = c1; p1[768] = 0.f;
  }
}

void launch_prep_cols(const StepCtx& c) {
  const Layout& L = c.L;
  float* colp = (float*)(c.ws + L.colp);
  const float bm = (float)L.b * (float)(L.B - 1);
  dim3 grid((unsigned)((L.ncol + 3) / 4)), block(256);
  if (L.bf16)
    hipLaunchKernelGGL(k_prep_cols<bf16_t>, grid, block, 0, c.s, (const bf16_t*)c.buf.img_glob,
                       (const bf16_t*)c.buf.txt_glob, c.cfg.ld_img, c.cfg.ld_txt, L.B, L.ncol, L.off, L.b, L.d,
                       c.buf.tau, c.buf.tau_glob_img, c.buf.tau_glob_txt, c.buf.u_glob_img, c.buf.u_glob_txt,
                       c.cfg.version, c.cfg.eps, bm, colp);
  else
    hipLaunchKernelGGL(k_prep_cols<float>, grid, block, 0, c.s, (const float*)c.buf.img_glob,
                       (const float*)c.buf.txt_glob, c.cfg.ld_img, c.cfg.ld_txt, L.B, L.ncol, L.off, L.b, L.d,
                       c.buf.tau, c.buf.tau_glob_img, c.buf.tau_glob_txt, c.buf.u_glob_img, c.buf.u_glob_txt,
                       c.cfg.version, c.cfg.eps, bm, colp);
}

// ------------------------------------------------------------------------------------------
// Accuracy path, strips (Proc. 1).  Block (r, side): anchor r against every contrast row j != p;
// side 0: image anchor vs texts (l1), side 1: text anchor vs images (l2).  One wavefront per
// contrast row, fp64 accumulation; stores l as fp32 and the two row sums.
__global__ void __launch_bounds__(256) k_strips_f32(const float* __restrict__ img, const float* __restrict__ txt,
                                                    int64_t ld_img, int64_t ld_txt, int64_t off, int64_t B,
                                                    int64_t d, const float* __restrict__ diag,
                                                    const float* __restrict__ tau1, const float* __restrict__ tau2,
                                                    float* __restrict__ E1, float* __restrict__ E2, int64_t ldE,
                                                    float* __restrict__ sums, int64_t bstride,
                                                    const float* __restrict__ colp, int64_t ncol,
                                                    float* __restrict__ F1, float* __restrict__ F2) {
  const int64_t r = blockIdx.x;
  const int side = blockIdx.y;
  const int64_t p = off + r;
  const float* anchor = side == 0 ? img + p * ld_img : txt + p * ld_txt;
  const float* X = side == 0 ? txt : img;
  const int64_t ldx = side == 0 ? ld_txt : ld_img;
  float* E = (side == 0 ? E1 : E2) + r * ldE;
  float* F = colp ? (side == 0 ? F1 : F2) + r * ldE : nullptr;   // gathered: c_j l(j, p) of every remote anchor j
  const double s_pp = (double)diag[r];
  const double tau = (double)(side == 0 ? tau1[r] : tau2[r]);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  double sg = 0.0, sh = 0.0;
  for (int64_t j = wave; j < B; j += 4) {
    const float* x = X + j * ldx;
    double acc = 0.0;
    for (int64_t k = lane; k < d; k += 64) acc += (double)anchor[k] * (double)x[k];
    acc = wave_sum(acc);
    const double xs = acc - s_pp;
    const double e = j == p ? 0.0 : exp(xs / tau);
    if (lane == 0) E[j] = (float)e;
    if (F && lane == 0) {
      const float* cp = colp + (((int64_t)side * (ncol >> 8) + (j >> 8)) * 4) * 256 + (j & 255);
      const double cj = (double)cp[512];
      F[j] = cj == 0.0 ? 0.f : (float)(cj * exp2(acc * (double)cp[0] - (double)cp[256]));
    }
    sg += e;
    sh += xs * e;
  }
  __shared__ double red[2][4];
  if (lane == 0) { red[0][wave] = sg; red[1][wave] = sh; }
  __syncthreads();
  if (threadIdx.x == 0) {
    // quantities 0,1 belong to side 0 (sum e1, sum x1 e1), 2,3 to side 1; nparts == 1 on this path
    sums[(size_t)(2 * side + 0) * bstride + r] = (float)(red[0][0] + red[0][1] + red[0][2] + red[0][3]);
    sums[(size_t)(2 * side + 1) * bstride + r] = (float)(red[1][0] + red[1][1] + red[1][2] + red[1][3]);
  }
}

void launch_strips_f32(const StepCtx& c) {
  const Layout& L = c.L;
  dim3 grid((unsigned)L.b, 2), block(256);
  hipLaunchKernelGGL(k_strips_f32, grid, block, 0, c.s, (const float*)c.buf.img_glob, (const float*)c.buf.txt_glob,
                     c.cfg.ld_img, c.cfg.ld_txt, L.off, L.B, L.d, (const float*)(c.ws + L.diag),
                     (const float*)(c.ws + L.tau1), (const float*)(c.ws + L.tau2), (float*)(c.ws + L.E[0]),
                     (float*)(c.ws + L.E[1]), L.ldE, (float*)(c.ws + L.sums), L.bstride,
                     L.gathered ? (const float*)(c.ws + L.colp) : nullptr, L.ncol,
                     L.gathered ? (float*)(c.ws + L.F[0]) : nullptr, L.gathered ? (float*)(c.ws + L.F[1]) : nullptr);
}


// Global temperature (V0, V3): one thread.
__global__ void k_tau_scalar(TauUpd u, float* tau, float* m, float* v, const float* d_tau) {
  if (threadIdx.x == 0 && blockIdx.x == 0) tau_step(u, tau, m, v, d_tau[0]);
}

// Individual temperatures (V2): one thread per local anchor, both sides; gathers and scatters by dataset index.
__global__ void __launch_bounds__(256) k_tau_sparse(TauUpd u, const int64_t* __restrict__ idx, int64_t b,
                                                    const float* __restrict__ g_img, const float* __restrict__ g_txt,
                                                    float* tau_img, float* tau_txt, float* m_img, float* v_img,
                                                    float* m_txt, float* v_txt) {
  const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (r >= b) return;
  const int64_t n = idx[r] * u.stride;
  tau_step(u, tau_img + n, m_img + n, v_img ? v_img + n : nullptr, g_img[r]);
  tau_step(u, tau_txt + n, m_txt + n, v_txt ? v_txt + n : nullptr, g_txt[r]);
}

void launch_tau_scalar(const TauUpd& u, const fastclip_tau_state& st, const float* d_tau, hipStream_t s) {
  hipLaunchKernelGGL(k_tau_scalar, dim3(1), dim3(64), 0, s, u, st.tau, st.m, st.v, d_tau);
}

void launch_tau_sparse(const TauUpd& u, const fastclip_tau_state& st, const int64_t* idx, int64_t b,
                       const float* d_tau_img, const float* d_tau_txt, hipStream_t s) {
  hipLaunchKernelGGL(k_tau_sparse, dim3((unsigned)((b + 255) / 256)), dim3(256), 0, s, u, idx, b, d_tau_img,
                     d_tau_txt, st.tau_img, st.tau_txt, st.m_img, st.v_img, st.m_txt, st.v_txt);
}

// ------------------------------------------------------------------------------------------
// State phase (Alg. 1 line 7 and the per-anchor half of lines 9 and 12): Eq. 1 at the batch's samples, the coefficients
// of Eqs. 2-7, Eq. 9, the partial sums of the loss and of Eqs. 8 / 10, and - if asked for - the temperature step of the
// same samples.  A thread owns ONE SIDE of one anchor (threads 2 r and 2 r + 1 are the image and the text side of
// anchor r), so the two words that a record layout keeps next to each other are moved by neighbouring lanes of one
// memory instruction.  256 threads = `lanes` partial-sum lanes x (256 / lanes) anchor sides; the threads of partial-sum
// lane 0 finish the anchor sides.  With canonical 8-float records a finishing thread moves its side's four fields
// {u, tau, m, v} as one 16-byte word: a sample costs one 32-byte sector each way, read and written whole.
// se / sx of partial-sum lane 0 plus those of lanes 1 .. LANES - 1, which sit 256 / LANES entries apart
template <int LANES>
__device__ __forceinline__ void add_parts(const float (*part)[256], int sa, float& se, float& sx) {
  float e[LANES], x[LANES];
#pragma unroll
  for (int q = 1; q < LANES; ++q) { e[q] = part[0][q * (256 / LANES) + sa]; x[q] = part[1][q * (256 / LANES) + sa]; }
#pragma unroll
  for (int q = 1; q < LANES; ++q) { se += e[q]; sx += x[q]; }
}

template <bool PRECISE>
__global__ void __launch_bounds__(256) k_state(StateArgs a) {
  __shared__ float part[2][256];
  __shared__ double scal[2][4];
  const int SA = 256 / a.lanes;                       // anchor sides per tile of a block
  const int sa = threadIdx.x % SA, pl = threadIdx.x / SA;
  const int side = sa & 1;
  double lterm = 0.0, hterm = 0.0;                    // this thread's terms of the two scalars, over all its tiles
  // a block takes the tiles blockIdx.x, blockIdx.x + gridDim.x, ..: the step launches one block per tile, the phase on
  // its own a bounded number of blocks (so that the scalars' partial sums stay few)
  for (int64_t tile = blockIdx.x; tile < a.ntiles; tile += gridDim.x) {
    const int64_t r = tile * (SA >> 1) + (sa >> 1);
    const bool finisher = pl == 0 && r < a.b;
    // the finishing threads' own inputs are requested first: the gather by dataset index is the longest latency here
    int64_t n = 0;
    float u_old = 0.f, tau = 0.f, m = 0.f, v = 0.f;
    if (finisher) {
      n = a.idx[r] * a.stride;
      if (a.records) {
        const float4 w = *(const float4*)(a.u_img + n + 4 * side);
        u_old = w.x; tau = w.y; m = w.z; v = w.w;
      } else if (a.gather) {
        u_old = (side ? a.u_txt : a.u_img)[n];
        tau = a.version == FASTCLIP_V2 ? (side ? a.tau_txt : a.tau_img)[n] : a.tau_glob[0];
      } else {
        u_old = (side ? a.uold2 : a.uold1)[r];
        tau = (side ? a.tau2 : a.tau1)[r];
      }
    }
    float se = 0.f, sx = 0.f;
    if (r < a.b) {
      const float* s0 = a.sums + (size_t)(2 * side) * a.nparts * a.bstride + r;
      const float* s1 = s0 + (size_t)a.nparts * a.bstride;
      // four partial sums of each quantity per round, so that eight loads are in flight instead of two
      int pt = pl;
      for (; pt + 3 * a.lanes < a.nparts; pt += 4 * a.lanes) {
        float e[4], x[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          e[q] = s0[(size_t)(pt + q * a.lanes) * a.bstride];
          x[q] = s1[(size_t)(pt + q * a.lanes) * a.bstride];
        }
        se += (e[0] + e[1]) + (e[2] + e[3]);
        sx += (x[0] + x[1]) + (x[2] + x[3]);
      }
      for (; pt < a.nparts; pt += a.lanes) {
        se += s0[(size_t)pt * a.bstride];
        sx += s1[(size_t)pt * a.bstride];
      }
    }
    if (a.lanes > 1) {                                   // block-uniform
      part[0][threadIdx.x] = se;
      part[1][threadIdx.x] = sx;
      __syncthreads();
      if (pl == 0) {      // all LDS reads of a thread issued together (compile-time trip counts), then added in order
        switch (a.lanes) {
          case 2: add_parts<2>(part, sa, se, sx); break;
          case 4: add_parts<4>(part, sa, se, sx); break;
          case 8: add_parts<8>(part, sa, se, sx); break;
          case 16: add_parts<16>(part, sa, se, sx); break;
          default: add_parts<32>(part, sa, se, sx); break;
        }
      }
      __syncthreads();                                   // before the next tile overwrites part
    }
    float ce = 0.f;
    if (finisher) {
      const SideResult o = state_side<PRECISE>(a, se, sx, u_old, tau);
      ce = o.ce;
      lterm += o.lterm;
      hterm += o.hterm;
      const bool step_tau = a.version == FASTCLIP_V2 && a.tau_upd.optimizer;
      if (a.records) {
        if (step_tau) {
          tau_step_values(a.tau_upd, tau, m, v, o.gt);
          *(float4*)(a.u_img + n + 4 * side) = make_float4(o.u, tau, m, v);
        } else {
          a.u_img[n + 4 * side] = o.u;
        }
      } else {
        (side ? a.u_txt : a.u_img)[n] = o.u;
        if (step_tau) {
          float* pv = side ? a.v_txt : a.v_img;
          tau_step(a.tau_upd, (side ? a.tau_txt : a.tau_img) + n, (side ? a.m_txt : a.m_img) + n, pv ? pv + n : nullptr,
                   o.gt);
        }
      }
      (side ? a.c2 : a.c1)[r] = o.c;
      if (a.version == FASTCLIP_V2) (side ? a.d_tau_txt : a.d_tau_img)[r] = o.gt;
      float* g_out = side ? a.g_txt : a.g_img;
      if (g_out) g_out[r] = se * (1.0f / a.M);
      float* u_out = side ? a.u_new_txt : a.u_new_img;
      if (u_out) u_out[r] = o.u;
    }
    const float ce_other = __shfl_xor(ce, 1);              // the two sides of an anchor are neighbouring lanes
    if (finisher && side == 0) a.dcoef[r] = ce + ce_other;  // c1 M g1 + c2 M g2
  }
  const double x = wave_sum_f64(lterm), y = wave_sum_f64(hterm);
  if ((threadIdx.x & 63) == 0) { scal[0][threadIdx.x >> 6] = x; scal[1][threadIdx.x >> 6] = y; }
  __syncthreads();
  if (threadIdx.x == 0) {
    a.red[2 * blockIdx.x + 0] = (scal[0][0] + scal[0][1]) + (scal[0][2] + scal[0][3]);
    a.red[2 * blockIdx.x + 1] = (scal[1][0] + scal[1][1]) + (scal[1][2] + scal[1][3]);
  }
}

// The per-sample arrays are the fields {u_1, tau_1, m_1, v_1, u_2, tau_2, m_2, v_2} of 32-byte aligned records.
bool state_records_are_canonical(const float* u_img, const float* u_txt, const fastclip_tau_state& t, int64_t stride) {
  return stride >= 8 && stride % 8 == 0 && ((uintptr_t)u_img & 31) == 0 && t.tau_img == u_img + 1 &&
         t.m_img == u_img + 2 && t.v_img == u_img + 3 && u_txt == u_img + 4 && t.tau_txt == u_img + 5 &&
         t.m_txt == u_img + 6 && t.v_txt == u_img + 7;
}

StateArgs make_state_args(const StepCtx& c) {
  const Layout& L = c.L;
  StateArgs a;
  a.idx = c.buf.idx; a.u_img = c.buf.u_img; a.u_txt = c.buf.u_txt;
  a.tau1 = (const float*)(c.ws + L.tau1); a.tau2 = (const float*)(c.ws + L.tau2);
  a.uold1 = (const float*)(c.ws + L.uold1); a.uold2 = (const float*)(c.ws + L.uold2);
  a.sums = (const float*)(c.ws + L.sums); a.nparts = L.nparts; a.bstride = L.bstride; a.b = L.b;
  a.fused = L.fused_state;
  a.stride = c.cfg.state_stride;
  a.M = (float)(L.B - 1); a.gamma = c.cfg.gamma; a.eps = c.cfg.eps; a.rho = c.cfg.rho;
  a.tau_scale = c.cfg.tau_grad_scale; a.version = c.cfg.version;
  a.c1 = (float*)(c.ws + L.c1); a.c2 = (float*)(c.ws + L.c2); a.dcoef = (float*)(c.ws + L.dcoef);
  a.red = (double*)(c.ws + L.red);
  a.d_tau_img = c.buf.d_tau_img; a.d_tau_txt = c.buf.d_tau_txt; a.g_img = c.buf.g_img; a.g_txt = c.buf.g_txt;
  a.u_new_img = c.buf.u_new_img; a.u_new_txt = c.buf.u_new_txt;
  a.tau_upd = c.tau_upd;
  if (c.cfg.version != FASTCLIP_V2) a.tau_upd.optimizer = 0;
  a.tau_img = c.tau_st.tau_img; a.tau_txt = c.tau_st.tau_txt;
  a.m_img = c.tau_st.m_img; a.v_img = c.tau_st.v_img; a.m_txt = c.tau_st.m_txt; a.v_txt = c.tau_st.v_txt;
  a.lanes = state_lanes(L.nparts);
  a.ntiles = L.nstate_blocks;
  a.tau_glob = c.buf.tau;
  // with the temperature update on canonical records the kernel takes u^t and the temperatures from the records
  // themselves (the same values that the prep kernel gathered): one 16-byte word per side holds all it needs
  a.records = a.tau_upd.optimizer && state_records_are_canonical(a.u_img, a.u_txt, c.tau_st, a.stride);
  a.gather = a.records;
  return a;
}

void launch_state(const StepCtx& c) {
  auto* kernel = c.L.bf16 ? k_state<false> : k_state<true>;
  hipLaunchKernelGGL(kernel, dim3((unsigned)c.L.nstate_blocks), dim3(256), 0, c.s, make_state_args(c));
}

// One wavefront: the scalars of a state phase that ran on its own.
__global__ void k_scalars(const double* red, int nblocks, int64_t b, int version, const float* tau, float rho,
                          float* loss, float* d_tau);

// The state phase on its own (fastclip_state_phase): n = cfg.b anchors whose four sums are given, everything else as
// in the step; the kernel gathers u^t and the temperatures itself.
void launch_state_phase(const fastclip_config& cfg, const fastclip_buffers& buf, const TauUpd& upd,
                        const fastclip_tau_state& tst, const float* sums, float* coef, double* red, int nblocks,
                        hipStream_t s) {
  StateArgs a;
  memset(&a, 0, sizeof(a));
  a.idx = buf.idx; a.u_img = buf.u_img; a.u_txt = buf.u_txt;
  a.sums = sums; a.nparts = 1; a.bstride = cfg.b; a.b = cfg.b;
  a.stride = cfg.state_stride;
  a.M = (float)(cfg.B - 1); a.gamma = cfg.gamma; a.eps = cfg.eps; a.rho = cfg.rho;
  a.tau_scale = cfg.tau_grad_scale; a.version = cfg.version;
  a.c1 = coef; a.c2 = coef + cfg.b; a.dcoef = coef + 2 * cfg.b;
  a.red = red;
  a.d_tau_img = buf.d_tau_img; a.d_tau_txt = buf.d_tau_txt; a.g_img = buf.g_img; a.g_txt = buf.g_txt;
  a.u_new_img = buf.u_new_img; a.u_new_txt = buf.u_new_txt;
  a.tau_upd = upd;
  if (cfg.version != FASTCLIP_V2) a.tau_upd.optimizer = 0;
  a.tau_img = a.tau_upd.optimizer ? tst.tau_img : const_cast<float*>(buf.tau_img);
  a.tau_txt = a.tau_upd.optimizer ? tst.tau_txt : const_cast<float*>(buf.tau_txt);
  a.m_img = tst.m_img; a.v_img = tst.v_img; a.m_txt = tst.m_txt; a.v_txt = tst.v_txt;
  a.lanes = 1;
  a.ntiles = (cfg.b + 127) / 128;
  a.tau_glob = buf.tau;
  a.gather = 1;
  a.records = cfg.version == FASTCLIP_V2 && a.tau_upd.optimizer &&
              state_records_are_canonical(a.u_img, a.u_txt, tst, a.stride);
  auto* kernel = cfg.emb_dtype == FASTCLIP_BF16 ? k_state<false> : k_state<true>;
  hipLaunchKernelGGL(kernel, dim3((unsigned)nblocks), dim3(256), 0, s, a);
  hipLaunchKernelGGL(k_scalars, dim3(1), dim3(64), 0, s, (const double*)red, nblocks, cfg.b, cfg.version, buf.tau,
                     cfg.rho, buf.loss, buf.d_tau);
}

// Eq. 1 alone, one thread per anchor (the same update as in k_state).
__global__ void __launch_bounds__(256) k_state_flat(const int64_t* __restrict__ idx, int64_t n, int64_t stride,
                                                    float gamma, float invM,
                                                    const float* __restrict__ s1, const float* __restrict__ s2,
                                                    float* __restrict__ u_img, float* __restrict__ u_txt,
                                                    float* __restrict__ o1, float* __restrict__ o2) {
  const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (r >= n) return;
  const int64_t i = idx[r] * stride;
  const float u1 = ema_update(u_img[i], s1[r] * invM, gamma);
  const float u2 = ema_update(u_txt[i], s2[r] * invM, gamma);
  u_img[i] = u1;
  u_txt[i] = u2;
  o1[r] = u1;
  o2[r] = u2;
}

void launch_state_flat(const int64_t* idx, int64_t n, int64_t stride, float gamma, float M, const float* sum_img,
                       const float* sum_txt, float* u_img, float* u_txt, float* u_new_img, float* u_new_txt,
                       hipStream_t s) {
  hipLaunchKernelGGL(k_state_flat, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, idx, n, stride, gamma, 1.0f / M, sum_img,
                     sum_txt, u_img, u_txt, u_new_img, u_new_txt);
}

__global__ void k_scalars(const double* red, int nblocks, int64_t b, int version, const float* tau, float rho,
                          float* loss, float* d_tau) {
  write_scalars(red, nblocks, b, version, tau, rho, loss, d_tau);
}

// ------------------------------------------------------------------------------------------
// Accuracy path, gradients (Eqs. 2-7 for the local rows).  Block (r, side) writes one output row:
//   side 0: d_img[r] = c1_r * sum_j l1(r,j) txt_j - (c1_r M g1_r + c2_r M g2_r) txt_p
//                      + sum_{r' != r} c2_{r'} l2(r', p) txt_{p'}
//   side 1: the mirror image.  The stored strips hold l with the anchor's own column zeroed.
__global__ void __launch_bounds__(256) k_grad_f32(const float* __restrict__ img, const float* __restrict__ txt,
                                                  int64_t ld_img, int64_t ld_txt, int64_t off, int64_t b, int64_t B,
                                                  int64_t d, const float* __restrict__ E1, const float* __restrict__ E2,
                                                  int64_t ldE, const float* __restrict__ c1, const float* __restrict__ c2,
                                                  const float* __restrict__ dcoef, float* __restrict__ d_img,
                                                  float* __restrict__ d_txt, const double* __restrict__ red, int nblocks,
                                                  int version, const float* __restrict__ tau, float rho,
                                                  float* __restrict__ loss, float* __restrict__ d_tau,
                                                  const float* __restrict__ F1, const float* __restrict__ F2,
                                                  const float* __restrict__ norm_img,
                                                  const float* __restrict__ norm_txt) {
  const int64_t r = blockIdx.x;
  const int side = blockIdx.y;
  const int64_t p = off + r;
  const float* Fown = F1 ? (side == 0 ? F1 : F2) + r * ldE : nullptr;   // gathered: remote anchors' weights
  const float* X = side == 0 ? txt : img;       // rows that the exp weights multiply
  const int64_t ldx = side == 0 ? ld_txt : ld_img;
  const float* Eown = (side == 0 ? E1 : E2) + r * ldE;       // l of this anchor over all contrasts
  const float* Eoth = side == 0 ? E2 : E1;                   // l of the other local anchors at column p
  const float* cown = side == 0 ? c1 : c2;
  const float* coth = side == 0 ? c2 : c1;
  float* out = (side == 0 ? d_img : d_txt) + r * d;
  int cw = 32;
  while (cw < 256 && cw < d) cw <<= 1;
  const int groups = 256 / cw;
  const int cl = threadIdx.x % cw, grp = threadIdx.x / cw;
  __shared__ double red2[256];
  for (int64_t c0 = 0; c0 < d; c0 += cw) {
    const int64_t col = c0 + cl;
    double acc = 0.0, acc6 = 0.0;
    if (col < d) {
      for (int64_t j = grp; j < B; j += groups) acc += (double)Eown[j] * (double)X[j * ldx + col];
      for (int64_t q = grp; q < b; q += groups)
        acc6 += (double)coth[q] * (double)Eoth[q * ldE + p] * (double)X[(off + q) * ldx + col];
      if (Fown)
        for (int64_t j = grp; j < B; j += groups) acc6 += (double)Fown[j] * (double)X[j * ldx + col];
    }
    red2[threadIdx.x] = (double)cown[r] * acc + acc6;
    __syncthreads();
    if (grp == 0 && col < d) {
      double t = 0.0;
      for (int g = 0; g < groups; ++g) t += red2[g * cw + cl];
      out[col] = (float)(t - (double)dcoef[r] * (double)X[p * ldx + col]);
    }
    __syncthreads();
  }
  if (norm_img) {
    // gradient through e^ = e / |e|: out := (out - e^ (e^ . out)) / |e|, e^ = this side's own row (see k_finalize_bf16)
    const float* ep = side == 0 ? img + p * ld_img : txt + p * ld_txt;
    double dot = 0.0;
    for (int64_t col = threadIdx.x; col < d; col += 256) dot += (double)out[col] * (double)ep[col];
    red2[threadIdx.x] = dot;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
      if ((int)threadIdx.x < w) red2[threadIdx.x] += red2[threadIdx.x + w];
      __syncthreads();
    }
    dot = red2[0];
    const double inv = 1.0 / (double)(side == 0 ? norm_img[r] : norm_txt[r]);
    for (int64_t col = threadIdx.x; col < d; col += 256)
      out[col] = (float)(((double)out[col] - dot * (double)ep[col]) * inv);
  }
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 64)
    write_scalars(red, nblocks, b, version, tau, rho, loss, d_tau);
}

void launch_grad_f32(const StepCtx& c) {
  const Layout& L = c.L;
  dim3 grid((unsigned)L.b, 2), block(256);
  hipLaunchKernelGGL(k_grad_f32, grid, block, 0, c.s, (const float*)c.buf.img_glob, (const float*)c.buf.txt_glob,
                     c.cfg.ld_img, c.cfg.ld_txt, L.off, L.b, L.B, L.d, (const float*)(c.ws + L.E[0]),
                     (const float*)(c.ws + L.E[1]), L.ldE, (const float*)(c.ws + L.c1), (const float*)(c.ws + L.c2),
                     (const float*)(c.ws + L.dcoef), c.buf.d_img, c.buf.d_txt, (const double*)(c.ws + L.red),
                     L.nstate_blocks, c.cfg.version, c.buf.tau, c.cfg.rho, c.buf.loss, c.buf.d_tau,
                     L.gathered ? (const float*)(c.ws + L.F[0]) : nullptr,
                     L.gathered ? (const float*)(c.ws + L.F[1]) : nullptr, c.buf.norm_img, c.buf.norm_txt);
}

// ------------------------------------------------------------------------------------------
// MFMA path, last phase.  d_img[r] = c1_r * (sum over splits of the contraction)[r] - dcoef_r txt_p, and the mirror
// image (the contraction already carries the contrast-side terms divided by c_r); block (0,0,0) also writes the
// scalars.  The split partials are whole 256 x 256 tiles of [64 groups of 4 rows][256 columns][4 rows] (the order in
// which k_contract_bf16's accumulators leave in 16-byte words), so a block of one wavefront takes four rows and the 256
// columns of one tile, 4 KiB of consecutive addresses per split, and a thread four columns.  A block is four
// wavefronts: four groups of rows (SHARE_SPLITS false), or, when that would leave most of the chip idle, one group
// of rows whose splits the four wavefronts share (wave w sums the splits w, w + 4, ..; the four sums meet in LDS and
// are added in the order of the waves).
template <bool SHARE_SPLITS>
__global__ void __launch_bounds__(256) k_finalize_bf16(const bf16_t* __restrict__ img, const bf16_t* __restrict__ txt,
                                                       int64_t ld_img, int64_t ld_txt, int64_t off, int64_t b, int64_t d,
                                                       const float* __restrict__ O1, const float* __restrict__ O2,
                                                       int nsplit, const float* __restrict__ c1,
                                                       const float* __restrict__ c2, const float* __restrict__ dcoef,
                                                       float* __restrict__ d_img, float* __restrict__ d_txt,
                                                       const double* __restrict__ red, int nblocks, int version,
                                                       const float* __restrict__ tau, float rho, float* __restrict__ loss,
                                                       float* __restrict__ d_tau) {
  __shared__ float4 meet[SHARE_SPLITS ? 3 : 1][4][64];     // [wave - 1][column of the thread][lane]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t r0 = ((int64_t)blockIdx.x * (SHARE_SPLITS ? 1 : 4) + (SHARE_SPLITS ? 0 : wave)) * 4;   // rows r0 .. r0 + 3
  const int64_t n0 = (int64_t)blockIdx.z * 256 + (int64_t)lane * 4;     // columns n0 .. n0 + 3 (d % 8 == 0)
  const int side = blockIdx.y;
  const bool live = r0 < b && n0 < d;
  const int nr = (int)(b - r0 < 4 ? b - r0 : 4);
  const bf16_t* X = side == 0 ? txt : img;          // the diagonal term takes the other side's row
  const int64_t ldx = side == 0 ? ld_txt : ld_img;
  float cown[4], dc[4];                             // requested ahead of the partial sums: one memory latency, not two
  uint2 xr[4];
  float acc[4][4] = {};                             // [column][row]
  if (live) {
    if (!SHARE_SPLITS || wave == 0) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int64_t r = r0 + (t < nr ? t : 0);
        cown[t] = (side == 0 ? c1 : c2)[r];
        dc[t] = dcoef[r];
        xr[t] = *(const uint2*)(X + (off + r) * ldx + n0);
      }
    }
    const float* O = side == 0 ? O1 : O2;
    const size_t split_stride = partial_split_floats(b, d);
    const int64_t tiles_m = (b + 255) / 256;
    const size_t at = (size_t)((n0 >> 8) * tiles_m + (r0 >> 8)) * kPartialTileFloats +
                      (size_t)((((r0 & 255) >> 2) * 256 + (n0 & 255)) * 4);
#pragma unroll 4
    for (int s = SHARE_SPLITS ? wave : 0; s < nsplit; s += SHARE_SPLITS ? 4 : 1) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float4 v = *(const float4*)(O + (size_t)s * split_stride + at + 4 * j);
        acc[j][0] += v.x; acc[j][1] += v.y; acc[j][2] += v.z; acc[j][3] += v.w;
      }
    }
  }
  if (SHARE_SPLITS) {
    if (wave > 0) {
#pragma unroll
      for (int j = 0; j < 4; ++j) meet[wave - 1][j][lane] = make_float4(acc[j][0], acc[j][1], acc[j][2], acc[j][3]);
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 0; w < 3; ++w)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float4 v = meet[w][j][lane];
        acc[j][0] += v.x; acc[j][1] += v.y; acc[j][2] += v.z; acc[j][3] += v.w;
      }
  }
  if (live) {
    float* out = (side == 0 ? d_img : d_txt) + r0 * d + n0;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (t >= nr) break;
      float4 o;
      o.x = cown[t] * acc[0][t] - dc[t] * __uint_as_float(xr[t].x << 16);
      o.y = cown[t] * acc[1][t] - dc[t] * __uint_as_float(xr[t].x & 0xffff0000u);
      o.z = cown[t] * acc[2][t] - dc[t] * __uint_as_float(xr[t].y << 16);
      o.w = cown[t] * acc[3][t] - dc[t] * __uint_as_float(xr[t].y & 0xffff0000u);
      *(float4*)(out + t * d) = o;
    }
  }
  if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x < 64)
    write_scalars(red, nblocks, b, version, tau, rho, loss, d_tau);
}

// Gradient through e^ = e / |e| (cosine similarity, Sec. 3) on the MFMA path, after k_finalize_bf16:
// out := (out - e^ (e^ . out)) / |e|, e^ = the side's own row.  One block per anchor and side.
__global__ void __launch_bounds__(256) k_norm_backward_bf16(const bf16_t* __restrict__ img, const bf16_t* __restrict__ txt,
                                                            int64_t ld_img, int64_t ld_txt, int64_t off, int64_t d,
                                                            float* __restrict__ d_img, float* __restrict__ d_txt,
                                                            const float* __restrict__ norm_img,
                                                            const float* __restrict__ norm_txt) {
  __shared__ float part[4];
  const int64_t r = blockIdx.x;
  const int side = blockIdx.y;
  const bf16_t* ep = side == 0 ? img + (off + r) * ld_img : txt + (off + r) * ld_txt;
  float* out = (side == 0 ? d_img : d_txt) + r * d;
  float dot = 0.f;
  for (int64_t n = threadIdx.x; n < d; n += 256) dot = fmaf(out[n], load_elem(ep + n), dot);
  dot = wave_sum(dot);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = dot;
  __syncthreads();
  dot = (part[0] + part[1]) + (part[2] + part[3]);
  const float inv = 1.0f / (side == 0 ? norm_img : norm_txt)[r];
  for (int64_t n = threadIdx.x; n < d; n += 256) out[n] = (out[n] - dot * load_elem(ep + n)) * inv;
}

void launch_finalize_bf16(const StepCtx& c) {
  const Layout& L = c.L;
  const dim3 block(256);
  const unsigned col_tiles = (unsigned)((L.d + 255) / 256);
  // four row groups per block unless that makes fewer than two blocks per compute unit: then one, its splits shared
  const bool share = (uint64_t)((L.b + 15) / 16) * 2 * col_tiles < 512 && L.nsplit >= 4;
  const dim3 grid((unsigned)(share ? (L.b + 3) / 4 : (L.b + 15) / 16), 2, col_tiles);
  auto* kernel = share ? k_finalize_bf16<true> : k_finalize_bf16<false>;
  hipLaunchKernelGGL(kernel, grid, block, 0, c.s, (const bf16_t*)c.buf.img_glob, (const bf16_t*)c.buf.txt_glob,
                     c.cfg.ld_img, c.cfg.ld_txt, L.off, L.b, L.d, (const float*)(c.ws + L.Opart[0]),
                     (const float*)(c.ws + L.Opart[1]), L.nsplit, (const float*)(c.ws + L.c1), (const float*)(c.ws + L.c2),
                     (const float*)(c.ws + L.dcoef), c.buf.d_img, c.buf.d_txt, (const double*)(c.ws + L.red),
                     L.nstate_blocks, c.cfg.version, c.buf.tau, c.cfg.rho, c.buf.loss, c.buf.d_tau);
}

void launch_norm_backward_bf16(const StepCtx& c) {
  const Layout& L = c.L;
  if (c.buf.norm_img)
    hipLaunchKernelGGL(k_norm_backward_bf16, dim3((unsigned)L.b, 2), dim3(256), 0, c.s, (const bf16_t*)c.buf.img_glob,
                       (const bf16_t*)c.buf.txt_glob, c.cfg.ld_img, c.cfg.ld_txt, L.off, L.d, c.buf.d_img, c.buf.d_txt,
                       c.buf.norm_img, c.buf.norm_txt);
}

// ------------------------------------------------------------------------------------------
// Index checker: open-addressing hash set of the b indices; flag word at ws[0].
__global__ void __launch_bounds__(256) k_idx_fill(int* flag, long long* table, size_t slots) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i == 0) *flag = 0;
  if (i < slots) table[i] = -1;
}

__global__ void __launch_bounds__(256) k_idx_insert(const int64_t* __restrict__ idx, int64_t b, int64_t N, int* flag,
                                                    unsigned long long* table, size_t slots, int shift) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= b) return;
  const int64_t v = idx[i];
  if (v < 0 || v >= N) { *flag = 1; return; }
  size_t h = (size_t)(((unsigned long long)v * 11400714819323198485ull) >> shift);
  for (size_t probe = 0; probe < slots; ++probe) {     // bounded: the table has at least 2b slots
    const unsigned long long old = atomicCAS(&table[h], ~0ull, (unsigned long long)v);
    if (old == ~0ull) return;
    if (old == (unsigned long long)v) { *flag = 1; return; }
    h = (h + 1) & (slots - 1);
  }
  *flag = 1;
}

void launch_check_indices(const int64_t* idx, int64_t b, int64_t N, void* ws, hipStream_t s) {
  size_t slots = 64;
  int log2s = 6;
  while (slots < (size_t)b * 2) { slots <<= 1; ++log2s; }
  int* flag = (int*)ws;
  long long* table = (long long*)((char*)ws + 256);
  hipLaunchKernelGGL(k_idx_fill, dim3((unsigned)((slots + 255) / 256)), dim3(256), 0, s, flag, table, slots);
  hipLaunchKernelGGL(k_idx_insert, dim3((unsigned)((b + 255) / 256)), dim3(256), 0, s, idx, b, N, flag,
                     (unsigned long long*)table, slots, 64 - log2s);
}

}  // namespace fc
