// MFMA kernels of the FCCO step on FINE tiles, for batches whose 256 x 256 tiles would leave most of the chip idle
// (the shapes the paper trains at: 128 - 640 anchors per worker of a global batch of 1024 - 5120, width 512):
//
//  k_strips_fine_bf16    the similarity strips of Proc. 1 on 128 x 128 tiles (any ragged edge): l = exp((s - s_ii) / tau),
//                        the per-anchor sums of l and (s - s_ii) l, l stored in the fragment order of the contraction;
//  k_contract_fine_bf16  the gradient contractions of Eqs. 2 - 7 on 64 x 64 output tiles.  With one split of the column
//                        range a workgroup owns its output tile for good and finishes it in place (coefficient,
//                        diagonal terms, the step's scalars): no partial results, no further kernel.  With several
//                        splits the partial tiles go to the workspace and k_finalize_fine_bf16 adds them up.
//
// Both kernels stage their operands through registers into a two-slot LDS ring (global load of stage s + 1 in flight
// while stage s is multiplied); many workgroups fit a compute unit, which hides what this simple pipeline leaves open.
// Layouts (stored strips, accumulator blocks) are those of the large-tile kernels: see kernels_mfma.hip.
#include <string.h>

#include "mfma_common.hpp"
#include "state_common.hpp"

namespace fc {

constexpr int kFT = 128;                 // rows of either operand in a fine strip tile
constexpr int kFK = 64;                  // contraction depth of a stage: 128 bytes per row
constexpr int kFOp = kFT * kFK * 2;      // one operand of a stage: 16 KiB

// LDS image of an operand of a stage (rows of 128 bytes): 16-byte chunk c of row r sits at chunk position
// c ^ ((r >> 1) & 7); the 16 consecutive rows that one operand read touches per cycle cover a whole bank window.
__device__ __forceinline__ int ft_swz(int row) { return (row >> 1) & 7; }

__global__ void __launch_bounds__(256) k_strips_fine_bf16(StripArgs a, int nAT, int nCT) {
  __shared__ __attribute__((aligned(1024))) char ring[2][2 * kFOp];   // [slot][contrast rows | anchor rows]
  __shared__ float sk[kFT];
  __shared__ float sdiag[kFT];
  __shared__ float sred[2][2][256];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave >> 1, wc = wave & 1, lr = lane & 31, hk = lane >> 5;
  const int t = blockIdx.x, per_strip = nAT * nCT;
  const int strip = t / per_strip, at = t % nAT, ct = (t / nAT) % nCT;
  const int64_t a0 = (int64_t)at * kFT, c0 = (int64_t)ct * kFT;
  if (tid < kFT) {
    const int64_t m = a0 + tid;
    sk[tid] = m < a.b ? a.kscale[strip][m] : 0.f;
    sdiag[tid] = m < a.b ? a.diag[m] : 0.f;
  }
  const bf16_t* X = a.contrasts[strip] + c0 * a.ld_contrast[strip];
  const bf16_t* A = a.anchors[strip] + a0 * a.ld_anchor[strip];
  const int64_t ldx = a.ld_contrast[strip], lda = a.ld_anchor[strip];
  const int64_t x_rows = a.B - c0, a_rows = a.B - a.off - a0;      // rows that exist below X / A
  const int S = (int)((a.d + kFK - 1) / kFK);
  // staging: thread -> chunk (tid & 7) of rows (tid >> 3) + 32 i, i = 0 .. 3, of both operands
  const int chunk = tid & 7, row0 = tid >> 3;
  u32x4 gx[4], ga[4];
  auto fetch = [&](int s) {
    const int64_t k = (int64_t)s * kFK + chunk * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = row0 + 32 * i;
      const u32x4 z = {0u, 0u, 0u, 0u};
      gx[i] = (k < a.d && row < x_rows) ? *(const u32x4*)(X + row * ldx + k) : z;
      ga[i] = (k < a.d && row < a_rows) ? *(const u32x4*)(A + row * lda + k) : z;
    }
  };
  auto stash = [&](int slot) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = row0 + 32 * i;
      const int o = row * 128 + ((chunk ^ ft_swz(row)) << 4);
      *(u32x4*)(ring[slot] + o) = gx[i];
      *(u32x4*)(ring[slot] + kFOp + o) = ga[i];
    }
  };
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  fetch(0);
  stash(0);
  __syncthreads();
  for (int s = 0; s < S; ++s) {
    if (s + 1 < S) fetch(s + 1);                       // in flight during the MFMAs below
    const char* sl = ring[s & 1];
#pragma unroll
    for (int j = 0; j < 4; ++j) {                      // 16-deep steps of the stage
      bf16x8 x[2], av[2];
#pragma unroll
      for (int ti = 0; ti < 2; ++ti) {
        const int row = wr * 64 + ti * 32 + lr;
        x[ti] = *(const bf16x8*)(sl + row * 128 + (((2 * j + hk) ^ ft_swz(row)) << 4));
      }
#pragma unroll
      for (int tj = 0; tj < 2; ++tj) {
        const int row = wc * 64 + tj * 32 + lr;
        av[tj] = *(const bf16x8*)(sl + kFOp + row * 128 + (((2 * j + hk) ^ ft_swz(row)) << 4));
      }
#pragma unroll
      for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int tj = 0; tj < 2; ++tj)
          acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[ti], av[tj], acc[ti][tj], 0, 0, 0);
    }
    if (s + 1 < S) stash((s + 1) & 1);                 // the other slot: last read before the previous barrier
    __syncthreads();
  }
  strip_epilogue<true, 2, 2>(a, acc, sk, sdiag, sred[wr], strip, a0, c0, wr * 64, wc * 64, lane);
  __syncthreads();
  if (tid < kFT) {
    const int64_t m = a0 + tid;
    if (m < a.b) {
#pragma unroll
      for (int q = 0; q < 2; ++q)
        a.sums[((size_t)(2 * strip + q) * a.nparts + ct) * a.bstride + m] = sred[0][q][tid] + sred[1][q][tid];
    }
  }
}

void launch_strips_fine_bf16(const StepCtx& c) {
  const Layout& L = c.L;
  const bf16_t* img = (const bf16_t*)c.buf.img_glob;
  const bf16_t* txt = (const bf16_t*)c.buf.txt_glob;
  StripArgs a;
  memset(&a, 0, sizeof(a));
  a.anchors[0] = img + L.off * c.cfg.ld_img;  a.ld_anchor[0] = c.cfg.ld_img;
  a.anchors[1] = txt + L.off * c.cfg.ld_txt;  a.ld_anchor[1] = c.cfg.ld_txt;
  a.contrasts[0] = txt;                       a.ld_contrast[0] = c.cfg.ld_txt;
  a.contrasts[1] = img;                       a.ld_contrast[1] = c.cfg.ld_img;
  a.diag = (const float*)(c.ws + L.diag);
  a.kscale[0] = (const float*)(c.ws + L.k1);
  a.kscale[1] = (const float*)(c.ws + L.k2);
  a.E[0] = (bf16_t*)(c.ws + L.E[0]);
  a.E[1] = (bf16_t*)(c.ws + L.E[1]);
  a.nCB = L.ldE / 16;
  a.ldE = L.ldE;
  a.sums = (float*)(c.ws + L.sums);
  a.nparts = L.nparts; a.bstride = L.bstride; a.b = L.b; a.B = L.B; a.d = L.d; a.off = L.off;
  const int nAT = (int)((L.b + kFT - 1) / kFT), nCT = (int)((L.B + kFT - 1) / kFT);
  hipLaunchKernelGGL(k_strips_fine_bf16, dim3((unsigned)(2 * nAT * nCT)), dim3(256), 0, c.s, a, nAT, nCT);
}

// ----------------------------------------------------------------------------------------------------------------
// Contraction on 64 x 64 output tiles.  C[m][n] = sum_c Efrag[m][c] X[c][n] over the contrast columns of one split.
// Waves (wm, wn): anchor block m0 / 32 + wm, columns n0 + 32 wn .. + 31, one accumulator block each.  The A operand
// (stored strip fragments) goes from global memory straight into the registers the MFMA reads (16 bytes per lane,
// 1 KiB per fragment and wave); the B operand, 64 rows x 64 columns of X per stage, goes through LDS in its natural
// layout (128-byte rows, 16-byte piece p of row k at piece position p ^ ((k & 2) << 1), so that the 4 rows x 64 bytes
// that a half wave's transposing read touches cover a whole bank window) and is read with ds_read_b64_tr_b16.
struct FineJob {
  const bf16_t* E;     // fragment-ordered strip of this side
  const bf16_t* X;     // the matrix whose rows the strip weights (texts for side 0, images for side 1): also the rows of
                       // the diagonal terms, d_img[r] -= dcoef[r] txt[off + r]
  const float* c_own;  // c1 (side 0) / c2 (side 1)
  float* out;          // d_img / d_txt
  int64_t ldx;
};
struct FineArgs {
  FineJob job[2];
  int64_t b, d, B, off, nCB;
  int tiles_m, tiles_n, nsplit, slice, stages;   // 64-deep stages in all, and per split
  float* part;         // nsplit > 1: [nsplit][2][b64][d64] partial results
  int64_t b64, d64;
  const float* dcoef;
  const double* red; int nred; int version; const float* tau; float rho; float* loss; float* d_tau;
};

__global__ void __launch_bounds__(256) k_contract_fine_bf16(FineArgs g) {
  __shared__ __attribute__((aligned(1024))) char ring[2][64 * 128];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1, lr = lane & 31, hk = lane >> 5;
  const int per_side = g.nsplit * g.tiles_m * g.tiles_n;
  const int side = (int)blockIdx.x / per_side, local = (int)blockIdx.x % per_side;
  const int split = local % g.nsplit, tile = local / g.nsplit;
  const int64_t m0 = (int64_t)(tile % g.tiles_m) * 64, n0 = (int64_t)(tile / g.tiles_m) * 64;
  const FineJob& J = g.job[side];
  const int s0 = split * g.slice;
  const int S = s0 + g.slice <= g.stages ? g.slice : g.stages - s0;      // >= 1 by construction
  // A operand: fragment (ab, cb) of this lane, cb = 4 stage + j
  const bf16_t* Ef = J.E + (((m0 >> 5) + wm) * g.nCB * 64 + lane) * 8;
  // B operand staging: thread -> piece (tid & 7) of rows (tid >> 3) and (tid >> 3) + 32 of the stage
  const int piece = tid & 7, krow = tid >> 3;
  const bool col_ok = n0 + piece * 8 < g.d;
  u32x4 gb[2];
  bf16x8 ga[4];
  auto fetch = [&](int s) {
    const int64_t cfirst = (int64_t)(s0 + s) * 64;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int64_t c = cfirst + krow + 32 * i;
      const u32x4 z = {0u, 0u, 0u, 0u};
      gb[i] = (col_ok && c < g.B) ? *(const u32x4*)(J.X + c * J.ldx + n0 + piece * 8) : z;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) ga[j] = *(const bf16x8*)(Ef + ((int64_t)(s0 + s) * 4 + j) * 512);
  };
  auto stash = [&](int slot) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int k = krow + 32 * i;
      *(u32x4*)(ring[slot] + k * 128 + ((piece ^ ((k & 2) << 1)) << 4)) = gb[i];
    }
  };
  // transposing read: the 16 lanes of a group hand each other 4 rows x 16 columns; lane L ends up with the 4 rows
  // 16 j + 8 half + 4 hk + (0 .. 3) of column wn 32 + (L & 31)
  const int s16 = lane & 15;
  const int ncol = wn * 32 + ((lane >> 4) & 1) * 16 + 4 * (s16 & 3);      // first of the 4 columns this lane reads
  auto read_b = [&](const char* sl, int j) {
    u32x2 h2[2];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int k = 16 * j + 8 * half + 4 * hk + (s16 >> 2);
      const char* p = sl + k * 128 + ((((ncol >> 3) ^ ((k & 2) << 1))) << 4) + ((ncol & 7) << 1);
      h2[half] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)(uintptr_t)lds_addr(p)));
    }
    return join_halves(h2[0], h2[1]);
  };
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  fetch(0);
  stash(0);
  __syncthreads();
  for (int s = 0; s < S; ++s) {
    bf16x8 a_now[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) a_now[j] = ga[j];
    if (s + 1 < S) fetch(s + 1);
    const char* sl = ring[s & 1];
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_now[j], read_b(sl, j), acc, 0, 0, 0);
    if (s + 1 < S) stash((s + 1) & 1);
    __syncthreads();
  }
  // accumulator v of lane (lr, hk): row m0 + 32 wm + 8 (v >> 2) + 4 hk + (v & 3), column n0 + 32 wn + lr
  const int64_t n = n0 + wn * 32 + lr;
  if (g.nsplit == 1) {
    // the tile is complete: d[r][n] = c_own[r] C[r][n] - (c1 M g1 + c2 M g2)[r] x_partner[off + r][n]
    if (n < g.d) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t m = m0 + wm * 32 + 8 * (v >> 2) + 4 * hk + (v & 3);
        if (m < g.b)
          J.out[m * g.d + n] = J.c_own[m] * acc[v] - g.dcoef[m] * bf2f(J.X[(g.off + m) * J.ldx + n]);
      }
    }
    if (blockIdx.x == 0 && tid < 64) write_scalars(g.red, g.nred, g.b, g.version, g.tau, g.rho, g.loss, g.d_tau);
  } else {
    float* P = g.part + ((size_t)(split * 2 + side) * g.b64) * g.d64;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t m = m0 + wm * 32 + 8 * (v >> 2) + 4 * hk + (v & 3);
      P[m * g.d64 + n] = acc[v];                                   // whole 64 x 64 tiles exist in the buffer
    }
  }
}

// Several splits: d[r][n] = c_own[r] (sum over the splits, in their order) - dcoef[r] x_partner[off + r][n].
// A thread takes four consecutive columns of one row (d % 8 == 0 on this path).
__global__ void __launch_bounds__(256) k_finalize_fine_bf16(FineArgs g) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t per_row = g.d / 4;
  const int side = blockIdx.y;
  const FineJob& J = g.job[side];
  if (q < g.b * per_row) {
    const int64_t m = q / per_row, n = (q % per_row) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < g.nsplit; ++s) {
      const float4 v = *(const float4*)(g.part + ((size_t)(s * 2 + side) * g.b64 + m) * g.d64 + n);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    const uint2 xr = *(const uint2*)(J.X + (g.off + m) * J.ldx + n);
    const float c = J.c_own[m], dc = g.dcoef[m];
    float4 o;
    o.x = c * acc.x - dc * __uint_as_float(xr.x << 16);
    o.y = c * acc.y - dc * __uint_as_float(xr.x & 0xffff0000u);
    o.z = c * acc.z - dc * __uint_as_float(xr.y << 16);
    o.w = c * acc.w - dc * __uint_as_float(xr.y & 0xffff0000u);
    *(float4*)(J.out + m * g.d + n) = o;
  }
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 64)
    write_scalars(g.red, g.nred, g.b, g.version, g.tau, g.rho, g.loss, g.d_tau);
}

void launch_contract_fine_bf16(const StepCtx& c) {
  const Layout& L = c.L;
  FineArgs g;
  memset(&g, 0, sizeof(g));
  for (int s = 0; s < 2; ++s) {
    FineJob& J = g.job[s];
    J.E = (const bf16_t*)(c.ws + L.E[s]);
    J.X = (const bf16_t*)(s == 0 ? c.buf.txt_glob : c.buf.img_glob);
    J.ldx = s == 0 ? c.cfg.ld_txt : c.cfg.ld_img;
    J.c_own = (const float*)(c.ws + (s == 0 ? L.c1 : L.c2));
    J.out = s == 0 ? c.buf.d_img : c.buf.d_txt;
  }
  g.b = L.b; g.d = L.d; g.B = L.B; g.off = L.off; g.nCB = L.ldE / 16;
  g.tiles_m = (int)((L.b + 63) / 64); g.tiles_n = (int)((L.d + 63) / 64);
  g.nsplit = L.nsplit; g.slice = (int)L.kslice; g.stages = (int)(L.ldE / 64);
  g.part = L.nsplit > 1 ? (float*)(c.ws + L.Opart[0]) : nullptr;
  g.b64 = (int64_t)round_up((size_t)L.b, 64); g.d64 = (int64_t)round_up((size_t)L.d, 64);
  g.dcoef = (const float*)(c.ws + L.dcoef);
  g.red = (const double*)(c.ws + L.red); g.nred = L.nstate_blocks; g.version = c.cfg.version; g.tau = c.buf.tau;
  g.rho = c.cfg.rho; g.loss = c.buf.loss; g.d_tau = c.buf.d_tau;
  const unsigned grid = 2u * (unsigned)(g.nsplit * g.tiles_m * g.tiles_n);
  hipLaunchKernelGGL(k_contract_fine_bf16, dim3(grid), dim3(256), 0, c.s, g);
  if (g.nsplit > 1) {
    const int64_t quads = L.b * (L.d / 4);
    hipLaunchKernelGGL(k_finalize_fine_bf16, dim3((unsigned)((quads + 255) / 256), 2), dim3(256), 0, c.s, g);
  }
}

}  // namespace fc
