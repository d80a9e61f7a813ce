// bf16 MFMA kernels of the FCCO step for gfx950 (wave64, v_mfma_f32_32x32x16_bf16).
//
//  k_strips_bf16   S = anchors x contrasts^T tile by tile from LDS-staged operands, then in registers
//                  l = exp((s - s_ii)/tau) (Sec. 3), row sums of l and of (s - s_ii) l (Proc. 1 and the
//                  nabla_3 l sums of Eqs. 8-10), and l rounded to bf16 stored as the operand of the
//                  gradient contraction.  The similarity matrix itself never reaches memory.
//  k_local_bf16    the local b x b block of the other side's strip, scaled by that side's coefficients
//                  and transposed: the operand of the contrast-side term of Eqs. 3 / 5 / 7.
//  k_gemm_nn_bf16  C = A x Bm with A [M][K] and Bm [K][N] both row-major (the contraction runs over the
//                  ROW index of Bm, so Bm tiles are transposed in registers on their way to LDS), split
//                  over K into per-slice fp32 partial results.  Used for sum_j l(r,j) x_j (Eqs. 2/4/6) and
//                  for the local contrast-side term.
//
// Workgroup = 256 threads = 2 x 2 wavefronts, each owning a 128 x 128 accumulator block (4 x 4 MFMA tiles,
// 256 fp32 accumulators per lane); workgroup tile 256 x 256, contraction depth 64 per LDS stage, two stages.
// MFMA operand layout used throughout (32x32x16, wave64): lane l supplies row (l & 31) of its operand and the
// 8 consecutive k values starting at 8 * (l >> 5); accumulator register v of lane l is
// D[8 * (v >> 2) + 4 * (l >> 5) + (v & 3)][l & 31].
#include "fc_internal.hpp"

namespace fc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int TM = 256, TN = 256, TK = 64;
constexpr int kTileElems = 256 * TK;      // one operand tile in LDS: 256 rows x 64 k (bf16) = 32 KiB

// 16-byte chunk c (0..7) of row `row` lives at chunk position c ^ swz(row): conflict-free both for
// row-wise stores (8 lanes per row), for the transposed stores of k_gemm_nn_bf16 (lanes 8 rows apart) and
// for MFMA operand reads (32 consecutive rows, one chunk).
__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * TK + ((chunk ^ swz(row)) << 3); }

__device__ __forceinline__ uint16_t f2bf(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }
__device__ __forceinline__ float bf2f(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }

// Global -> registers for a K-contiguous operand tile (256 rows x 64 k): thread t fetches chunk (t & 7)
// of rows (t >> 3) + 32 i.  Rows >= rows_valid and k >= k_valid read as zero.
__device__ __forceinline__ void gload_rows(u32x4 (&reg)[8], const bf16_t* __restrict__ base, int64_t ld,
                                           int64_t row0, int64_t rows_valid, int64_t k0, int64_t k_valid, int tid) {
  const int64_t k = k0 + ((tid & 7) << 3);
  const bool kok = k < k_valid;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t row = row0 + (tid >> 3) + 32 * i;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (kok && row < rows_valid) v = *(const u32x4*)(base + row * ld + k);
    reg[i] = v;
  }
}
__device__ __forceinline__ void lds_store_rows(bf16_t* tile, const u32x4 (&reg)[8], int tid) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = (tid >> 3) + 32 * i;
    *(u32x4*)(tile + lds_off(row, tid & 7)) = reg[i];
  }
}

// Global -> registers for a tile of a [K][N] row-major matrix (64 k rows x 256 n columns): thread t fetches,
// for k rows 8 (t >> 5) + i, the 8 columns starting at 8 (t & 31).  Then an 8 x 8 transpose in registers and
// a store so that LDS holds the tile as [n][k], k contiguous, exactly like a K-contiguous operand.
__device__ __forceinline__ void gload_cols(u32x4 (&reg)[8], const bf16_t* __restrict__ base, int64_t ld,
                                           int64_t k0, int64_t k_valid, int64_t n0, int64_t n_valid, int tid) {
  const int64_t n = n0 + ((tid & 31) << 3);
  const bool nok = n < n_valid;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t k = k0 + ((tid >> 5) << 3) + i;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (nok && k < k_valid) v = *(const u32x4*)(base + k * ld + n);
    reg[i] = v;
  }
}
__device__ __forceinline__ void lds_store_cols_transposed(bf16_t* tile, const u32x4 (&reg)[8], int tid) {
  const int kchunk = tid >> 5;
#pragma unroll
  for (int j = 0; j < 8; ++j) {          // column n = 8 (t & 31) + j of the tile
    u32x4 o;
#pragma unroll
    for (int w = 0; w < 4; ++w) {        // output word w holds k = 2w (low half) and 2w + 1 (high half)
      const uint32_t lo = reg[2 * w][j >> 1], hi = reg[2 * w + 1][j >> 1];
      o[w] = (j & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
    }
    const int row = ((tid & 31) << 3) + j;
    *(u32x4*)(tile + lds_off(row, kchunk)) = o;
  }
}

// One LDS stage: acc[ti][tj] += A(128 rows of this wave) x B(128 rows of this wave)^T over 64 k.
__device__ __forceinline__ void mma_stage(f32x16 (&acc)[4][4], const bf16_t* tA, const bf16_t* tB, int wm, int wn,
                                          int lane) {
  const int lr = lane & 31, hk = lane >> 5;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    bf16x8 a[4], bq[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      a[t] = *(const bf16x8*)(tA + lds_off(wm * 128 + t * 32 + lr, kk * 2 + hk));
      bq[t] = *(const bf16x8*)(tB + lds_off(wn * 128 + t * 32 + lr, kk * 2 + hk));
    }
#pragma unroll
    for (int ti = 0; ti < 4; ++ti)
#pragma unroll
      for (int tj = 0; tj < 4; ++tj)
        acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ti], bq[tj], acc[ti][tj], 0, 0, 0);
  }
}

// Sum each of v[0..15] over the 32 lanes of a half-wave.  On return lane l holds, in the result, the total
// of register index (l & 31) >> 1 (both lanes of a pair hold the same value).
__device__ __forceinline__ float halfwave_sum16(const float (&v)[16], int lane) {
  float r8[8], r4[4], r2[2];
  const bool b4 = lane & 16, b3 = lane & 8, b2 = lane & 4, b1 = lane & 2;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float mine = b4 ? v[i + 8] : v[i], send = b4 ? v[i] : v[i + 8];
    r8[i] = mine + __shfl_xor(send, 16);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float mine = b3 ? r8[i + 4] : r8[i], send = b3 ? r8[i] : r8[i + 4];
    r4[i] = mine + __shfl_xor(send, 8);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float mine = b2 ? r4[i + 2] : r4[i], send = b2 ? r4[i] : r4[i + 2];
    r2[i] = mine + __shfl_xor(send, 4);
  }
  const float mine = b1 ? r2[1] : r2[0], send = b1 ? r2[0] : r2[1];
  float r = mine + __shfl_xor(send, 2);
  r += __shfl_xor(r, 1);
  return r;   // register index = b1 + 2 b2 + 4 b3 + 8 b4 = (lane & 31) >> 1
}

// ------------------------------------------------------------------------------------------
struct StripArgs {
  const bf16_t* anchors[2];     // first local row of the anchor side (image rows for strip 0, text rows for strip 1)
  const bf16_t* contrasts[2];   // row 0 of the contrast side (texts for strip 0, images for strip 1)
  int64_t ld_anchor[2], ld_contrast[2];
  const float* diag;            // s_pp per local anchor
  const float* kscale[2];       // log2(e) / tau of the anchor for each strip
  bf16_t* E[2];                 // [b][ldE] out
  int64_t ldE;
  float* sums;                  // [4][nparts][bstride] out
  int nparts;
  int64_t bstride, b, B, d, off;
  int nAT, nCT;
};

template <bool GUARD>
__device__ __forceinline__ void strip_epilogue(const StripArgs& a, f32x16 (&acc)[4][4], const float* sdiag,
                                               const float* sk, float (*sred)[2][256], int strip, int64_t m0,
                                               int64_t n0, int wm, int wn, int lane) {
  const int lr = lane & 31, hk = lane >> 5;
  bf16_t* __restrict__ E = a.E[strip];
#pragma unroll
  for (int ti = 0; ti < 4; ++ti) {
    float sg[16], sh[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) { sg[v] = 0.f; sh[v] = 0.f; }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int rl = wm * 128 + ti * 32 + 8 * q + 4 * hk;           // first of 4 consecutive tile rows
      const float4 dg = *(const float4*)(sdiag + rl);
      const float4 ks = *(const float4*)(sk + rl);
      const float dgv[4] = {dg.x, dg.y, dg.z, dg.w}, ksv[4] = {ks.x, ks.y, ks.z, ks.w};
#pragma unroll
      for (int tj = 0; tj < 4; ++tj) {
        const int64_t n = n0 + wn * 128 + tj * 32 + lr;             // global contrast row
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int v = 4 * q + t;
          const int64_t m = m0 + rl + t;                            // local anchor
          const float x = acc[ti][tj][v] - dgv[t];
          float e = __builtin_amdgcn_exp2f(x * ksv[t]);
          if (GUARD) {
            const bool ok = (n < a.B) && (m < a.b) && (n != a.off + m);
            e = ok ? e : 0.f;
            if (m < a.b && n < a.ldE) E[m * a.ldE + n] = f2bf(e);
          } else {
            E[m * a.ldE + n] = f2bf(e);
          }
          sg[v] += e;
          sh[v] += x * e;
        }
      }
    }
    const float tg = halfwave_sum16(sg, lane);
    const float th = halfwave_sum16(sh, lane);
    if ((lr & 1) == 0) {
      const int v = lr >> 1;
      const int row = wm * 128 + ti * 32 + 8 * (v >> 2) + 4 * hk + (v & 3);
      sred[wn][0][row] = tg;
      sred[wn][1][row] = th;
    }
  }
}

__global__ void __launch_bounds__(256) k_strips_bf16(StripArgs a) {
  __shared__ __attribute__((aligned(16))) bf16_t lds[2][2][kTileElems];   // [stage][anchors | contrasts]
  __shared__ __attribute__((aligned(16))) float sdiag[256];
  __shared__ __attribute__((aligned(16))) float sk[256];
  __shared__ float sred[2][2][256];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int strip = blockIdx.y;
  // workgroups that share a contrast tile sit on the same XCD (round-robin dispatch: id mod 8) back to back
  const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
  const int at = jj % a.nAT;
  const int ct = (jj / a.nAT) * 8 + xcd;
  if (ct >= a.nCT) return;
  const int64_t m0 = (int64_t)at * TM, n0 = (int64_t)ct * TN;

  {
    const int64_t m = m0 + tid;
    sdiag[tid] = m < a.b ? a.diag[m] : 0.f;
    sk[tid] = m < a.b ? a.kscale[strip][m] : 0.f;
  }

  const bf16_t* __restrict__ A = a.anchors[strip];
  const bf16_t* __restrict__ X = a.contrasts[strip];
  const int64_t lda = a.ld_anchor[strip], ldx = a.ld_contrast[strip];

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int KT = (int)((a.d + TK - 1) / TK);
  u32x4 ra[8], rb[8];
  gload_rows(ra, A, lda, m0, a.b, 0, a.d, tid);
  gload_rows(rb, X, ldx, n0, a.B, 0, a.d, tid);
  lds_store_rows(lds[0][0], ra, tid);
  lds_store_rows(lds[0][1], rb, tid);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < KT;
    if (more) {
      gload_rows(ra, A, lda, m0, a.b, (int64_t)(kt + 1) * TK, a.d, tid);
      gload_rows(rb, X, ldx, n0, a.B, (int64_t)(kt + 1) * TK, a.d, tid);
    }
    mma_stage(acc, lds[cur][0], lds[cur][1], wm, wn, lane);
    if (more) {
      lds_store_rows(lds[cur ^ 1][0], ra, tid);
      lds_store_rows(lds[cur ^ 1][1], rb, tid);
    }
    __syncthreads();
  }

  // tiles that touch the own-column diagonal or a ragged edge take the guarded epilogue
  const bool ragged = (m0 + TM > a.b) || (n0 + TN > a.B);
  const bool diagonal = (n0 < a.off + m0 + TM) && (n0 + TN > a.off + m0);
  if (ragged || diagonal)
    strip_epilogue<true>(a, acc, sdiag, sk, sred, strip, m0, n0, wm, wn, lane);
  else
    strip_epilogue<false>(a, acc, sdiag, sk, sred, strip, m0, n0, wm, wn, lane);
  __syncthreads();
  {
    const int64_t m = m0 + tid;
    if (m < a.b) {
#pragma unroll
      for (int q = 0; q < 2; ++q)
        a.sums[((size_t)(2 * strip + q) * a.nparts + ct) * a.bstride + m] = sred[0][q][tid] + sred[1][q][tid];
    }
  }
}

void launch_strips_bf16(const StepCtx& c) {
  const Layout& L = c.L;
  const bf16_t* img = (const bf16_t*)c.buf.img_glob;
  const bf16_t* txt = (const bf16_t*)c.buf.txt_glob;
  StripArgs a;
  a.anchors[0] = img + L.off * c.cfg.ld_img;  a.ld_anchor[0] = c.cfg.ld_img;
  a.anchors[1] = txt + L.off * c.cfg.ld_txt;  a.ld_anchor[1] = c.cfg.ld_txt;
  a.contrasts[0] = txt;                       a.ld_contrast[0] = c.cfg.ld_txt;
  a.contrasts[1] = img;                       a.ld_contrast[1] = c.cfg.ld_img;
  a.diag = (const float*)(c.ws + L.diag);
  a.kscale[0] = (const float*)(c.ws + L.k1);
  a.kscale[1] = (const float*)(c.ws + L.k2);
  a.E[0] = (bf16_t*)(c.ws + L.E[0]);
  a.E[1] = (bf16_t*)(c.ws + L.E[1]);
  a.ldE = L.ldE;
  a.sums = (float*)(c.ws + L.sums);
  a.nparts = L.nparts; a.bstride = L.bstride; a.b = L.b; a.B = L.B; a.d = L.d; a.off = L.off;
  a.nAT = (int)((L.b + TM - 1) / TM);
  a.nCT = (int)((L.B + TN - 1) / TN);
  const unsigned gx = 8u * (unsigned)a.nAT * (unsigned)((a.nCT + 7) / 8);
  hipLaunchKernelGGL(k_strips_bf16, dim3(gx, 2), dim3(256), 0, c.s, a);
}

// ------------------------------------------------------------------------------------------
// WT[side][r][q] = c_other[q] * l_other(q, off + r)  for local anchors q != r (the stored strips already hold 0
// at q == r), zero for q >= b.  side 0 feeds d_img (other = text side: c2, l2), side 1 feeds d_txt.
__global__ void __launch_bounds__(256) k_local_bf16(const bf16_t* __restrict__ E1, const bf16_t* __restrict__ E2,
                                                    int64_t ldE, const float* __restrict__ c1,
                                                    const float* __restrict__ c2, int64_t off, int64_t b,
                                                    bf16_t* __restrict__ WT0, bf16_t* __restrict__ WT1, int64_t ldW) {
  __shared__ float tile[64][65];
  const int side = blockIdx.z;
  const bf16_t* __restrict__ E = side == 0 ? E2 : E1;
  const float* __restrict__ cc = side == 0 ? c2 : c1;
  bf16_t* __restrict__ WT = side == 0 ? WT0 : WT1;
  const int64_t r0 = (int64_t)blockIdx.x * 64, q0 = (int64_t)blockIdx.y * 64;
  const int x = threadIdx.x & 63, y = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int64_t q = q0 + y + 4 * i, r = r0 + x;
    float v = 0.f;
    if (q < b && r < b) v = cc[q] * bf2f(E[q * ldE + off + r]);
    tile[y + 4 * i][x] = v;          // [q][r]
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int64_t r = r0 + y + 4 * i, q = q0 + x;
    if (r < b && q < ldW) WT[r * ldW + q] = f2bf(tile[x][y + 4 * i]);
  }
}

void launch_local_bf16(const StepCtx& c) {
  const Layout& L = c.L;
  dim3 grid((unsigned)((L.b + 63) / 64), (unsigned)(L.ldW / 64), 2);
  hipLaunchKernelGGL(k_local_bf16, grid, dim3(256), 0, c.s, (const bf16_t*)(c.ws + L.E[0]),
                     (const bf16_t*)(c.ws + L.E[1]), L.ldE, (const float*)(c.ws + L.c1), (const float*)(c.ws + L.c2),
                     L.off, L.b, (bf16_t*)(c.ws + L.WT[0]), (bf16_t*)(c.ws + L.WT[1]), L.ldW);
}

// ------------------------------------------------------------------------------------------
struct GemmJob {
  const bf16_t* A;    // [M][lda], K contiguous; readable and zero beyond K up to a_kvalid (multiple of 8)
  const bf16_t* Bm;   // [K][ldb], N contiguous
  float* C;           // [nsplit][M][ldc]
  int64_t lda, ldb, ldc, a_kvalid, M, N, K, kslice;
  size_t split_stride;
  int nsplit, tiles_m, wg_begin, wg_end;
};
struct GemmArgs {
  GemmJob job[4];
  int njobs;
};

__global__ void __launch_bounds__(256) k_gemm_nn_bf16(GemmArgs g) {
  __shared__ __attribute__((aligned(16))) bf16_t lds[2][2][kTileElems];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int ji = 0;
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if (i < g.njobs && (int)blockIdx.x >= g.job[i].wg_begin) ji = i;
  const GemmJob& J = g.job[ji];
  const int local = (int)blockIdx.x - J.wg_begin;
  const int split = local % J.nsplit;           // consecutive ids -> different XCDs -> different K slices
  const int tile = local / J.nsplit;
  const int64_t m0 = (int64_t)(tile % J.tiles_m) * TM, n0 = (int64_t)(tile / J.tiles_m) * TN;
  const int64_t kbeg = (int64_t)split * J.kslice;
  const int64_t kend = kbeg + J.kslice < J.K ? kbeg + J.kslice : J.K;
  const int64_t a_kend = kbeg + J.kslice < J.a_kvalid ? kbeg + J.kslice : J.a_kvalid;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int KT = (int)((kend - kbeg + TK - 1) / TK);
  u32x4 ra[8], rb[8];
  if (KT > 0) {
    gload_rows(ra, J.A, J.lda, m0, J.M, kbeg, a_kend, tid);
    gload_cols(rb, J.Bm, J.ldb, kbeg, kend, n0, J.N, tid);
    lds_store_rows(lds[0][0], ra, tid);
    lds_store_cols_transposed(lds[0][1], rb, tid);
  }
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < KT;
    if (more) {
      gload_rows(ra, J.A, J.lda, m0, J.M, kbeg + (int64_t)(kt + 1) * TK, a_kend, tid);
      gload_cols(rb, J.Bm, J.ldb, kbeg + (int64_t)(kt + 1) * TK, kend, n0, J.N, tid);
    }
    mma_stage(acc, lds[cur][0], lds[cur][1], wm, wn, lane);
    if (more) {
      lds_store_rows(lds[cur ^ 1][0], ra, tid);
      lds_store_cols_transposed(lds[cur ^ 1][1], rb, tid);
    }
    __syncthreads();
  }

  float* __restrict__ C = J.C + (size_t)split * J.split_stride;
  const int lr = lane & 31, hk = lane >> 5;
#pragma unroll
  for (int ti = 0; ti < 4; ++ti)
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
      const int64_t n = n0 + wn * 128 + tj * 32 + lr;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t m = m0 + wm * 128 + ti * 32 + 8 * (v >> 2) + 4 * hk + (v & 3);
        if (m < J.M && n < J.N) C[m * J.ldc + n] = acc[ti][tj][v];
      }
    }
}

void launch_contract_bf16(const StepCtx& c) {
  const Layout& L = c.L;
  const bf16_t* img = (const bf16_t*)c.buf.img_glob;
  const bf16_t* txt = (const bf16_t*)c.buf.txt_glob;
  GemmArgs g;
  g.njobs = 4;
  const int tiles_m = (int)((L.b + TM - 1) / TM), tiles_n = (int)((L.d + TN - 1) / TN);
  int wg = 0;
  for (int s = 0; s < 2; ++s) {           // sum_j l(r, j) x_j over all contrasts, split over j
    GemmJob& J = g.job[s];
    J.A = (const bf16_t*)(c.ws + L.E[s]);  J.lda = L.ldE;  J.a_kvalid = L.ldE;
    J.Bm = s == 0 ? txt : img;             J.ldb = s == 0 ? c.cfg.ld_txt : c.cfg.ld_img;
    J.C = (float*)(c.ws + L.Opart[s]);     J.ldc = L.d;
    J.split_stride = (size_t)L.b * (size_t)L.d;
    J.M = L.b; J.N = L.d; J.K = L.B; J.kslice = L.kslice; J.nsplit = L.nsplit; J.tiles_m = tiles_m;
    J.wg_begin = wg;  wg += tiles_m * tiles_n * L.nsplit;  J.wg_end = wg;
  }
  for (int s = 0; s < 2; ++s) {           // local contrast-side term: WT[s] x (local rows of the same matrix)
    GemmJob& J = g.job[2 + s];
    J.A = (const bf16_t*)(c.ws + L.WT[s]); J.lda = L.ldW;  J.a_kvalid = L.ldW;
    J.Bm = s == 0 ? txt + L.off * c.cfg.ld_txt : img + L.off * c.cfg.ld_img;
    J.ldb = s == 0 ? c.cfg.ld_txt : c.cfg.ld_img;
    J.C = (float*)(c.ws + L.A6[s]);        J.ldc = L.d;
    J.split_stride = 0;
    J.M = L.b; J.N = L.d; J.K = L.b; J.kslice = (int64_t)round_up((size_t)L.b, TK); J.nsplit = 1; J.tiles_m = tiles_m;
    J.wg_begin = wg;  wg += tiles_m * tiles_n;  J.wg_end = wg;
  }
  hipLaunchKernelGGL(k_gemm_nn_bf16, dim3((unsigned)wg), dim3(256), 0, c.s, g);
}

}  // namespace fc
