// MFMA kernels of the FCCO step on 128 x 128 tiles, for batches whose 256 x 256 tiles would leave most of the chip idle
// (the shapes the paper trains at: 128 - 640 anchors per worker of a global batch of 1024 - 5120, width 512):
//
//  k_strips_t128_bf16    the similarity strips of Proc. 1: l = exp((s - s_ii) / tau), the per-anchor sums of l and
//                        (s - s_ii) l, l stored in the fragment order of the contraction; any ragged edge;
//  k_contract_t128_bf16  the gradient contractions of Eqs. 2 - 7 on 128 x 128 output tiles.  With one split of the column
//                        range a workgroup owns its output tile for good and finishes it in place (coefficient,
//                        diagonal terms, the step's scalars): no partial results, no further kernel.  With several
//                        splits the partial tiles go to the workspace and k_finalize_t128_bf16 adds them up.
//
// Both run the pipeline of the large-tile contraction in small: a ring of five LDS slots, each one 32-deep stage of
// both operands (16 KiB), filled by direct-to-LDS loads four stages ahead, one barrier per stage; four wavefronts with
// 2 x 2 accumulator blocks each.  Two workgroups share a compute unit (80 KiB of LDS each), which hides what the plain
// instruction order of the loop leaves open.  Layouts (stored strips, accumulator blocks, LDS images) are those of the
// large-tile kernels: see kernels_mfma.hip.
#include <string.h>

#include "mfma_common.hpp"
#include "state_common.hpp"

namespace fc {

constexpr int kT = 128;                         // rows of either operand of a strip tile; rows and columns of an output tile
constexpr int kHalf = kT * BK * 2;              // one operand of a stage: 8 KiB
constexpr int kSlot = 2 * kHalf;                // 16 KiB
constexpr int kSlots = 5;                       // stages are requested four ahead (eight ahead in a ring of nine measured no faster)
constexpr int kSmallRing = kSlots * kSlot;      // 80 KiB: two workgroups per compute unit

// "at most 4 n loads of this wave in flight", n = 0 .. 7 (s_waitcnt takes an immediate)
__device__ __forceinline__ void wait_younger_stages(int n) {
  switch (n) {
    case 0: __builtin_amdgcn_s_waitcnt(0x0f70); break;
    case 1: __builtin_amdgcn_s_waitcnt(0x0f74); break;
    case 2: __builtin_amdgcn_s_waitcnt(0x0f78); break;
    case 3: __builtin_amdgcn_s_waitcnt(0x0f7c); break;
    case 4: __builtin_amdgcn_s_waitcnt(0x4f70); break;
    case 5: __builtin_amdgcn_s_waitcnt(0x4f74); break;
    case 6: __builtin_amdgcn_s_waitcnt(0x4f78); break;
    default: __builtin_amdgcn_s_waitcnt(0x4f7c); break;
  }
}
// nothing may move across: the compiler does not see the direct-to-LDS loads write the ring
#define FC_FENCE() do { FC_PIN(); asm volatile("" ::: "memory"); FC_PIN(); } while (0)

// acc += (A operand tile) x (B operand tile)^T over the stages [s0, s0 + S), S >= 1.  Tile::dma(i, stage, slot address),
// i = 0 .. 3, issues this wave's four wave loads of a stage.  Stage s lives in slot s mod 5; its loads are issued four
// stages before it is read, right after the barrier of stage s - 4 ... which every wave passes only after its last read
// of stage s - 5, the slot's previous tenant.  Vector memory operations complete in order, so "stage s has landed" is
// "at most 4 x (stages requested after it) loads in flight".  On return no wave reads the ring any more.
template <typename Tile>
__device__ __forceinline__ void small_ring(f32x16 (&acc)[2][2], const Tile& T, char* ring, uint32_t ring_addr, int s0,
                                           int S) {
  constexpr int kAhead = kSlots - 1;
#pragma unroll
  for (int p = 0; p < kAhead; ++p)
    if (p < S) {
#pragma unroll
      for (int i = 0; i < 4; ++i) T.dma(i, s0 + p, ring_addr + (uint32_t)(p * kSlot));
    }
  int slot = 0, fill = kAhead;                  // slot of stage s; slot that the stage kAhead on goes to
  for (int s = 0; s < S; ++s) {
    wait_younger_stages(S - 1 - s < kAhead - 1 ? S - 1 - s : kAhead - 1);
    __builtin_amdgcn_s_barrier();
    FC_FENCE();
    if (s + kAhead < S) {
#pragma unroll
      for (int i = 0; i < 4; ++i) T.dma(i, s0 + s + kAhead, ring_addr + (uint32_t)(fill * kSlot));
    }
    const char* sl = ring + slot * kSlot;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) { a[t] = T.read_a(sl, t, kk); b[t] = T.read_b(sl, t, kk); }
#pragma unroll
      for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int tj = 0; tj < 2; ++tj)
          acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ti], b[tj], acc[ti][tj], 0, 0, 0);
    }
    FC_FENCE();
    slot = slot + 1 == kSlots ? 0 : slot + 1;
    fill = fill + 1 == kSlots ? 0 : fill + 1;
  }
  __syncthreads();
}

// The same for stages at a ragged end: one at a time through registers, zero fill outside (Tile::fill_guarded).
template <typename Tile>
__device__ __forceinline__ void small_guarded(f32x16 (&acc)[2][2], const Tile& T, char* ring, int s0, int S, int tid) {
  for (int s = 0; s < S; ++s) {
    __syncthreads();
    T.fill_guarded(s0 + s, ring, tid);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) { a[t] = T.read_a(ring, t, kk); b[t] = T.read_b(ring, t, kk); }
#pragma unroll
      for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int tj = 0; tj < 2; ++tj)
          acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ti], b[tj], acc[ti][tj], 0, 0, 0);
    }
  }
  __syncthreads();
}

// ----------------------------------------------------------------------------------------------------------------
// Strip tile: both operands are K-contiguous row tiles of 128 rows x 32 of k (64 bytes per row, LDS image rt_off).
// A operand of the MFMA = contrast rows, B operand = anchor rows.  A wave load takes 16 rows; wave w issues the loads
// 2 w, 2 w + 1 of either operand.
struct StripTile128 {
  const bf16_t *X, *A;     // wave-uniform: first contrast row / first anchor row of the tile
  int64_t ldx, lda, x_rows, a_rows, d;
  uint32_t ox[2], oa[2];   // per-lane byte offsets of the wave loads (relative to X / A, stage 0)
  uint32_t lx[2], la[2];   // LDS byte offsets inside a slot (wave-uniform)
  int wr, wc, lr, hk;

  __device__ __forceinline__ void setup(const bf16_t* Xc, int64_t ldx_, int64_t c0, int64_t B, const bf16_t* An,
                                        int64_t lda_, int64_t a0, int64_t rows_a, int64_t d_, int tid) {
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    wr = wave >> 1; wc = wave & 1; lr = lane & 31; hk = lane >> 5;
    X = Xc + c0 * ldx_; ldx = ldx_; x_rows = B - c0;
    A = An + a0 * lda_; lda = lda_; a_rows = rows_a - a0;
    d = d_;
    // a row of the tile that does not exist is fetched as the tile's last existing row (x_rows, a_rows >= 1): what it
    // contributes lands in elements that the guarded epilogue discards
    const int x_last = (int)(x_rows < kT ? x_rows : kT) - 1, a_last = (int)(a_rows < kT ? a_rows : kT) - 1;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int j = wave * 2 + i;                      // wave load j covers rows 16 j .. 16 j + 15 of the tile
      const int row = 16 * j + (lane >> 2);
      const int chunk = (lane & 3) ^ rt_swz(row);      // logical chunk fetched into position (lane & 3)
      ox[i] = (uint32_t)((row < x_last ? row : x_last) * (int)ldx_ + chunk * 8) * 2u;
      oa[i] = (uint32_t)((row < a_last ? row : a_last) * (int)lda_ + chunk * 8) * 2u;
      lx[i] = (uint32_t)(j * 1024);
      la[i] = (uint32_t)(kHalf + j * 1024);
    }
  }
  __device__ __forceinline__ void dma(int i, int stage, uint32_t slot) const {
    if (i < 2) dma16(X + (int64_t)stage * BK, ox[i], slot + lx[i]);
    else dma16(A + (int64_t)stage * BK, oa[i - 2], slot + la[i - 2]);
  }
  __device__ __forceinline__ void fill_guarded(int stage, char* slot, int tid) const {
    const int chunk = tid & 3;
    const int64_t k = (int64_t)stage * BK + chunk * 8;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = (tid >> 2) + 64 * i;
      u32x4 vx = {0u, 0u, 0u, 0u}, va = {0u, 0u, 0u, 0u};
      if (k < d && row < x_rows) vx = *(const u32x4*)(X + row * ldx + k);
      if (k < d && row < a_rows) va = *(const u32x4*)(A + row * lda + k);
      *(u32x4*)(slot + rt_off(row, chunk)) = vx;
      *(u32x4*)(slot + kHalf + rt_off(row, chunk)) = va;
    }
  }
  __device__ __forceinline__ bf16x8 read_a(const char* slot, int t, int kk) const {
    return *(const bf16x8*)(slot + rt_off(wr * 64 + t * 32 + lr, kk * 2 + hk));
  }
  __device__ __forceinline__ bf16x8 read_b(const char* slot, int t, int kk) const {
    return *(const bf16x8*)(slot + kHalf + rt_off(wc * 64 + t * 32 + lr, kk * 2 + hk));
  }
};

__global__ void __launch_bounds__(256, 2) k_strips_t128_bf16(StripArgs a, int nAT, int nCT) {
  __shared__ __attribute__((aligned(1024))) char ring[kSmallRing];
  // after the main loop the ring is free and holds the epilogue's scalars and cross-wave sums
  float* sk = (float*)ring;                                          // [128] log2(e)/tau of the tile's anchors
  float* sdiag = sk + kT;                                            // [128] s_pp
  float (*sred)[2][256] = (float (*)[2][256])(ring + 1024);          // [contrast half][quantity][anchor in the tile]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave >> 1, wc = wave & 1;
  const int t = blockIdx.x, per_strip = nAT * nCT;
  const int strip = t / per_strip, at = t % nAT, ct = (t / nAT) % nCT;
  const int64_t a0 = (int64_t)at * kT, c0 = (int64_t)ct * kT;
  const int S = (int)((a.d + BK - 1) / BK), S_ring = (int)(a.d / BK);
  StripTile128 T;
  // anchor rows exist up to the end of the global batch (rows beyond b belong to other workers; their results are
  // discarded like those of replaced rows)
  T.setup(a.contrasts[strip], a.ld_contrast[strip], c0, a.B, a.anchors[strip], a.ld_anchor[strip], a0, a.B - a.off, a.d,
          tid);
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  if (S_ring > 0) small_ring(acc, T, ring, lds_addr(ring), 0, S_ring);
  if (S_ring < S) small_guarded(acc, T, ring, S_ring, S - S_ring, tid);
  if (tid < kT) {
    const int64_t m = a0 + tid;
    sk[tid] = m < a.b ? a.kscale[strip][m] : 0.f;
    sdiag[tid] = m < a.b ? a.diag[m] : 0.f;
  }
  __syncthreads();
  strip_epilogue<true, 2, 2>(a, acc, sk, sdiag, sred[wr], strip, a0, c0, wr * 64, wc * 64, lane);
  __syncthreads();
  if (tid < kT) {
    const int64_t m = a0 + tid;
    if (m < a.b) {
#pragma unroll
      for (int q = 0; q < 2; ++q)
        a.sums[((size_t)(2 * strip + q) * a.nparts + ct) * a.bstride + m] = sred[0][q][tid] + sred[1][q][tid];
    }
  }
}

void launch_strips_t128_bf16(const StepCtx& c) {
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
  const int nAT = (int)((L.b + kT - 1) / kT), nCT = (int)((L.B + kT - 1) / kT);
  hipLaunchKernelGGL(k_strips_t128_bf16, dim3((unsigned)(2 * nAT * nCT)), dim3(256), 0, c.s, a, nAT, nCT);
}

// ----------------------------------------------------------------------------------------------------------------
// Contraction on 128 x 128 output tiles: C[m][n] = sum_c Efrag[m][c] X[c][n] over the contrast columns of one split.
// A operand of a stage = 4 anchor blocks x 2 column blocks of the stored strip (8 fragments of 1 KiB, copied as they
// are); B operand = 32 rows x 128 columns of X in its natural layout (256-byte rows; 16-byte piece p of row k at piece
// position p ^ ((k & 3) << 2), so that the 4 rows x 64 bytes a transposing read touches per cycle cover a bank window).
struct ContractTile128 {
  const bf16_t* Efr;       // wave-uniform: fragment (first anchor block of the tile, column block 0)
  const bf16_t* Xn;        // wave-uniform: X + n0
  int64_t ldx, n0, N, B;
  uint32_t oa[2], ob[2], la[2], lb[2];
  int wm, wn, lane;

  __device__ __forceinline__ static int swz(int k) { return (k & 3) << 2; }
  __device__ __forceinline__ void setup(const bf16_t* E, int64_t nCB, int64_t ab0, const bf16_t* X_, int64_t ldx_,
                                        int64_t n0_, int64_t N_, int64_t B_, int tid) {
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    lane = tid & 63; wm = wave >> 1; wn = wave & 1;
    Efr = E + ab0 * nCB * 512; Xn = X_ + n0_; ldx = ldx_; n0 = n0_; N = N_; B = B_;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int f = wave * 2 + i;                       // A: fragment (anchor block f / 2, column block f % 2 of the stage)
      oa[i] = (uint32_t)(((f >> 1) * (int)nCB + (f & 1)) * 512 + lane * 8) * 2u;
      la[i] = (uint32_t)(f * 1024);
      const int k = 4 * f + (lane >> 4);                // B: wave load f covers the stage's rows 4 f .. 4 f + 3
      const int piece = (lane & 15) ^ swz(k);           // logical piece fetched into position (lane & 15)
      ob[i] = (uint32_t)(k * (int)ldx_ + piece * 8) * 2u;
      lb[i] = (uint32_t)(kHalf + f * 1024);
    }
  }
  __device__ __forceinline__ const bf16_t* stage_rows(int stage) const { return Xn + (int64_t)stage * BK * ldx; }
  __device__ __forceinline__ void dma(int i, int stage, uint32_t slot) const {
    if (i < 2) dma16(Efr + (int64_t)stage * 1024, oa[i], slot + la[i]);
    else dma16(stage_rows(stage), ob[i - 2], slot + lb[i - 2]);
  }
  __device__ __forceinline__ void fill_guarded(int stage, char* slot, int tid) const {
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int f = wave * 2 + i;
      *(u32x4*)(slot + f * 1024 + lane * 16) = *(const u32x4*)((const char*)(Efr + (int64_t)stage * 1024) + oa[i]);
      const int k = 4 * f + (lane >> 4);
      const int piece = (lane & 15) ^ swz(k);
      const int64_t c = (int64_t)stage * BK + k;        // contrast column = row of X
      u32x4 v = {0u, 0u, 0u, 0u};
      if (c < B && n0 + piece * 8 < N) v = *(const u32x4*)((const char*)stage_rows(stage) + ob[i]);
      *(u32x4*)(slot + kHalf + f * 1024 + lane * 16) = v;
    }
  }
  __device__ __forceinline__ bf16x8 read_a(const char* slot, int t, int kk) const {
    return *(const bf16x8*)(slot + (((wm * 2 + t) * 2 + kk) * 1024 + lane * 16));
  }
  // slots e = 0..3 <-> rows 16 kk + 4 h + e, slots 4..7 <-> rows 16 kk + 8 + 4 h + (e - 4): two transposing reads, each
  // taking 4 rows x 16 columns per group of 16 lanes (source lane s: row s / 4, columns 4 (s % 4) ..)
  __device__ __forceinline__ bf16x8 read_b(const char* slot, int t, int kk) const {
    const int h = lane >> 5, s = lane & 15;
    const int n = wn * 64 + t * 32 + ((lane >> 4) & 1) * 16 + 4 * (s & 3);   // first of the 4 columns this lane reads
    u32x2 half2[2];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int k = 16 * kk + 8 * half + 4 * h + (s >> 2);
      const char* p = slot + kHalf + k * 256 + (((n >> 3) ^ swz(k)) << 4) + ((n & 7) << 1);
      half2[half] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)(uintptr_t)lds_addr(p)));
    }
    return join_halves(half2[0], half2[1]);
  }
};

struct T128Job {
  const bf16_t* E;     // fragment-ordered strip of this side
  const bf16_t* X;     // the matrix whose rows the strip weights (texts for side 0, images for side 1): also the rows of
                       // the diagonal terms, d_img[r] -= dcoef[r] txt[off + r]
  const float* c_own;  // c1 (side 0) / c2 (side 1)
  float* out;          // d_img / d_txt
  int64_t ldx;
};
struct T128Args {
  T128Job job[2];
  int64_t b, d, B, off, nCB;
  int tiles_m, tiles_n, nsplit, slice, stages;   // 32-deep stages per split and in all
  float* part;         // nsplit > 1: [nsplit][2][b128][d128] partial results
  int64_t b128, d128;
  const float* dcoef;
  const double* red; int nred; int version; const float* tau; float rho; float* loss; float* d_tau;
};

__global__ void __launch_bounds__(256, 2) k_contract_t128_bf16(T128Args g) {
  __shared__ __attribute__((aligned(1024))) char ring[kSmallRing];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1, lr = lane & 31, hk = lane >> 5;
  const int per_side = g.nsplit * g.tiles_m * g.tiles_n;
  const int side = (int)blockIdx.x / per_side, local = (int)blockIdx.x % per_side;
  const int split = local % g.nsplit, tile = local / g.nsplit;
  const int64_t m0 = (int64_t)(tile % g.tiles_m) * kT, n0 = (int64_t)(tile / g.tiles_m) * kT;
  const T128Job& J = g.job[side];
  const int s0 = split * g.slice;
  const int S = s0 + g.slice <= g.stages ? g.slice : g.stages - s0;      // >= 1 by construction
  ContractTile128 T;
  T.setup(J.E, g.nCB, m0 >> 5, J.X, J.ldx, n0, g.d, g.B, tid);
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // Unguarded loads of a stage take 32 whole rows of X and 128 columns from n0 on: they stay inside the matrix (B rows of
  // ldx elements, the last one of d) for the stages below `safe`; words past a row's end are the next rows', and what
  // they put into the columns from d on reaches no output.  The rest goes one stage at a time with guards.
  int64_t rows_ok = g.B;
  if (n0 + kT > g.d) rows_ok -= (n0 + kT - g.d + J.ldx - 1) / J.ldx;
  const int safe = rows_ok > 0 ? (int)(rows_ok / BK) : 0;
  const int S_ring = s0 + S <= safe ? S : (safe > s0 ? safe - s0 : 0);
  if (S_ring > 0) small_ring(acc, T, ring, lds_addr(ring), s0, S_ring);
  if (S_ring < S) small_guarded(acc, T, ring, s0 + S_ring, S - S_ring, tid);
  // accumulator (ti, tj, v) of lane (lr, hk): row m0 + 64 wm + 32 ti + 8 (v >> 2) + 4 hk + (v & 3), column n0 + 64 wn + 32 tj + lr
  if (g.nsplit == 1) {
    // the tile is complete: d[r][n] = c_own[r] C[r][n] - (c1 M g1 + c2 M g2)[r] x_partner[off + r][n]
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
      for (int tj = 0; tj < 2; ++tj) {
        const int64_t n = n0 + wn * 64 + tj * 32 + lr;
        if (n < g.d) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int64_t m = m0 + wm * 64 + ti * 32 + 8 * (v >> 2) + 4 * hk + (v & 3);
            if (m < g.b)
              J.out[m * g.d + n] = J.c_own[m] * acc[ti][tj][v] - g.dcoef[m] * bf2f(J.X[(g.off + m) * J.ldx + n]);
          }
        }
      }
    if (blockIdx.x == 0 && tid < 64) write_scalars(g.red, g.nred, g.b, g.version, g.tau, g.rho, g.loss, g.d_tau);
  } else {
    float* P = g.part + ((size_t)(split * 2 + side) * g.b128) * g.d128;   // whole 128 x 128 tiles exist in the buffer
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
      for (int tj = 0; tj < 2; ++tj) {
        const int64_t n = n0 + wn * 64 + tj * 32 + lr;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int64_t m = m0 + wm * 64 + ti * 32 + 8 * (v >> 2) + 4 * hk + (v & 3);
          P[m * g.d128 + n] = acc[ti][tj][v];
        }
      }
  }
}

// Several splits: d[r][n] = c_own[r] (sum over the splits, in their order) - dcoef[r] x_partner[off + r][n].
// A thread takes four consecutive columns of one row (d % 8 == 0 on this path).
__global__ void __launch_bounds__(256) k_finalize_t128_bf16(T128Args g) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t per_row = g.d / 4;
  const int side = blockIdx.y;
  const T128Job& J = g.job[side];
  if (q < g.b * per_row) {
    const int64_t m = q / per_row, n = (q % per_row) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < g.nsplit; ++s) {
      const float4 v = *(const float4*)(g.part + ((size_t)(s * 2 + side) * g.b128 + m) * g.d128 + n);
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

void launch_contract_t128_bf16(const StepCtx& c) {
  const Layout& L = c.L;
  T128Args g;
  memset(&g, 0, sizeof(g));
  for (int s = 0; s < 2; ++s) {
    T128Job& J = g.job[s];
    J.E = (const bf16_t*)(c.ws + L.E[s]);
    J.X = (const bf16_t*)(s == 0 ? c.buf.txt_glob : c.buf.img_glob);
    J.ldx = s == 0 ? c.cfg.ld_txt : c.cfg.ld_img;
    J.c_own = (const float*)(c.ws + (s == 0 ? L.c1 : L.c2));
    J.out = s == 0 ? c.buf.d_img : c.buf.d_txt;
  }
  g.b = L.b; g.d = L.d; g.B = L.B; g.off = L.off; g.nCB = L.ldE / 16;
  g.tiles_m = (int)((L.b + kT - 1) / kT); g.tiles_n = (int)((L.d + kT - 1) / kT);
  g.nsplit = L.nsplit; g.slice = (int)L.kslice; g.stages = (int)(L.ldE / BK);
  g.part = L.nsplit > 1 ? (float*)(c.ws + L.Opart[0]) : nullptr;
  g.b128 = (int64_t)round_up((size_t)L.b, kT); g.d128 = (int64_t)round_up((size_t)L.d, kT);
  g.dcoef = (const float*)(c.ws + L.dcoef);
  g.red = (const double*)(c.ws + L.red); g.nred = L.nstate_blocks; g.version = c.cfg.version; g.tau = c.buf.tau;
  g.rho = c.cfg.rho; g.loss = c.buf.loss; g.d_tau = c.buf.d_tau;
  const unsigned grid = 2u * (unsigned)(g.nsplit * g.tiles_m * g.tiles_n);
  hipLaunchKernelGGL(k_contract_t128_bf16, dim3(grid), dim3(256), 0, c.s, g);
  if (g.nsplit > 1) {
    const int64_t quads = L.b * (L.d / 4);
    hipLaunchKernelGGL(k_finalize_t128_bf16, dim3((unsigned)((quads + 255) / 256), 2), dim3(256), 0, c.s, g);
  }
}

}  // namespace fc
