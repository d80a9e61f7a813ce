// bf16 MFMA kernels of the FCCO step for gfx950 (wave64, v_mfma_f32_32x32x16_bf16).
//
//  k_strips_edge_bf16  the strip tiles with a ragged edge (whole tiles: k_strips_bf16 in kernels_strips.hip):
//                   S^T tile = contrasts x anchors^T (256 x 256 per workgroup), then in registers
//                   l = exp((s - s_ii)/tau) (Sec. 3), per-anchor sums of l and of (s - s_ii) l (Proc. 1 and the
//                   nabla_3 l sums of Eqs. 8-10), and l rounded to bf16 stored as the operand of the gradient
//                   contraction.  The similarity matrix itself never reaches memory.  Anchors run along lanes, so
//                   the sums are lane-local and every store is a contiguous 1 KiB per wavefront.
//  k_fold_bf16      the local contrast-side term of Eqs. 3 / 5 / 7: c_other[q] l_other(q, p_r) / c_own[r] is added to
//                   the strip element (r, off + q), which weights the same row of X, so that one contraction yields
//                   sum_j l(r,j) x_j + (1/c_r) sum_q c_q l(q,p_r) x_q.
//  k_contract_bf16  C[r][n] = sum_c Efrag[r][c] X[c][n] over the contrast columns, split over c into fp32
//                   partial results (Eqs. 2/4/6 plus the local part of Eqs. 3/5/7).
//
// Stored exp strips ("Efrag"): for anchor block ab = r / 32 and column block cb = c / 16 one 1 KiB fragment, laid out
// exactly as the A operand of the 32x32x16 MFMA: lane L = (r % 32) + 32 h holds 8 bf16, slot e <-> column
// 16 cb + 8 (e / 4) + 4 h + (e % 4).  The same slot order is used for the rows of X in the contraction, so the
// permutation cancels.  Columns [0, ldE) are contrasts (global rows, zero beyond B).
//
// MFMA layout facts used (32x32x16, wave64): lane l supplies row/column (l & 31) of its operand and 8 contraction
// slots selected by (l >> 5); accumulator register v of lane l is D[8 (v >> 2) + 4 (l >> 5) + (v & 3)][l & 31].
//
// Main loop of the contraction (whole tiles): a ring of five 32 KiB LDS slots, each one 32-deep stage of both operands,
// filled by global_load_lds_dwordx4 (no VGPR staging) four stages ahead; one barrier per stage; LDS operand reads of
// the next 16-deep step are issued between the MFMAs of the current one.  Tiles that touch a ragged edge use guarded
// register loads into the same LDS images, one stage at a time.
#include "mfma_common.hpp"
#include "state_common.hpp"

namespace fc {

// ----------------------------------------------------------------------------------------------------------------
// Operand sources.  Each describes, for one workgroup tile, how a stage is brought into an LDS slot (dma: 8 wave
// loads per thread and stage, indices 0..3 = A operand, 4..7 = B operand; fill_guarded: the same image through
// registers with zero fill) and how a wave reads its MFMA operands from the slot.
//
// Strip kernel: both operands are K-contiguous row tiles.  A operand = 256 contrast rows, B operand = 256 anchor rows.
struct StripTile {
  const bf16_t *X, *A;   // wave-uniform: first contrast row / first anchor row of the tile
  int64_t ldx, lda;
  uint32_t oa[4], ob[4]; // per-lane byte offsets of the 4 + 4 wave loads of a stage (relative to X / A, stage 0)
  uint32_t la[4], lb[4]; // LDS byte offsets inside a slot (wave-uniform)
  int wr, wc_, lr, hk;   // wave row/col block, lane split
  int64_t x_rows, a_rows, d;   // valid rows below X / A, contraction length (guarded path)

  // Xc / An: row 0 of the contrast / anchor matrix; c0 / a0: first row of the tile; B / b: rows of the matrices.
  __device__ __forceinline__ void setup(const bf16_t* Xc, int64_t ldx_, int64_t c0, int64_t B, const bf16_t* An,
                                        int64_t lda_, int64_t a0, int64_t b, int64_t d_, int tid) {
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;   // wave-uniform, kept in SGPRs
    wr = wave >> 1; wc_ = wave & 1; lr = lane & 31; hk = lane >> 5;
    X = Xc + c0 * ldx_; ldx = ldx_; x_rows = B - c0;
    A = An + a0 * lda_; lda = lda_; a_rows = b - a0;
    d = d_;
    // The unguarded wave loads fetch, for a row of the tile that does not exist, the tile's last existing row instead
    // (x_rows, a_rows >= 1): whatever such a row contributes lands in elements that the guarded epilogue discards.
    const int x_last = (int)(x_rows < 256 ? x_rows : 256) - 1, a_last = (int)(a_rows < 256 ? a_rows : 256) - 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = wave * 4 + i;                      // wave load j covers rows 16 j .. 16 j + 15 of the tile
      const int row = 16 * j + (lane >> 2);
      const int chunk = (lane & 3) ^ rt_swz(row);      // logical chunk fetched into position (lane & 3)
      oa[i] = (uint32_t)((row < x_last ? row : x_last) * (int)ldx_ + chunk * 8) * 2u;
      ob[i] = (uint32_t)((row < a_last ? row : a_last) * (int)lda_ + chunk * 8) * 2u;
      la[i] = (uint32_t)(j * 1024);
      lb[i] = (uint32_t)(kOpBytes + j * 1024);
    }
  }
  __device__ __forceinline__ void dma(int i, int stage, uint32_t slot) const {
    if (i < 4) dma16(X + (int64_t)stage * BK, oa[i], slot + la[i]);
    else dma16(A + (int64_t)stage * BK, ob[i - 4], slot + lb[i - 4]);
  }
  __device__ __forceinline__ void fill_guarded(int stage, char* slot, int tid) const {
    const int chunk = tid & 3;
    const int64_t k = (int64_t)stage * BK + chunk * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (tid >> 2) + 64 * i;
      u32x4 va = {0u, 0u, 0u, 0u}, vb = {0u, 0u, 0u, 0u};
      if (k < d && row < x_rows) va = *(const u32x4*)(X + row * ldx + k);
      if (k < d && row < a_rows) vb = *(const u32x4*)(A + row * lda + k);
      *(u32x4*)(slot + rt_off(row, chunk)) = va;
      *(u32x4*)(slot + kOpBytes + rt_off(row, chunk)) = vb;
    }
  }
  __device__ __forceinline__ bf16x8 read_a(const char* slot, int t, int kk) const {
    return *(const bf16x8*)(slot + rt_off(wr * 128 + t * 32 + lr, kk * 2 + hk));
  }
  __device__ __forceinline__ bf16x8 read_b(const char* slot, int t, int kk) const {
    return *(const bf16x8*)(slot + kOpBytes + rt_off(wc_ * 128 + t * 32 + lr, kk * 2 + hk));
  }
  __device__ __forceinline__ u32x2 read_b_half(const char* slot, int t, int kk, int half) const {   // for the ring loop
    return *(const u32x2*)(slot + kOpBytes + rt_off(wc_ * 128 + t * 32 + lr, kk * 2 + hk) + 8 * half);
  }
};

// Contraction kernel: A operand = 8 anchor blocks x 2 column blocks of Efrag per stage (fragments are copied as they
// are), B operand = 32 rows x 256 columns of X in its natural layout, read with transposing LDS reads.
struct ContractTile {
  const bf16_t* Efr;       // wave-uniform: fragment (ab0, column block 0) of the strip
  const bf16_t* Xn;        // wave-uniform: X + n0
  int64_t ldx;
  uint32_t oa[4], ob[4];   // per-lane byte offsets of the wave loads (A: relative to Efr; B: relative to row 0 of a stage)
  uint32_t la[4], lb[4];
  int wm, wn, lane;
  int64_t n0, N, B;   // guarded path

  __device__ __forceinline__ void setup(const bf16_t* E, int64_t nCB, int64_t ab0, const bf16_t* X_, int64_t ldx_,
                                        int64_t n0_, int64_t N_, int64_t B_, int tid) {
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in SGPRs
    lane = tid & 63; wm = wave >> 1; wn = wave & 1;
    Efr = E + ab0 * nCB * 512; Xn = X_ + n0_; ldx = ldx_;
    n0 = n0_; N = N_; B = B_;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int f = wave * 4 + i;                       // fragment f = 2 * (anchor block) + (column block in stage)
      oa[i] = (uint32_t)(((f >> 1) * (int)nCB + (f & 1)) * 512 + lane * 8) * 2u;
      la[i] = (uint32_t)(f * 1024);
      const int k = 2 * f + (lane >> 5);                // wave load f covers stage rows 2 f, 2 f + 1
      const int piece = (lane & 31) ^ nt_swz(k);        // logical piece fetched into position (lane & 31)
      ob[i] = (uint32_t)(k * (int)ldx_ + piece * 8) * 2u;
      lb[i] = (uint32_t)(kOpBytes + f * 1024);
    }
  }
  __device__ __forceinline__ const bf16_t* stage_rows(int stage) const {   // X row of stage row 0, plus n0
    return Xn + (int64_t)stage * BK * ldx;
  }
  __device__ __forceinline__ void dma(int i, int stage, uint32_t slot) const {
    if (i < 4) dma16(Efr + (int64_t)stage * 1024, oa[i], slot + la[i]);
    else dma16(stage_rows(stage), ob[i - 4], slot + lb[i - 4]);
  }
  __device__ __forceinline__ void fill_guarded(int stage, char* slot, int tid) const {
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int f = wave * 4 + i;
      *(u32x4*)(slot + f * 1024 + lane * 16) = *(const u32x4*)((const char*)(Efr + (int64_t)stage * 1024) + oa[i]);
      const int k = 2 * f + (lane >> 5);
      const int piece = (lane & 31) ^ nt_swz(k);
      const int64_t c = (int64_t)stage * BK + k;        // contrast column = row of X
      const bool ok = c < B && (n0 + piece * 8 < N);
      u32x4 v = {0u, 0u, 0u, 0u};
      if (ok) v = *(const u32x4*)((const char*)stage_rows(stage) + ob[i]);
      *(u32x4*)(slot + kOpBytes + f * 1024 + lane * 16) = v;
    }
  }
  __device__ __forceinline__ bf16x8 read_a(const char* slot, int t, int kk) const {
    return *(const bf16x8*)(slot + (((wm * 4 + t) * 2 + kk) * 1024 + lane * 16));
  }
  // slots e = 0..3 <-> rows 16 kk + 4 h + e, slots 4..7 <-> rows 16 kk + 8 + 4 h + (e - 4): two transposing reads
  // (half 0 / 1), each taking 4 rows x 16 columns per group of 16 lanes (source lane s: row s / 4, columns 4 (s % 4) ..).
  __device__ __forceinline__ u32x2 read_b_half(const char* slot, int t, int kk, int half) const {
    const int h = lane >> 5, s = lane & 15;
    const int n = wn * 128 + t * 32 + ((lane >> 4) & 1) * 16 + 4 * (s & 3);   // first of 4 columns read by this lane
    const int k = 16 * kk + 8 * half + 4 * h + (s >> 2);
    const char* base = slot + kOpBytes + ((n & 7) << 1);
    lds_v4s* p = (lds_v4s*)(uintptr_t)lds_addr(base + nt_off(k, n >> 3));
    return __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16(p));
  }
  __device__ __forceinline__ bf16x8 read_b(const char* slot, int t, int kk) const {
    return join_halves(read_b_half(slot, t, kk, 0), read_b_half(slot, t, kk, 1));
  }
};

#define FC_MM(ti, tj, A_, B_) acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A_[ti], B_[tj], acc[ti][tj], 0, 0, 0)
// The same with the B operand held as the two halves that the transposing reads deliver.
#define FC_MMH(ti, tj, A_, BL_, BH_) \
  acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A_[ti], join_halves(BL_[tj], BH_[tj]), acc[ti][tj], 0, 0, 0)

// One 32-deep stage of the ring: 16 MFMAs on the operands already in registers while the operands of the second
// 16-deep step are read; then "stage s+1 has landed" (vmcnt) + barrier, which also retires the slot of stage s-1; then
// 16 MFMAs while the first operands of stage s+1 are read.  A lone wavefront per SIMD issues in order: whatever sits
// between two MFMAs delays the second one once it takes longer than the first one runs (32 cycles), so the 4 + 8 LDS
// reads and the 4 wave loads of a half stage are dealt out ONE per MFMA.  The 8 wave loads of a stage x are spread
// over a whole stage time, so that the load unit sees a steady trickle instead of a burst: the four A-operand loads
// in the second half of stage x-4 (DMAA, into the slot just retired), the four B-operand loads in the first half of
// stage x-3 (DMAB).  cur / nxt / prv / pp: byte offsets of the slots of stages s, s+1, s-1, s-2 in a ring of five.
// WAIT: loads that may stay in flight at the barrier (those of stages s+2 and s+3): 16, 8 or 0.
// The barrier is the bare instruction: the LDS reads of the first half need not have returned (their slot is written
// again only after the NEXT stage's barrier, and their consumers wait for them by themselves), so there is no
// "wait for all LDS traffic" in front of it as __syncthreads() would put.
// One MFMA followed by one other statement.
#define FC_SLOT(ti, tj, AP, BLP, BHP, STMT) FC_MMH(ti, tj, AP, BLP, BHP); FC_PIN(); STMT; FC_PIN();
// 16 MFMAs on operand set (AP, BLP, BHP) while the set (AQ, BLQ, BHQ) is read from slot `src`, step KQ, in the order in
// which the following half stage consumes it (its MFMAs run over tj fastest), and D0 .. D3 are issued.
#define FC_HALF(AP, BLP, BHP, AQ, BLQ, BHQ, src, KQ, RD, D0, D1, D2, D3)                                            \
    FC_SLOT(0, 0, AP, BLP, BHP, if (RD) BLQ[0] = T.read_b_half(src, 0, KQ, 0))                                      \
    FC_SLOT(0, 1, AP, BLP, BHP, if (RD) BHQ[0] = T.read_b_half(src, 0, KQ, 1))                                      \
    FC_SLOT(0, 2, AP, BLP, BHP, if (RD) AQ[0] = T.read_a(src, 0, KQ))                                               \
    FC_SLOT(0, 3, AP, BLP, BHP, D0)                                                                                 \
    FC_SLOT(1, 0, AP, BLP, BHP, if (RD) BLQ[1] = T.read_b_half(src, 1, KQ, 0))                                      \
    FC_SLOT(1, 1, AP, BLP, BHP, if (RD) BHQ[1] = T.read_b_half(src, 1, KQ, 1))                                      \
    FC_SLOT(1, 2, AP, BLP, BHP, if (RD) BLQ[2] = T.read_b_half(src, 2, KQ, 0))                                      \
    FC_SLOT(1, 3, AP, BLP, BHP, D1)                                                                                 \
    FC_SLOT(2, 0, AP, BLP, BHP, if (RD) BHQ[2] = T.read_b_half(src, 2, KQ, 1))                                      \
    FC_SLOT(2, 1, AP, BLP, BHP, if (RD) BLQ[3] = T.read_b_half(src, 3, KQ, 0))                                      \
    FC_SLOT(2, 2, AP, BLP, BHP, if (RD) BHQ[3] = T.read_b_half(src, 3, KQ, 1))                                      \
    FC_SLOT(2, 3, AP, BLP, BHP, D2)                                                                                 \
    FC_SLOT(3, 0, AP, BLP, BHP, if (RD) AQ[1] = T.read_a(src, 1, KQ))                                               \
    FC_SLOT(3, 1, AP, BLP, BHP, if (RD) AQ[2] = T.read_a(src, 2, KQ))                                               \
    FC_SLOT(3, 2, AP, BLP, BHP, if (RD) AQ[3] = T.read_a(src, 3, KQ))                                               \
    FC_SLOT(3, 3, AP, BLP, BHP, D3)
#define FC_STAGE(T, MORE, DMAB, DMAA, WAIT)                                                                         \
  {                                                                                                                 \
    const char* sl = ring + cur;                                                                                    \
    const uint32_t bslot = ring_addr + pp;                                                                          \
    FC_HALF(a0, bl0, bh0, a1, bl1, bh1, sl, 1, true, if (DMAB) T.dma(4, s0 + s + 3, bslot),                         \
            if (DMAB) T.dma(5, s0 + s + 3, bslot), if (DMAB) T.dma(6, s0 + s + 3, bslot),                           \
            if (DMAB) T.dma(7, s0 + s + 3, bslot))                                                                  \
    if (WAIT == 16) FC_WAIT_VMCNT16(); else if (WAIT == 8) FC_WAIT_VMCNT8(); else FC_WAIT_VMCNT0();                 \
    __builtin_amdgcn_s_barrier();                                                                                   \
    FC_PIN();                                                                                                       \
    const char* nx = ring + nxt;                                                                                    \
    const uint32_t aslot = ring_addr + prv;                                                                         \
    FC_HALF(a1, bl1, bh1, a0, bl0, bh0, nx, 0, MORE, if (DMAA) T.dma(0, s0 + s + 4, aslot),                         \
            if (DMAA) T.dma(1, s0 + s + 4, aslot), if (DMAA) T.dma(2, s0 + s + 4, aslot),                           \
            if (DMAA) T.dma(3, s0 + s + 4, aslot))                                                                  \
    pp = prv; prv = cur; cur = nxt;                                                                                 \
    nxt = (nxt + (uint32_t)kStageBytes == (uint32_t)kRingBytes) ? 0u : nxt + (uint32_t)kStageBytes;                 \
    ++s;                                                                                                            \
  }

// Issue the wave loads of the first stages [s0, ...) of a tile into ring slots 0 .. 3: stages 0 .. 2 whole and of
// stage 3 the A-operand half (its B-operand half follows in the first half of stage 0, as for every later stage);
// tiles of at most 4 stages are requested whole.
template <typename Tile>
__device__ __forceinline__ void ring_prologue(const Tile& T, uint32_t ring_addr, int s0, int S) {
#pragma unroll
  for (int p = 0; p < 4; ++p)
    if (p < S) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (p < 3 || i < 4 || S == 4) T.dma(i, s0 + p, ring_addr + p * kStageBytes);
    }
}

// acc += (A operand tile) x (B operand tile)^T over stages [s0, s0 + S); the prologue must have been issued, and
// nothing else may have touched the ring since.  Vector memory operations complete in order, so every wait names
// the number of younger loads that may stay in flight.  On return no wave reads the ring any more.
template <typename Tile>
__device__ __forceinline__ void ring_mainloop(f32x16 (&acc)[4][4], const Tile& T, char* ring, uint32_t ring_addr,
                                              int s0, int S) {
  // stage 0 has landed; stages 1, 2 and (half or all of) 3 may be in flight
  if (S >= 5) FC_WAIT_VMCNT20(); else if (S == 4) FC_WAIT_VMCNT24(); else FC_WAIT_VMCNT0();
  __syncthreads();
  bf16x8 a0[4], a1[4];
  u32x2 bl0[4], bh0[4], bl1[4], bh1[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    a0[t] = T.read_a(ring, t, 0);
    bl0[t] = T.read_b_half(ring, t, 0, 0);
    bh0[t] = T.read_b_half(ring, t, 0, 1);
  }
  uint32_t cur = 0u, nxt = (uint32_t)kStageBytes, prv = 4u * (uint32_t)kStageBytes, pp = 3u * (uint32_t)kStageBytes;
  int s = 0;
  while (s + 4 < S) FC_STAGE(T, true, true, true, 16)               // s = 0 .. S-5
  while (s + 4 == S && S >= 5) FC_STAGE(T, true, true, false, 16)   // s = S-4: the last B-operand loads
  while (s + 3 < S) FC_STAGE(T, true, false, false, 16)             // S == 4 only
  while (s + 2 < S) FC_STAGE(T, true, false, false, 8)
  while (s + 1 < S) FC_STAGE(T, true, false, false, 0)
  FC_STAGE(T, false, false, false, 0)
  __syncthreads();
}

// Same contraction for tiles with a ragged edge: one stage at a time through registers, zero fill outside.
template <typename Tile>
__device__ __forceinline__ void guarded_mainloop(f32x16 (&acc)[4][4], const Tile& T, char* ring, int s0, int S,
                                                 int tid) {
  bf16x8 a[4], bq[4];
  for (int s = 0; s < S; ++s) {
    __syncthreads();
    T.fill_guarded(s0 + s, ring, tid);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
      for (int t = 0; t < 4; ++t) { a[t] = T.read_a(ring, t, kk); bq[t] = T.read_b(ring, t, kk); }
#pragma unroll
      for (int ti = 0; ti < 4; ++ti)
#pragma unroll
        for (int tj = 0; tj < 4; ++tj) FC_MM(ti, tj, a, bq);
    }
  }
  __syncthreads();
}

// Second pass over the accumulators of one wave of an edge tile when the whole batch is local (b == B, off == 0; the
// first pass is strip_epilogue with the image anchors' row parameters).  Every element s_pj also yields
// f = l2(j, p) = 2^((s - s_jj) log2(e)/tau2_j) of the TEXT anchor j = its contrast column; f goes to the second strip
// F[0] in the form of E[0] and is summed over the wave's anchors.  scol_k / scol_d: log2(e)/tau2_j and s_jj of the
// tile's 256 columns (0 beyond the batch); sredc_w[quantity][column inside the tile] receives the wave's column sums
// of f and of (s - s_jj) f.  Zero outside the batch and on the diagonal j == p (B_{j-} excludes j).  Accumulator
// (ti, tj, v) of lane (lr, hk): contrast c0 + cw + 32 ti + 8 (v >> 2) + 4 hk + (v & 3), anchor a0 + aw + 32 tj + lr.
__device__ __forceinline__ void edge_epilogue_cols(const StripArgs& a, f32x16 (&acc)[4][4], const float* scol_k,
                                                   const float* scol_d, float (*sredc_w)[256], int64_t a0, int64_t c0,
                                                   int cw, int aw, int lane) {
  const int lr = lane & 31, hk = lane >> 5;
  const int B = (int)a.B, b = (int)a.b;
  bf16_t* __restrict__ F = a.F[0];
  const int64_t ab0 = (a0 + aw) >> 5, cb0 = (c0 + cw) >> 4;
#pragma unroll
  for (int ti = 0; ti < 4; ++ti) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {            // the 16-byte fragment store j holds the groups g = 2 j, 2 j + 1
      const int cl = cw + ti * 32 + 16 * j + 4 * hk;     // column inside the tile of (g = 2 j, q = 0)
      const float4 k0 = *(const float4*)(scol_k + cl), k1 = *(const float4*)(scol_k + cl + 8);
      const float4 d0 = *(const float4*)(scol_d + cl), d1 = *(const float4*)(scol_d + cl + 8);
      const float ck[8] = {k0.x, k0.y, k0.z, k0.w, k1.x, k1.y, k1.z, k1.w};
      const float cdk[8] = {d0.x * k0.x, d0.y * k0.y, d0.z * k0.z, d0.w * k0.w,
                            d1.x * k1.x, d1.y * k1.y, d1.z * k1.z, d1.w * k1.w};
      float cs[16];                          // column sums of this lane: f of 8 columns, then t f of 8 columns
#pragma unroll
      for (int i = 0; i < 16; ++i) cs[i] = 0.f;
      const int64_t cb = cb0 + 2 * ti + j;
#pragma unroll
      for (int tj = 0; tj < 4; ++tj) {
        const int anchor = (int)a0 + aw + tj * 32 + lr;
        uint32_t pf[4];
#pragma unroll
        for (int gi = 0; gi < 2; ++gi) {
          const int g = 2 * j + gi;
          float t2[4], f[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) t2[q] = fmaf(acc_read(acc[ti][tj][4 * g + q]), ck[4 * gi + q], -cdk[4 * gi + q]);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int c = (int)c0 + cl + 8 * gi + q;
            const bool ok = (c < B) && (anchor < b) && (c != anchor);
            f[q] = ok ? __builtin_amdgcn_exp2f(t2[q]) : 0.f;
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            cs[4 * gi + q] += f[q];
            cs[8 + 4 * gi + q] = fmaf(t2[q], f[q], cs[8 + 4 * gi + q]);
          }
          pf[2 * gi] = pack_bf16x2(f[0], f[1]);
          pf[2 * gi + 1] = pack_bf16x2(f[2], f[3]);
          FC_PIN();
        }
        const u32x4 wf = {pf[0], pf[1], pf[2], pf[3]};
        if (16 * cb < a.ldE) *(u32x4*)(F + (((ab0 + tj) * a.nCBF + cb) * 64 + lane) * 8) = wf;
        FC_PIN();
      }
      // divide the second quantity by log2(e)/tau_j while each lane still knows its columns, then sum over the lanes
#pragma unroll
      for (int i = 0; i < 8; ++i) cs[8 + i] = ck[i] > 0.f ? cs[8 + i] * __builtin_amdgcn_rcpf(ck[i]) : 0.f;
      lanes32_sum(cs, lane);
      if ((lr & 1) == 0) {
        const int v = lr >> 1, gi = (v >> 2) & 1, q = v & 3;     // value v = 8 quantity + 4 gi + q
        sredc_w[v >> 3][cl + 8 * gi + q] = cs[0];
      }
      FC_PIN();
    }
  }
}

// Tiles with a ragged edge (anchors, contrasts or width not a multiple of the tile): one workgroup per tile, guarded
// epilogue.  The stages that lie wholly inside the width run through the ring of the contraction kernel with unguarded
// direct-to-LDS loads (rows that do not exist are replaced by the tile's last existing row, see StripTile::setup); a
// ragged last stage goes through registers with zero fill.  When the whole batch is local and the similarity matrix is
// formed once (StripArgs::square) the tile also yields the text anchors' exponentials and their sums down the columns.
// After the main loop the ring is free and holds the epilogue's scalars and cross-wave sums.
__global__ void __launch_bounds__(256) k_strips_edge_bf16(StripArgs a) {
  __shared__ __attribute__((aligned(1024))) char ring[kRingBytes];
  float* sk = (float*)ring;                                          // [256] log2(e)/tau of the tile's anchors
  float* sdiag = sk + 256;                                           // [256] s_pp
  float (*sred)[2][256] = (float (*)[2][256])(ring + 2048);          // [contrast half][quantity][anchor]
  float* scol = (float*)(ring + 6144);                               // square: [2][256] log2(e)/tau2_j, s_jj of the columns
  float (*sredc)[2][256] = (float (*)[2][256])(ring + 8192);         // square: [anchor half][quantity][column]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int t = blockIdx.x;
  const int per_strip = a.nAT * a.nCT;
  const int strip = t / per_strip, at = t % a.nAT, ct = (t / a.nAT) % a.nCT;
  const int64_t a0 = strip_anchor_first(a, at, a.square), c0 = (int64_t)ct * 256;
  if (strip_tile_is_interior(a, a0, c0)) return;
  const int S = (int)((a.d + BK - 1) / BK), S_ring = (int)(a.d / BK);
  StripTile T;
  T.setup(a.contrasts[strip], a.ld_contrast[strip], c0, a.B, a.anchors[strip], a.ld_anchor[strip], a0, a.b, a.d, tid);
  f32x16 acc[4][4];
  zero_acc(acc);
  if (S_ring > 0) {
    ring_prologue(T, lds_addr(ring), 0, S_ring);
    ring_mainloop(acc, T, ring, lds_addr(ring), 0, S_ring);
  }
  if (S_ring < S) guarded_mainloop(acc, T, ring, S_ring, S - S_ring, tid);
  {
    const int64_t m = a0 + tid;
    sk[tid] = m < a.b ? a.kscale[strip][m] : 0.f;
    sdiag[tid] = m < a.b ? a.diag[m] : 0.f;
    if (a.square) {                    // off == 0: text anchor j is global row j
      const int64_t j = c0 + tid;
      scol[tid] = j < a.b ? a.kscale[1][j] : 0.f;
      scol[256 + tid] = j < a.b ? a.diag[j] : 0.f;
    }
  }
  __syncthreads();
  strip_epilogue<true, 4, 4>(a, acc, sk, sdiag, sred[wr], strip, a0, c0, wr * 128, wc * 128, lane);
  if (a.square) edge_epilogue_cols(a, acc, scol, scol + 256, sredc[wc], a0, c0, wr * 128, wc * 128, lane);
  __syncthreads();
  const int64_t m = a0 + tid;
  if (m < a.b) {
#pragma unroll
    for (int q = 0; q < 2; ++q)
      a.sums[((size_t)(2 * strip + q) * a.nparts + ct) * a.bstride + m] = sred[0][q][tid] + sred[1][q][tid];
  }
  // the text anchors' sums (quantities 2, 3): partial number = the anchor tile, position = the column
  const int64_t j = c0 + tid;
  if (a.square && j < a.b) {
#pragma unroll
    for (int q = 0; q < 2; ++q)
      a.sums[((size_t)(2 + q) * a.nparts + at) * a.bstride + j] = sredc[0][q][tid] + sredc[1][q][tid];
  }
}

static void make_strip_args(const StepCtx& c, StripArgs* out, bool* any_interior, bool* any_edge);

void launch_strips_bf16(const StepCtx& c) {
  StripArgs a;
  bool any_interior, any_edge;
  make_strip_args(c, &a, &any_interior, &any_edge);
  if (any_interior) launch_strips_interior_bf16(a, c.s);
  if (any_edge) hipLaunchKernelGGL(k_strips_edge_bf16, dim3((unsigned)a.ntiles), dim3(256), 0, c.s, a);
}

// Measurement: the whole-tile strip kernel of the plain mode with parts compiled out and cycle counters (kAbl* in
// kernels_strips.hip).  Only for layouts in which every tile is whole and the mode is the plain one.
bool launch_strips_measure(const StepCtx& c, int ablation, uint64_t* cycles) {
  StripArgs a;
  bool any_interior, any_edge;
  make_strip_args(c, &a, &any_interior, &any_edge);
  if (!any_interior || any_edge || a.square || a.colp) return false;
  a.cycles = cycles;
  return launch_strips_measure_bf16(a, ablation, c.s);
}

static void make_strip_args(const StepCtx& c, StripArgs* out, bool* any_interior_out, bool* any_edge_out) {
  const Layout& L = c.L;
  const bf16_t* img = (const bf16_t*)c.buf.img_glob;
  const bf16_t* txt = (const bf16_t*)c.buf.txt_glob;
  StripArgs& a = *out;
  a.cycles = nullptr;
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
  a.nAT = (int)((L.b + 255) / 256);
  a.nCT = (int)((L.B + 255) / 256);
  a.square = L.square;
  a.ntiles = (L.square ? 1 : 2) * a.nAT * a.nCT;
  a.colp = L.gathered ? (const float*)(c.ws + L.colp) : nullptr;
  a.F[0] = (L.gathered || L.square) ? (bf16_t*)(c.ws + L.F[0]) : nullptr;
  a.F[1] = L.gathered ? (bf16_t*)(c.ws + L.F[1]) : nullptr;
  a.nCBF = L.ldE / 16;
  const bool d_ok = L.d % 64 == 0 && L.d >= 128;
  bool any_interior = false, any_edge = !d_ok || (L.B % 256);
  for (int at = 0; at < a.nAT; ++at) {
    const bool in = strip_tile_is_interior(a, strip_anchor_first(a, at, a.square), 0);
    any_interior |= in && L.B >= 256;
    any_edge |= !in;
  }
  *any_interior_out = any_interior;
  *any_edge_out = any_edge;
}

// ----------------------------------------------------------------------------------------------------------------
// Local contrast-side term of Eqs. 3 / 5 / 7, folded into the stored strips.  For two local anchors r, q the image
// row of r receives c1_r l1(r, p_q) txt_{p_q} (anchor side, Eq. 2) and c2_q l2(q, p_r) txt_{p_q} (contrast side of
// the text anchor q, Eq. 3): the same row of X with the weight w = c1_r l1(r, p_q) + c2_q l2(q, p_r), which is also
// the weight of img_{p_r} in the text gradient of q.  The strips hold l1(r, .) and l2(q, .) at exactly these
// columns, so the block (rb, qb) replaces E0[r][off + q] by w / c1_r and E1[q][off + r] by w / c2_q (the contraction's
// result is multiplied by the row's own coefficient afterwards) and one contraction per side yields both terms.
//
// A 64 x 64 window of a strip (rows row0 .., columns col0 ..) is read as whole 16-byte fragment chunks and laid out
// as tile[row][column] in LDS; col0 need not be a multiple of 16, so up to 5 column blocks are touched.
__device__ __forceinline__ void fold_load(const bf16_t* __restrict__ E, int64_t nCB, int64_t row0, int64_t col0,
                                          int64_t rows, float (*tile)[65]) {
  const int64_t cb_first = col0 >> 4, cb_last = (col0 + 63) >> 4;
  for (int i = threadIdx.x; i < 64 * 10; i += 256) {
    const int rl = i & 63, ch = i >> 6;
    const int64_t cb = cb_first + (ch >> 1);
    const int h = ch & 1;
    const int64_t row = row0 + rl;
    if (cb > cb_last || cb >= nCB || row >= rows) continue;
    const uint4 raw = *(const uint4*)(E + (((row >> 5) * nCB + cb) * 64 + (row & 31) + 32 * h) * 8);
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int64_t cl = 16 * cb + 8 * (e >> 2) + 4 * h + (e & 3) - col0;
      const uint32_t bits = (e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16);
      if (cl >= 0 && cl < 64) tile[rl][cl] = __uint_as_float(bits);
    }
  }
}
// The way back: a chunk that lies wholly inside the window's valid columns is stored as 16 bytes, any other chunk
// element by element (its remaining elements belong to a neighbouring block, which may be storing them right now).
__device__ __forceinline__ void fold_store(bf16_t* __restrict__ E, int64_t nCB, int64_t row0, int64_t col0,
                                           int64_t rows, int cols, float (*tile)[65]) {
  const int64_t cb_first = col0 >> 4, cb_last = (col0 + 63) >> 4;
  for (int i = threadIdx.x; i < 64 * 10; i += 256) {
    const int rl = i & 63, ch = i >> 6;
    const int64_t cb = cb_first + (ch >> 1);
    const int h = ch & 1;
    const int64_t row = row0 + rl;
    if (cb > cb_last || row >= rows) continue;
    bf16_t* dst = E + (((row >> 5) * nCB + cb) * 64 + (row & 31) + 32 * h) * 8;
    const int64_t cl_lo = 16 * cb + 4 * h - col0, cl_hi = cl_lo + 8;   // slots 0..3 and 4..7
    if (cl_lo >= 0 && cl_hi + 3 < cols) {
      const u32x4 w = {pack_bf16x2(tile[rl][cl_lo], tile[rl][cl_lo + 1]), pack_bf16x2(tile[rl][cl_lo + 2], tile[rl][cl_lo + 3]),
                       pack_bf16x2(tile[rl][cl_hi], tile[rl][cl_hi + 1]), pack_bf16x2(tile[rl][cl_hi + 2], tile[rl][cl_hi + 3])};
      *(u32x4*)dst = w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int64_t cl = (e < 4 ? cl_lo : cl_hi) + (e & 3);
        if (cl >= 0 && cl < cols) dst[e] = f2bf(tile[rl][cl]);
      }
    }
  }
}

// The state phase inside the fold kernels (Layout::fused_state; otherwise k_state has run and the coefficients are
// read).  A block needs the coefficients c1 of its 64 rows r0 .. and c2 of its 64 rows q0 ..: it sums the strip
// phase's partial sums of those anchors (4 threads per anchor and side, then LDS, always in the same order, so every
// block that forms an anchor's coefficient gets the same bits) and applies Eq. 1 to the u^t that the prep kernel
// gathered.  Blocks on the diagonal (r0 == q0) have both sides of their anchors and finish them: scatter of u^{t+1},
// coefficients and diagonal factor for the later phases, Eq. 9, the scalars' partial sums.
// sc: c1_r, c2_q, 1 / c1_r, 1 / c2_q; rows at or beyond b get 1.
struct FoldState {
  float part[4][4][64];   // [quantity][part lane][anchor]
};
__device__ __forceinline__ void fold_coefficients(const StateArgs& a, int64_t r0, int64_t q0, float (*sc)[64],
                                                  FoldState& fs) {
  const int al = threadIdx.x & 63, pl = threadIdx.x >> 6;
  const bool diag = r0 == q0;
  const int side = threadIdx.x >> 6;                       // threads 0..63: side 0 of row r0 + al, 64..127: side 1 of q0 + al
  const int64_t m = (side == 0 ? r0 : q0) + al;
  if (!a.fused) {                                          // the state kernel has left the coefficients
    if (threadIdx.x < 128) {
      const float c = m < a.b ? (side == 0 ? a.c1 : a.c2)[m] : 1.0f;
      sc[side][al] = c;
      sc[2 + side][al] = 1.0f / c;
    }
    return;
  }
  // per-anchor inputs of the threads that form the coefficients below, requested before the sums
  float uo = 0.f, tt = 0.07f, uo_other = 0.f, tt_other = 0.07f;
  if (threadIdx.x < 128 && m < a.b) {
    uo = (side == 0 ? a.uold1 : a.uold2)[m];
    tt = (side == 0 ? a.tau1 : a.tau2)[m];
    if (diag && side == 0) { uo_other = a.uold2[m]; tt_other = a.tau2[m]; }
  }
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int pt = pl; pt < a.nparts; pt += 4) {              // rows up to bstride exist (whole 256-anchor tiles)
    acc[0] += a.sums[((size_t)0 * a.nparts + pt) * a.bstride + r0 + al];
    acc[2] += a.sums[((size_t)2 * a.nparts + pt) * a.bstride + q0 + al];
    if (diag) {
      acc[1] += a.sums[((size_t)1 * a.nparts + pt) * a.bstride + r0 + al];
      acc[3] += a.sums[((size_t)3 * a.nparts + pt) * a.bstride + q0 + al];
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) fs.part[q][pl][al] = acc[q];
  __syncthreads();
  auto total = [&](int q) { return (fs.part[q][0][al] + fs.part[q][1][al]) + (fs.part[q][2][al] + fs.part[q][3][al]); };
  if (diag) {
    if (threadIdx.x < 64) {
      float c1 = 1.0f, c2 = 1.0f;
      double lsum = 0.0, hsum = 0.0;
      if (m < a.b) {
        const float s4[4] = {total(0), total(1), total(2), total(3)};
        state_finish_anchor<false>(a, m, s4, uo, uo_other, tt, tt_other, &c1, &c2, &lsum, &hsum);
      }
      sc[0][al] = c1; sc[1][al] = c2; sc[2][al] = 1.0f / c1; sc[3][al] = 1.0f / c2;
      // the 64 anchors' terms of the loss and of the h sums (Eqs. 8 / 10): one pair per diagonal block
      const double x = wave_sum_f64(lsum), y = wave_sum_f64(hsum);
      if (threadIdx.x == 0) { a.red[2 * blockIdx.x + 0] = x; a.red[2 * blockIdx.x + 1] = y; }
    }
  } else if (threadIdx.x < 128) {
    float c = 1.0f, u_new;
    if (m < a.b) c = anchor_coefficient(a, total(side == 0 ? 0 : 2), uo, tt, &u_new);
    sc[side][al] = c;
    sc[2 + side][al] = 1.0f / c;
  }
}

__global__ void __launch_bounds__(256) k_fold_bf16(bf16_t* __restrict__ E0, bf16_t* __restrict__ E1, int64_t nCB,
                                                   StateArgs a, int64_t off) {
  __shared__ float t0[64][65];   // [r][q]: l1(r, off + q), then w / c1_r
  __shared__ float t1[64][65];   // [q][r]: l2(q, off + r), then w / c2_q
  __shared__ float sc[4][64];    // c1_r, c2_q, 1 / c1_r, 1 / c2_q of the block's rows
  __shared__ FoldState fs;
  const int64_t b = a.b;
  const int64_t r0 = (int64_t)blockIdx.x * 64, q0 = (int64_t)blockIdx.y * 64;
  if (!a.fused) fold_coefficients(a, r0, q0, sc, fs);   // two loads per thread, requested first
  fold_load(E0, nCB, r0, off + q0, b, t0);      // independent of the coefficients: in flight while they are formed
  fold_load(E1, nCB, q0, off + r0, b, t1);
  if (a.fused) fold_coefficients(a, r0, q0, sc, fs);
  __syncthreads();
  const int nr = (int)(b - r0 < 64 ? b - r0 : 64), nq = (int)(b - q0 < 64 ? b - q0 : 64);
  {
    const int ql = threadIdx.x & 63;
    const float cq = sc[1][ql], icq = sc[3][ql];
#pragma unroll 4
    for (int rl = threadIdx.x >> 6; rl < 64; rl += 4) {
      if (rl >= nr || ql >= nq) continue;
      const float w = fmaf(sc[0][rl], t0[rl][ql], cq * t1[ql][rl]);
      t0[rl][ql] = w * sc[2][rl];
      t1[ql][rl] = w * icq;
    }
  }
  __syncthreads();
  fold_store(E0, nCB, r0, off + q0, b, nq, t0);
  fold_store(E1, nCB, q0, off + r0, b, nr, t1);
}

// The same when the whole batch is local and the similarity matrix was formed once: F0[r][q] holds l2(q, p_r) in the
// layout of E0 (off == 0), so w = c1_r E0[r][q] + c2_q F0[r][q]; w / c1_r goes back to E0[r][q] and w / c2_q, transposed,
// to E1[q][r], which nothing has written before: a block writes all 64 columns of its rows of E1, zeros beyond the
// batch, so that every column of E1 up to its padded width holds a number for the contraction.
__global__ void __launch_bounds__(256) k_fold_square_bf16(bf16_t* __restrict__ E0, const bf16_t* __restrict__ F0,
                                                          bf16_t* __restrict__ E1, int64_t nCB, StateArgs a) {
  __shared__ float t0[64][65];   // [r][q]: l1(r, q), then w / c1_r
  __shared__ float t1[64][65];   // [r][q]: l2(q, r); then [q][r]: w / c2_q
  __shared__ float sc[4][64];
  __shared__ FoldState fs;
  const int64_t b = a.b;
  const int64_t r0 = (int64_t)blockIdx.x * 64, q0 = (int64_t)blockIdx.y * 64;
  if (!a.fused) fold_coefficients(a, r0, q0, sc, fs);
  fold_load(E0, nCB, r0, q0, b, t0);
  fold_load(F0, nCB, r0, q0, b, t1);
  if (a.fused) fold_coefficients(a, r0, q0, sc, fs);
  __syncthreads();
  const int nr = (int)(b - r0 < 64 ? b - r0 : 64), nq = (int)(b - q0 < 64 ? b - q0 : 64);
  float keep[16];
  {
    const int ql = threadIdx.x & 63;
    const float cq = sc[1][ql], icq = sc[3][ql];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int rl = (threadIdx.x >> 6) + 4 * i;
      const float w = (rl < nr && ql < nq) ? fmaf(sc[0][rl], t0[rl][ql], cq * t1[rl][ql]) : 0.f;
      t0[rl][ql] = w * sc[2][rl];
      keep[i] = w * icq;
    }
  }
  __syncthreads();               // every thread has read its part of t1 in the [r][q] order
  {
    const int ql = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < 16; ++i) t1[ql][(threadIdx.x >> 6) + 4 * i] = keep[i];
  }
  __syncthreads();
  fold_store(E0, nCB, r0, q0, b, 64, t0);
  fold_store(E1, nCB, q0, r0, b, 64, t1);
}

// Gathered state: the weights c_j l(j, p_r) of the remote anchors (strip F, stored by the strip kernel in the layout of
// E) multiply the same rows of X as l(r, j) does, so E[r][j] += F[r][j] / c_own[r] lets one contraction per side
// produce both sums (its result is multiplied by c_own[r] afterwards).  F is 0 at the local rows' columns, which
// k_fold_bf16 handles, so the two folds touch E independently.  One 16-byte fragment chunk per thread.
__global__ void __launch_bounds__(256) k_fold_remote_bf16(bf16_t* __restrict__ E0, const bf16_t* __restrict__ F0,
                                                          bf16_t* __restrict__ E1, const bf16_t* __restrict__ F1,
                                                          const float* __restrict__ c1, const float* __restrict__ c2,
                                                          int64_t chunks_per_row_block, int64_t b) {
  const int side = blockIdx.y;
  bf16_t* __restrict__ E = side == 0 ? E0 : E1;
  const bf16_t* __restrict__ F = side == 0 ? F0 : F1;
  const float* __restrict__ c_own = side == 0 ? c1 : c2;
  const int64_t chunk = (int64_t)blockIdx.x * 256 + threadIdx.x;      // (anchor block, column block, lane)
  const int64_t ab = chunk / chunks_per_row_block;
  const int64_t r = ab * 32 + (chunk & 31);
  if (r >= b) return;
  const float inv = 1.0f / c_own[r];
  const uint4 e = *(const uint4*)(E + chunk * 8), f = *(const uint4*)(F + chunk * 8);
  const uint32_t ew[4] = {e.x, e.y, e.z, e.w}, fw[4] = {f.x, f.y, f.z, f.w};
  uint32_t o[4];
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float lo = fmaf(__uint_as_float(fw[w] << 16), inv, __uint_as_float(ew[w] << 16));
    const float hi = fmaf(__uint_as_float(fw[w] & 0xffff0000u), inv, __uint_as_float(ew[w] & 0xffff0000u));
    o[w] = pack_bf16x2(lo, hi);
  }
  const u32x4 ov = {o[0], o[1], o[2], o[3]};
  *(u32x4*)(E + chunk * 8) = ov;
}

void launch_fold_bf16(const StepCtx& c) {
  const Layout& L = c.L;
  const unsigned nb = (unsigned)((L.b + 63) / 64);
  const StateArgs st = make_state_args(c);
  if (L.square)
    hipLaunchKernelGGL(k_fold_square_bf16, dim3(nb, nb), dim3(256), 0, c.s, (bf16_t*)(c.ws + L.E[0]),
                       (const bf16_t*)(c.ws + L.F[0]), (bf16_t*)(c.ws + L.E[1]), L.ldE / 16, st);
  else
    hipLaunchKernelGGL(k_fold_bf16, dim3(nb, nb), dim3(256), 0, c.s, (bf16_t*)(c.ws + L.E[0]), (bf16_t*)(c.ws + L.E[1]),
                       L.ldE / 16, st, L.off);
  if (L.gathered) {   // after the kernel above: it leaves the coefficients of all local rows
    const int64_t per_block = (L.ldE / 16) * 64;                       // chunks per block of 32 anchors
    const int64_t chunks = (int64_t)((L.b + 31) / 32) * per_block;
    hipLaunchKernelGGL(k_fold_remote_bf16, dim3((unsigned)((chunks + 255) / 256), 2), dim3(256), 0, c.s,
                       (bf16_t*)(c.ws + L.E[0]), (const bf16_t*)(c.ws + L.F[0]), (bf16_t*)(c.ws + L.E[1]),
                       (const bf16_t*)(c.ws + L.F[1]), (const float*)(c.ws + L.c1), (const float*)(c.ws + L.c2),
                       per_block, L.b);
  }
}

// ----------------------------------------------------------------------------------------------------------------
struct ContractJob {
  const bf16_t* E;    // fragment-ordered strip: l of the local anchors with the contrast-side weights folded in
  const bf16_t* X;    // the matrix whose rows the strip weights: texts for strip 0, images for strip 1
  float* C;           // [nsplit][tile][64 groups of 4 rows][256 columns][4 rows]: whole 256 x 256 tiles
  int64_t ldx;
  size_t split_stride;
  int64_t nCB;        // column blocks (of 16) per anchor block of E
  int stages, slice;  // 32-deep stages in all; stages per split
};
struct ContractArgs {
  ContractJob job[2];   // the two strips
  int64_t M, N, B;
  int nsplit, tiles_m, tiles_n;
};

__global__ void __launch_bounds__(256) k_contract_bf16(ContractArgs g) {
  __shared__ __attribute__((aligned(1024))) char ring[kRingBytes];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const uint32_t ring_addr = lds_addr(ring);
  const int per_job = g.nsplit * g.tiles_m * g.tiles_n;
  const int ji = (int)blockIdx.x / per_job;
  const int local = (int)blockIdx.x % per_job;
  const ContractJob& J = g.job[ji];
  const int split = local % g.nsplit;            // consecutive ids -> different XCDs -> different column slices
  const int tile = local / g.nsplit;
  const int64_t m0 = (int64_t)(tile % g.tiles_m) * 256, n0 = (int64_t)(tile / g.tiles_m) * 256;
  const int s0 = split * J.slice;
  const int S = (s0 + J.slice <= J.stages ? J.slice : J.stages - s0);

  f32x16 acc[4][4];
  zero_acc(acc);
  if (S > 0) {
    ContractTile T;
    T.setup(J.E, J.nCB, m0 >> 5, J.X, J.ldx, n0, g.N, g.B, tid);
    // The unguarded loads of a stage take 32 whole rows of X and 256 columns from n0 on.  They stay inside the matrix
    // (B rows of ldx elements, the last one of N) for the stages below `safe`: rows beyond B never, and where the tile
    // is wider than what is left of a row (n0 + 256 > N) the words past the row's end are the next rows' - they exist
    // except behind the last rows, and what they put into the columns from N on reaches no output.  Those stages run
    // through the ring; the few that are left at the ragged end go one at a time with guards.
    int64_t rows_ok = g.B;
    if (n0 + 256 > g.N) rows_ok -= (n0 + 256 - g.N + J.ldx - 1) / J.ldx;
    const int safe = rows_ok > 0 ? (int)(rows_ok / BK) : 0;
    const int S_ring = s0 + S <= safe ? S : (safe > s0 ? safe - s0 : 0);
    if (S_ring > 0) {
      ring_prologue(T, ring_addr, s0, S_ring);
      ring_mainloop(acc, T, ring, ring_addr, s0, S_ring);
    }
    if (S_ring < S) guarded_mainloop(acc, T, ring, s0 + S_ring, S - S_ring, tid);
  }
  // The partial result leaves as whole tiles of [64 groups of 4 rows][256 columns][4 rows]: a lane holds C[m][n] for
  // n = n0 + wn 128 + tj 32 + lr and the rows m = m0 + wm 128 + ti 32 + 8 q + 4 hk + t, t = 0..3, so its four values of one
  // q are one 16-byte word of that layout and a wave store covers two runs of 512 consecutive bytes.  The buffer holds
  // whole tiles, so nothing is guarded here; k_finalize_bf16 reads four rows at a time in the same order.
  const int lr = lane & 31, hk = lane >> 5;
  float* __restrict__ C = J.C + (size_t)split * J.split_stride + (size_t)tile * kPartialTileFloats +
                          ((wm * 32 + hk) * 256 + wn * 128 + lr) * 4;
#pragma unroll
  for (int ti = 0; ti < 4; ++ti)
#pragma unroll
    for (int tj = 0; tj < 4; ++tj)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 v = {acc[ti][tj][4 * q], acc[ti][tj][4 * q + 1], acc[ti][tj][4 * q + 2], acc[ti][tj][4 * q + 3]};
        *(f32x4*)(C + ((ti * 8 + q * 2) * 256 + tj * 32) * 4) = v;
      }
}

void launch_contract_bf16(const StepCtx& c) {
  const Layout& L = c.L;
  ContractArgs g;
  const int njobs = 2;
  for (int j = 0; j < njobs; ++j) {
    const int s = j & 1;
    ContractJob& J = g.job[j];
    J.E = (const bf16_t*)(c.ws + L.E[s]);
    J.X = (const bf16_t*)(s == 0 ? c.buf.txt_glob : c.buf.img_glob);
    J.ldx = s == 0 ? c.cfg.ld_txt : c.cfg.ld_img;
    J.C = (float*)(c.ws + L.Opart[s]);
    J.split_stride = partial_split_floats(L.b, L.d);
    J.nCB = L.ldE / 16;
    J.stages = (int)(L.ldE / BK);
    J.slice = (int)L.kslice;
  }
  g.M = L.b; g.N = L.d; g.B = L.B;
  g.nsplit = L.nsplit;
  g.tiles_m = (int)((L.b + 255) / 256);
  g.tiles_n = (int)((L.d + 255) / 256);
  const unsigned grid = (unsigned)njobs * (unsigned)(g.nsplit * g.tiles_m * g.tiles_n);
  hipLaunchKernelGGL(k_contract_bf16, dim3(grid), dim3(256), 0, c.s, g);
}

}  // namespace fc
