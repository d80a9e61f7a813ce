// k_strips_bf16: the similarity strips of Proc. 1 on whole 256 x 256 tiles (gfx950, wave64, MFMA 32x32x16 bf16).
//
// For every tile (strip, 256 anchors, 256 contrasts) the kernel forms s = x_contrast . x_anchor in registers, then
// l = exp((s - s_pp) / tau_p) (Sec. 3), adds l and (s - s_pp) l into per-anchor partial sums (Proc. 1; the sums behind
// Eqs. 8-10), and stores l rounded to bf16 in the fragment order the gradient contraction reads.
//
// Shape of the work.  One workgroup of EIGHT waves per compute unit computes a 256 x 256 tile (the largest that the
// accumulator registers of a compute unit hold, hence the fewest operand bytes per flop); a wave owns 64 contrasts x
// 128 anchors = 2 x 4 accumulator blocks (128 AGPRs), so every SIMD runs two waves and always has a second
// instruction stream when one waits for LDS data.
//
// Data movement.  Operands go global -> LDS with direct-to-LDS loads, 64 deep in k per stage: every row contributes
// one whole 128-byte line per stage (half-line requests reach only about 60 % of the load path's rate).  A panel is
// 256 rows x 64 of k = 32 KiB of either the contrast rows X or the anchor rows A, and the LDS is a ring of FIVE
// panels (160 KiB, all of it).  During stage g the ring holds X_g A_g X_g+1 A_g+1 X_g+2: the contrast panel, which is
// new to the L2 for the first workgroup that touches it and then comes from HBM, is requested two stage times
// before it is needed; the anchor panel (the same 256 rows for every tile of a workgroup, L2 hits) one.  (With two
// whole-stage slots both had one stage time, less than an HBM access takes under load, and a fifth of the loop went
// into waiting for data.)  The barrier three quarters into stage g retires X_g and A_g; A_g+2 is requested into the
// first, X_g+3 into the second, A before X, so that "A_g+1 has landed" is vmcnt(8): vector memory operations
// complete in order, and only the eight younger X loads may still fly.  The requests form one continuous stream over
// stages and tiles; past the last tile the stream keeps re-requesting its last stage (nobody reads it), which keeps
// every s_waitcnt immediate constant.  Nothing else has LDS of its own: at the end of a tile the panel that waits
// for X_g+3 is free, and the tile's per-anchor scalars, column parameters and cross-wave sums use it.
//
// Who requests.  A SIMD runs waves w and w + 4, and its matrix core serves the older wave first: with the requests
// shared evenly, waves 0 .. 3 reached every barrier about 700 cycles before waves 4 .. 7 and idled there (a wave
// that issues a direct-to-LDS load is held for about 60 cycles).  So waves 0 .. 3 issue ALL requests, their own rows
// and those of their SIMD's other wave (16 wave loads per stage), and waves 4 .. 7 none: 2970 -> 2620 cycles per
// 64-deep stage (2048 being the MFMA time).
//
// MODE 1 (gathered state): every element additionally yields the weight of Eqs. 3 / 5 / 7 with which its contrast
// column, taken as an anchor of another worker, moves the local row; it goes to a second strip of the same form.
// MODE 2 (the whole batch is local, b == B): the text strip is the transpose of the image strip, so only the image
// strip is formed; every element s_pj yields l1(p, j) (row parameters, summed along the row as before) and l2(j, p)
// (column parameters: text anchor j against image p), which is stored as a second strip of the same form and summed
// down the columns.
#include "mfma_common.hpp"

namespace fc {

constexpr int kSK = 64;                         // contraction depth of a stage: 128 bytes per row
constexpr int kSOp = 256 * kSK * 2;             // one operand of a stage: 32 KiB

// LDS image of an operand of a stage (256 rows x 128 bytes): 16-byte chunk c of row r sits at chunk position
// c ^ ((r >> 1) & 7), so that the 16 consecutive rows one operand read touches per cycle cover all 16 chunk slots
// of a 256-byte bank window.
__device__ __forceinline__ int st_swz(int row) { return (row >> 1) & 7; }


// 16 bytes per lane from uniform_base + lane_byte_off into LDS at (lds_uniform + IMM) + 16 * lane.
template <int IMM>
__device__ __forceinline__ void dma16i(const void* uniform_base, uint32_t lane_byte_off, uint32_t lds_uniform) {
  asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_byte_off), "s"(uniform_base), "s"(lds_uniform), "n"(IMM)
               : "memory", "scc");
}

__device__ __forceinline__ void zero_acc24(f32x16 (&acc)[2][4]) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
}

#define FC_HMM(ti, tj, A_, B_) \
  acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A_[ti], B_[tj], acc[ti][tj], 0, 0, 0)
#define FC_LDS16(p) (*(const bf16x8*)(p))
// An operand read of the main loop; the measurement variants without operand reads keep what the register holds.
#define FC_RD(p, keep) (((ABL) & kAblNoOperandReads) ? (keep) : FC_LDS16(p))

// Measurement variants of k_strips_bf16 (template parameter ABL, 0 in the step): parts of the kernel compiled out, to
// learn what each costs, and per-wave cycle counters.  Their results are meaningless; they write where the step writes.
constexpr int kAblNoRequests = 1;       // no global -> LDS requests (operands are whatever the LDS holds)
constexpr int kAblNoOperandReads = 2;   // no LDS operand reads in the main loop (register operands never change)
constexpr int kAblNoEpilogue = 4;       // no exponentials, sums or stores
constexpr int kAblTimed = 8;            // cycle counters of waves 0 and 4 of every workgroup go to StripArgs::cycles

// Epilogue of one wave (64 contrasts x 128 anchors).  Accumulator (ti, tj, v) of lane (lr, hk): contrast
// c_first + 32 ti + 8 (v >> 2) + 4 hk + (v & 3), anchor anchor0 + 32 tj + lr.  t = (s - s_pp) log2(e)/tau, l = 2^t.
// MASK: the anchor's own column may fall among these contrasts (B_{i-} excludes i): l := 0 there.
// frag0: fragment (anchor block of tj = 0, column block of c_first) of the stored strip; row_bytes: bytes from one
// anchor block to the next.  sg / st: sums of l and t l per anchor (added to).
template <bool MASK>
__device__ __forceinline__ void half_epilogue(f32x16 (&acc)[2][4], const float* sk, const float* sdiag,
                                              float (&sg)[4], float (&st)[4], char* frag0, int64_t row_bytes,
                                              int c_first, int own0, int al0, int lane) {
  const int lr = lane & 31, hk = lane >> 5;
#pragma unroll
  for (int tj = 0; tj < 4; ++tj) {
    const int al = al0 + tj * 32 + lr;
    const float kk = sk[al], dk = sdiag[al] * kk;   // log2(e)/tau and s_pp log2(e)/tau of this anchor
    const int own = own0 + tj * 32 + lr;            // global row of the anchor itself
    char* fr = frag0 + tj * row_bytes;              // wave-uniform
    float sgv[4] = {0.f, 0.f, 0.f, 0.f}, stv[4] = {0.f, 0.f, 0.f, 0.f};   // independent chains
#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
      const int crow = c_first + ti * 32 + 4 * hk;
      uint32_t pk[8];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float t[4], e[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) t[q] = fmaf(acc_read(acc[ti][tj][4 * g + q]), kk, -dk);
#pragma unroll
        for (int q = 0; q < 4; ++q) e[q] = __builtin_amdgcn_exp2f(t[q]);
        if (MASK) {
#pragma unroll
          for (int q = 0; q < 4; ++q) e[q] = (crow + 8 * g + q != own) ? e[q] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          sgv[q] += e[q];
          stv[q] = fmaf(t[q], e[q], stv[q]);
        }
        pk[2 * g] = pack_bf16x2(e[0], e[1]);
        pk[2 * g + 1] = pack_bf16x2(e[2], e[3]);
        FC_PIN();
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const u32x4 w = {pk[4 * j], pk[4 * j + 1], pk[4 * j + 2], pk[4 * j + 3]};
        *(u32x4*)(fr + (2 * ti + j) * 1024 + lane * 16) = w;
      }
      FC_PIN();
    }
    sg[tj] += (sgv[0] + sgv[1]) + (sgv[2] + sgv[3]);
    st[tj] += (stv[0] + stv[1]) + (stv[2] + stv[3]);
  }
}

// The same with the second strip of the gathered-state mode: besides l of the anchor (row parameters) every element
// also yields f = c_j 2^(s k_j - d_j), the weight with which contrast column j, taken as an ANCHOR, moves the local
// row (Eqs. 3 / 5 / 7); scol = the tile's column parameters [4][256] in LDS, cl0 = this lane's first column inside
// the tile for ti = 0, g = 0.  No mask is needed for f: the own column is a local row, whose c is 0.
template <bool MASK>
__device__ __forceinline__ void half_epilogue_remote(f32x16 (&acc)[2][4], const float* sk, const float* sdiag,
                                                     const float* scol, float (&sg)[4], float (&st)[4], char* frag0,
                                                     int64_t row_bytes, char* fragF0, int64_t row_bytesF, int c_first,
                                                     int own0, int al0, int cl0, int lane) {
  const int lr = lane & 31, hk = lane >> 5;
#pragma unroll
  for (int tj = 0; tj < 4; ++tj) {
    const int al = al0 + tj * 32 + lr;
    const float kk = sk[al], dk = sdiag[al] * kk;
    const int own = own0 + tj * 32 + lr;
    char* fr = frag0 + tj * row_bytes;              // wave-uniform
    char* frF = fragF0 + tj * row_bytesF;
    float sgv[4] = {0.f, 0.f, 0.f, 0.f}, stv[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
      const int crow = c_first + ti * 32 + 4 * hk;
      uint32_t pk[8], pf[8];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cl = cl0 + ti * 32 + 8 * g;
        const float4 ck = *(const float4*)(scol + cl), cd = *(const float4*)(scol + 256 + cl),
                     cc = *(const float4*)(scol + 512 + cl);
        const float ckq[4] = {ck.x, ck.y, ck.z, ck.w}, cdq[4] = {cd.x, cd.y, cd.z, cd.w},
                    ccq[4] = {cc.x, cc.y, cc.z, cc.w};
        float sv[4], t[4], e[4], f[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) sv[q] = acc_read(acc[ti][tj][4 * g + q]);
#pragma unroll
        for (int q = 0; q < 4; ++q) t[q] = fmaf(sv[q], kk, -dk);
#pragma unroll
        for (int q = 0; q < 4; ++q) e[q] = __builtin_amdgcn_exp2f(t[q]);
#pragma unroll
        for (int q = 0; q < 4; ++q) f[q] = ccq[q] * __builtin_amdgcn_exp2f(fmaf(sv[q], ckq[q], -cdq[q]));
        if (MASK) {
#pragma unroll
          for (int q = 0; q < 4; ++q) e[q] = (crow + 8 * g + q != own) ? e[q] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          sgv[q] += e[q];
          stv[q] = fmaf(t[q], e[q], stv[q]);
        }
        pk[2 * g] = pack_bf16x2(e[0], e[1]);
        pk[2 * g + 1] = pack_bf16x2(e[2], e[3]);
        pf[2 * g] = pack_bf16x2(f[0], f[1]);
        pf[2 * g + 1] = pack_bf16x2(f[2], f[3]);
        FC_PIN();
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const u32x4 w = {pk[4 * j], pk[4 * j + 1], pk[4 * j + 2], pk[4 * j + 3]};
        *(u32x4*)(fr + (2 * ti + j) * 1024 + lane * 16) = w;
        const u32x4 wf = {pf[4 * j], pf[4 * j + 1], pf[4 * j + 2], pf[4 * j + 3]};
        *(u32x4*)(frF + (2 * ti + j) * 1024 + lane * 16) = wf;
      }
      FC_PIN();
    }
    sg[tj] += (sgv[0] + sgv[1]) + (sgv[2] + sgv[3]);
    st[tj] += (stv[0] + stv[1]) + (stv[2] + stv[3]);
  }
}

// Second pass over the accumulators of one wave when the whole batch is local (the first pass is half_epilogue, with
// the image anchors' row parameters).  Every element s_pj also yields f = l2(j, p) = 2^((s - s_jj) log2(e)/tau2_j) of
// the TEXT anchor j = its contrast column; f is stored in a second strip of the same form (fragF0) and summed over the
// anchors of the wave: scol_k / scol_d hold log2(e)/tau2_j and s_jj of the tile's 256 columns, cl0 = this lane's
// first column in the tile for ti = 0, g = 0; sredc[quantity][column] receives the wave's column sums of f and of
// (s - s_jj) f.  MASK: the tile holds diagonal elements j == p, which are not in B_{j-}: f := 0.
template <bool MASK>
__device__ __forceinline__ void half_epilogue_cols(f32x16 (&acc)[2][4], const float* scol_k, const float* scol_d,
                                                   float (*sredc)[256], char* fragF0, int64_t row_bytesF, int c_first,
                                                   int own0, int cl0, int lane) {
  const int lr = lane & 31, hk = lane >> 5;
#pragma unroll
  for (int ti = 0; ti < 2; ++ti) {
    const int crow = c_first + ti * 32 + 4 * hk;
#pragma unroll
    for (int j = 0; j < 2; ++j) {            // the 16-byte fragment store j holds the groups g = 2 j, 2 j + 1
      const int cl = cl0 + ti * 32 + 16 * j;
      const float4 k0 = *(const float4*)(scol_k + cl), k1 = *(const float4*)(scol_k + cl + 8);
      const float4 d0 = *(const float4*)(scol_d + cl), d1 = *(const float4*)(scol_d + cl + 8);
      const float ck[8] = {k0.x, k0.y, k0.z, k0.w, k1.x, k1.y, k1.z, k1.w};
      const float cdk[8] = {d0.x * k0.x, d0.y * k0.y, d0.z * k0.z, d0.w * k0.w,
                            d1.x * k1.x, d1.y * k1.y, d1.z * k1.z, d1.w * k1.w};
      float cs[16];                          // column sums of this lane: f of 8 columns, then t f of 8 columns
#pragma unroll
      for (int i = 0; i < 16; ++i) cs[i] = 0.f;
#pragma unroll
      for (int tj = 0; tj < 4; ++tj) {
        const int drow = own0 + tj * 32 + lr - crow;     // the diagonal element sits at 8 g + q == drow
        uint32_t pf[4];
#pragma unroll
        for (int gi = 0; gi < 2; ++gi) {
          const int g = 2 * j + gi;
          float t2[4], f[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) t2[q] = fmaf(acc_read(acc[ti][tj][4 * g + q]), ck[4 * gi + q], -cdk[4 * gi + q]);
#pragma unroll
          for (int q = 0; q < 4; ++q) f[q] = __builtin_amdgcn_exp2f(t2[q]);
          if (MASK) {
#pragma unroll
            for (int q = 0; q < 4; ++q) f[q] = (drow == 8 * g + q) ? 0.f : f[q];
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
        *(u32x4*)(fragF0 + tj * row_bytesF + (2 * ti + j) * 1024 + lane * 16) = wf;
        FC_PIN();
      }
      // divide the second quantity by log2(e)/tau_j while each lane still knows its columns, then sum over the lanes
#pragma unroll
      for (int i = 0; i < 8; ++i) cs[8 + i] = ck[i] > 0.f ? cs[8 + i] * __builtin_amdgcn_rcpf(ck[i]) : 0.f;
      lanes32_sum(cs, lane);
      if ((lr & 1) == 0) {
        const int v = lr >> 1, gi = (v >> 2) & 1, q = v & 3;     // value v = 8 quantity + 4 gi + q
        sredc[v >> 3][cl + 8 * gi + q] = cs[0];
      }
      FC_PIN();
    }
  }
}

// One 16-deep step: 8 MFMAs on operand set P while operand set Q is read for the following step from px / pa;
// D0 .. D7 are statements (requests or nothing) placed one per MFMA.
#define FC_NONE (void)0
#define FC_STEP(XP, AP, XQ, AQ, px, pa, D0, D1, D2, D3, D4, D5, D6, D7)                               \
  FC_HMM(0, 0, XP, AP); FC_PIN(); XQ[0] = FC_RD(px, XQ[0]);         FC_PIN(); D0; FC_PIN();          \
  FC_HMM(0, 1, XP, AP); FC_PIN(); AQ[0] = FC_RD(pa, AQ[0]);         FC_PIN(); D1; FC_PIN();          \
  FC_HMM(0, 2, XP, AP); FC_PIN(); XQ[1] = FC_RD(px + 4096, XQ[1]);  FC_PIN(); D2; FC_PIN();          \
  FC_HMM(0, 3, XP, AP); FC_PIN(); AQ[1] = FC_RD(pa + 4096, AQ[1]);  FC_PIN(); D3; FC_PIN();          \
  FC_HMM(1, 0, XP, AP); FC_PIN(); AQ[2] = FC_RD(pa + 8192, AQ[2]);  FC_PIN(); D4; FC_PIN();          \
  FC_HMM(1, 1, XP, AP); FC_PIN(); AQ[3] = FC_RD(pa + 12288, AQ[3]); FC_PIN(); D5; FC_PIN();          \
  FC_HMM(1, 2, XP, AP); FC_PIN(); D6; FC_PIN();                                                      \
  FC_HMM(1, 3, XP, AP); FC_PIN(); D7; FC_PIN()
#define FC_STEP_PLAIN(XP, AP, XQ, AQ, px, pa) \
  FC_STEP(XP, AP, XQ, AQ, px, pa, FC_NONE, FC_NONE, FC_NONE, FC_NONE, FC_NONE, FC_NONE, FC_NONE, FC_NONE)


constexpr int kPart = kSOp;               // 32 KiB
constexpr int kRing5 = 5 * kPart;         // 160 KiB
// what the free panel holds during an epilogue, after the per-anchor scalars sk[256], sdiag[256] (byte offsets)
constexpr uint32_t kScolOff = 2048u, kSredOff = 6144u, kSredcOff = 14336u;
// s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] in bits 3:0, vmcnt[5:4] in bits 15:14; expcnt and lgkmcnt left open)
#define FC_WAIT_VMCNT25() __builtin_amdgcn_s_waitcnt(0x4f79)   // 25 = 0b011001
#define FC_WAIT_VMCNT41() __builtin_amdgcn_s_waitcnt(0x8f79)   // 41 = 0b101001
#define FC_WAIT_VMCNT42() __builtin_amdgcn_s_waitcnt(0x8f7a)   // 42 = 0b101010

template <int MODE, int ABL>
__global__ void __launch_bounds__(512, 2) k_strips_bf16(StripArgs a) {
  constexpr bool REMOTE = MODE == 1, SQUARE = MODE == 2;
  uint64_t t_begin = 0, t_wall = 0, t_epilogue = 0;
  if constexpr ((ABL & kAblTimed) != 0) { t_begin = __builtin_readcyclecounter(); t_wall = wall_clock64(); }
  __shared__ __attribute__((aligned(1024))) char ring[kRing5];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave >> 1, wc = wave & 1, lr = lane & 31, hk = lane >> 5;
  const uint32_t ring_addr = lds_addr(ring);
  const int S = (int)(a.d / kSK);   // >= 2
  // ids that share an XCD (id mod 8 under round-robin dispatch) take neighbouring tiles, and neighbouring tiles are
  // the anchor tiles of one contrast tile, so a contrast tile is fetched once per L2
  const int G = gridDim.x;
  const int vid = (G % 8 == 0) ? (int)(blockIdx.x % 8) * (G / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
  const int per_strip = a.nAT * a.nCT;
  auto next_interior = [&](int tt) {
    while (tt < a.ntiles &&
           !strip_tile_is_interior(a, strip_anchor_first(a, tt % a.nAT, SQUARE), (int64_t)((tt / a.nAT) % a.nCT) * 256))
      tt += G;
    return tt;
  };

  // ---- the two request streams (waves 0 .. 3 only): wave w requests rows 32 w .. 32 w + 31 and 128 + 32 w .. of a
  // panel, 8 wave loads of 8 rows x 128 bytes; lane l of a wave load fetches chunk (l & 7) ^ swz of row (l >> 3) (rows
  // 128 apart share their swizzle, so loads 4 .. 7 use the lane offsets of loads 0 .. 3 on a base 128 rows on).  The X
  // stream runs one stage ahead of the A stream, so near a tile change the two are in different tiles.
  uint32_t ox[4], oa[4];
  const bf16_t *qx, *qa;
  int x_left, x_tile, a_left, a_tile;
  int64_t ldx = 0, lda = 0;
  auto open_x = [&](int tt) {
    const int strip = tt / per_strip, ct = (tt / a.nAT) % a.nCT;
    const int64_t ld = a.ld_contrast[strip];
    qx = a.contrasts[strip] + (int64_t)ct * 256 * ld;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 8 * (4 * wave + i) + (lane >> 3);
      ox[i] = (uint32_t)(row * (int)ld + ((((lane & 7) ^ st_swz(row))) << 3)) * 2u;
    }
    x_left = S; x_tile = tt; ldx = ld;
  };
  auto open_a = [&](int tt) {
    const int strip = tt / per_strip, at = tt % a.nAT;
    const int64_t ld = a.ld_anchor[strip];
    qa = a.anchors[strip] + strip_anchor_first(a, at, SQUARE) * ld;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 8 * (4 * wave + i) + (lane >> 3);
      oa[i] = (uint32_t)(row * (int)ld + ((((lane & 7) ^ st_swz(row))) << 3)) * 2u;
    }
    a_left = S; a_tile = tt; lda = ld;
  };
  auto advance_x = [&]() {
    if (x_tile >= a.ntiles) return;          // past the end: keep re-requesting the last stage
    if (--x_left > 0) { qx += kSK; return; }
    const int tn = next_interior(x_tile + G);
    if (tn < a.ntiles) open_x(tn); else x_tile = tn;
  };
  auto advance_a = [&]() {
    if (a_tile >= a.ntiles) return;
    if (--a_left > 0) { qa += kSK; return; }
    const int tn = next_interior(a_tile + G);
    if (tn < a.ntiles) open_a(tn); else a_tile = tn;
  };
  const uint32_t my = ring_addr + (uint32_t)wave * 4096u;   // this wave's rows inside a panel
#define FC5_X(i, part) \
  dma16i<((i) & 3) * 1024>(qx + ((i) >> 2) * 128 * ldx, ox[(i) & 3], my + (part) + (uint32_t)((i) >> 2) * 16384u)
#define FC5_A(i, part) \
  dma16i<((i) & 3) * 1024>(qa + ((i) >> 2) * 128 * lda, oa[(i) & 3], my + (part) + (uint32_t)((i) >> 2) * 16384u)
#define FC5_X8(p) FC5_X(0, p); FC5_X(1, p); FC5_X(2, p); FC5_X(3, p); FC5_X(4, p); FC5_X(5, p); FC5_X(6, p); FC5_X(7, p)
#define FC5_A8(p) FC5_A(0, p); FC5_A(1, p); FC5_A(2, p); FC5_A(3, p); FC5_A(4, p); FC5_A(5, p); FC5_A(6, p); FC5_A(7, p)

  int t = next_interior(vid);
  if (t >= a.ntiles) return;
  // ring positions (byte offsets) of X_g A_g X_g+1 A_g+1 X_g+2; every stage moves on by two
  uint32_t P0 = 0u, P1 = (uint32_t)kPart, P2 = 2u * kPart, P3 = 3u * kPart, P4 = 4u * kPart;
  const bool requester = (ABL & kAblNoRequests) ? false : wave < 4;
  open_x(t);
  open_a(t);
  if (requester) {
    FC5_X8(P0); advance_x();
    FC5_A8(P1); advance_a();
    FC5_X8(P2); advance_x();
    FC5_A8(P3); advance_a();
    FC5_X8(P4); advance_x();
  }

  // operand reads: the lane's address inside a panel for the 16-deep step 0 (step j: bits 5..6 XORed by j)
  const uint32_t bx = (uint32_t)((wr * 64 + lr) * 128 + ((hk ^ st_swz(wr * 64 + lr)) << 4));
  const uint32_t ba = (uint32_t)((wc * 128 + lr) * 128 + ((hk ^ st_swz(wc * 128 + lr)) << 4));

  FC_WAIT_VMCNT0();
  __syncthreads();
  bf16x8 x0[2], a0[4], x1[2], a1[4];
  x0[0] = FC_LDS16(ring + P0 + bx); x0[1] = FC_LDS16(ring + P0 + bx + 4096);
#pragma unroll
  for (int j = 0; j < 4; ++j) a0[j] = FC_LDS16(ring + P1 + ba + j * 4096);
  if constexpr ((ABL & kAblNoOperandReads) != 0) {   // both operand sets start from the same (arbitrary) LDS contents
    x1[0] = x0[1]; x1[1] = x0[0];
#pragma unroll
    for (int j = 0; j < 4; ++j) a1[j] = a0[3 - j];
  }

  bool pend_x = false;   // X_g+2 is still to be requested (always during the first step after a barrier's last step)
  bool after_epilogue = false;
  while (t < a.ntiles) {
    const int strip = t / per_strip, at = t % a.nAT, ct = (t / a.nAT) % a.nCT;
    const int a_first = (int)strip_anchor_first(a, at, SQUARE), c_tile = ct * 256;
    f32x16 acc[2][4];
    zero_acc24(acc);
#pragma unroll 1
    for (int s = 0; s < S; ++s) {
      const bool last = s + 1 == S;
      {
        const char* px = ring + ((bx ^ 32u) + P0);
        const char* pa = ring + ((ba ^ 32u) + P1);
        // X_g+2 into the panel that A_g-1 left (now called P4); at the start of a tile this comes after the
        // epilogue, which used that panel
        FC_STEP(x0, a0, x1, a1, px, pa, if (pend_x) FC5_X(0, P4), if (pend_x) FC5_X(1, P4), if (pend_x) FC5_X(2, P4),
                if (pend_x) FC5_X(3, P4), if (pend_x) FC5_X(4, P4), if (pend_x) FC5_X(5, P4), if (pend_x) FC5_X(6, P4),
                if (pend_x) FC5_X(7, P4));
        if (pend_x) advance_x();
        pend_x = false;
      }
      {
        const char* px = ring + ((bx ^ 64u) + P0);
        const char* pa = ring + ((ba ^ 64u) + P1);
        FC_STEP_PLAIN(x1, a1, x0, a0, px, pa);
      }
      {
        const char* px = ring + ((bx ^ 96u) + P0);
        const char* pa = ring + ((ba ^ 96u) + P1);
        FC_STEP_PLAIN(x0, a0, x1, a1, px, pa);
      }
      // A_g+1 has landed (X_g+1 long before): younger are only the eight loads of X_g+2, and once after an epilogue
      // its fragment stores (16; with a second strip 32) and its sum stores (1; MODE 2: 2) as well.  The barrier
      // publishes it to the waves that request nothing and retires X_g and A_g.
      if (requester) {
        if (!after_epilogue) FC_WAIT_VMCNT8();
        else if (REMOTE) FC_WAIT_VMCNT41();
        else if (SQUARE) FC_WAIT_VMCNT42();
        else FC_WAIT_VMCNT25();
      }
      after_epilogue = false;
      __syncthreads();
      FC_PIN();
      if (last && !(ABL & kAblNoRequests)) {   // the tile's per-anchor scalars go into the panel A_g has just left (free until X_g+3 is requested)
        if (wave < 4) dma4(a.kscale[strip] + a_first + wave * 64, lane * 4, ring_addr + P1 + (uint32_t)wave * 256u);
        else dma4(a.diag + a_first + (wave - 4) * 64, lane * 4, ring_addr + P1 + 1024u + (uint32_t)(wave - 4) * 256u);
        if constexpr (REMOTE) {   // the tile's column parameters [4][256], two 256-byte pieces per wave
          const float* cp = a.colp + ((int64_t)strip * a.nCT + ct) * 1024;
          dma4(cp + wave * 64, lane * 4, ring_addr + P1 + kScolOff + (uint32_t)wave * 256u);
          dma4(cp + (wave + 8) * 64, lane * 4, ring_addr + P1 + kScolOff + (uint32_t)(wave + 8) * 256u);
        }
        if constexpr (SQUARE) {   // the text anchors of the tile's columns (off == 0: anchor index == global row)
          if (wave < 4) dma4(a.kscale[1] + c_tile + wave * 64, lane * 4, ring_addr + P1 + kScolOff + (uint32_t)wave * 256u);
          else dma4(a.diag + c_tile + (wave - 4) * 64, lane * 4, ring_addr + P1 + kScolOff + 1024u + (uint32_t)(wave - 4) * 256u);
        }
      }
      {
        // last step; meanwhile read the first step's operands of stage g + 1 and request A_g+2 into X_g's panel
        // (X_g+3 follows during the next step, into A_g's)
        const char* px = ring + (bx + P2);
        const char* pa = ring + (ba + P3);
        FC_STEP(x1, a1, x0, a0, px, pa, if (requester) FC5_A(0, P0), if (requester) FC5_A(1, P0),
                if (requester) FC5_A(2, P0), if (requester) FC5_A(3, P0), if (requester) FC5_A(4, P0),
                if (requester) FC5_A(5, P0), if (requester) FC5_A(6, P0), if (requester) FC5_A(7, P0));
        if (requester) advance_a();
        pend_x = requester;
      }
      const uint32_t n0 = P2, n1 = P3, n2 = P4, n3 = P0, n4 = P1;
      P0 = n0; P1 = n1; P2 = n2; P3 = n3; P4 = n4;
    }
    // the scalars have landed (for the requesting waves the eight loads of A_g+2 are younger); the free panel is now
    // called P4
    if (requester) FC_WAIT_VMCNT8(); else FC_WAIT_VMCNT0();
    __syncthreads();
    uint64_t t_e0 = 0;
    if constexpr ((ABL & kAblTimed) != 0) t_e0 = __builtin_readcyclecounter();
    if constexpr ((ABL & kAblNoEpilogue) == 0) {
      const float* sk = (const float*)(ring + P4);
      const float* sdiag = sk + 256;
      const float* scol = (const float*)(ring + P4 + kScolOff);                    // MODE 1: [4][256]; MODE 2: [2][256]
      float (*sred)[2][256] = (float (*)[2][256])(ring + P4 + kSredOff);           // [4 contrast quarters][2][256]
      float (*sredc)[2][256] = (float (*)[2][256])(ring + P4 + kSredcOff);         // MODE 2: [2 anchor halves][2][256]
      float sg[4] = {0.f, 0.f, 0.f, 0.f}, st[4] = {0.f, 0.f, 0.f, 0.f};
      const int c_first = c_tile + wr * 64;
      char* frag0 = (char*)a.E[strip] + (((int64_t)(a_first + wc * 128) >> 5) * a.nCB + (c_first >> 4)) * 1024;
      const int64_t row_bytes = a.nCB * 1024;
      const int own0 = (int)a.off + a_first + wc * 128;
      const bool diagonal = (c_first < own0 + 128) && (c_first + 64 > own0);
      if constexpr (REMOTE) {
        char* fragF0 = (char*)a.F[strip] + (((int64_t)(a_first + wc * 128) >> 5) * a.nCBF + (c_first >> 4)) * 1024;
        const int64_t row_bytesF = a.nCBF * 1024;
        const int cl0 = wr * 64 + 4 * (lane >> 5);
        if (diagonal)
          half_epilogue_remote<true>(acc, sk, sdiag, scol, sg, st, frag0, row_bytes, fragF0, row_bytesF, c_first, own0,
                                     wc * 128, cl0, lane);
        else
          half_epilogue_remote<false>(acc, sk, sdiag, scol, sg, st, frag0, row_bytes, fragF0, row_bytesF, c_first, own0,
                                      wc * 128, cl0, lane);
      } else {
        if (diagonal) half_epilogue<true>(acc, sk, sdiag, sg, st, frag0, row_bytes, c_first, own0, wc * 128, lane);
        else half_epilogue<false>(acc, sk, sdiag, sg, st, frag0, row_bytes, c_first, own0, wc * 128, lane);
      }
      if constexpr (SQUARE) {
        char* fragF0 = (char*)a.F[0] + (((int64_t)(a_first + wc * 128) >> 5) * a.nCBF + (c_first >> 4)) * 1024;
        const int64_t row_bytesF = a.nCBF * 1024;
        const int cl0 = wr * 64 + 4 * (lane >> 5);
        if (diagonal) half_epilogue_cols<true>(acc, scol, scol + 256, sredc[wc], fragF0, row_bytesF, c_first, own0, cl0, lane);
        else half_epilogue_cols<false>(acc, scol, scol + 256, sredc[wc], fragF0, row_bytesF, c_first, own0, cl0, lane);
      }
  #pragma unroll
      for (int tj = 0; tj < 4; ++tj) {
        const int al = wc * 128 + tj * 32 + lr;
        const float kk = sk[al];
        const float g2 = sg[tj] + __shfl_xor(sg[tj], 32);
        const float t2 = st[tj] + __shfl_xor(st[tj], 32);
        if (hk == 0) {
          sred[wr][0][al] = g2;
          sred[wr][1][al] = kk > 0.f ? t2 * __builtin_amdgcn_rcpf(kk) : 0.f;   // sum of (s - s_pp) l
        }
      }
      __syncthreads();
      {
        const int q = tid >> 8, m = tid & 255;
        a.sums[((size_t)(2 * strip + q) * a.nparts + ct) * a.bstride + a_first + m] =
            (sred[0][q][m] + sred[1][q][m]) + (sred[2][q][m] + sred[3][q][m]);
        // the text anchors' sums (quantities 2, 3): partial number = the anchor tile, position = the column
        if constexpr (SQUARE) a.sums[((size_t)(2 + q) * a.nparts + at) * a.bstride + c_tile + m] = sredc[0][q][m] + sredc[1][q][m];
      }
    }
    if constexpr ((ABL & kAblNoEpilogue) != 0) {      // nothing reads the accumulators: keep the MFMAs that wrote them
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) asm volatile("" : : "a"(acc[i][j][v]));
    }
    __syncthreads();     // the panel is given back: X_g+3 is requested into it during the next step
    if constexpr ((ABL & kAblTimed) != 0) t_epilogue += __builtin_readcyclecounter() - t_e0;
    if constexpr (MODE != 0) {
      // the first operands of the next tile (read during the last step above) are read again here, so that their
      // registers are free during these modes' larger epilogues; their panels are retired only by the next barrier
      x0[0] = FC_LDS16(ring + P0 + bx); x0[1] = FC_LDS16(ring + P0 + bx + 4096);
#pragma unroll
      for (int j = 0; j < 4; ++j) a0[j] = FC_LDS16(ring + P1 + ba + j * 4096);
    }
    after_epilogue = (ABL & kAblNoEpilogue) == 0;    // the epilogue's stores are what the longer wait counts
    t = next_interior(t + G);
  }
  FC_WAIT_VMCNT0();   // the trailing re-requests write LDS: they must land before the workgroup gives it back
  if constexpr ((ABL & kAblTimed) != 0) {
    if (a.cycles && lane == 0 && (wave & 3) == 0) {      // waves 0 and 4: the older and the younger wave of SIMD 0
      uint64_t* o = a.cycles + ((size_t)blockIdx.x * 2 + (wave >> 2)) * 4;
      o[0] = __builtin_readcyclecounter() - t_begin;
      o[1] = t_epilogue;
      o[2] = wall_clock64() - t_wall;
      o[3] = 0;
    }
  }
}

void launch_strips_interior_bf16(const StripArgs& a, hipStream_t s) {
  const int grid = a.ntiles < 256 ? a.ntiles : 256;
  if (a.square) hipLaunchKernelGGL((k_strips_bf16<2, 0>), dim3((unsigned)grid), dim3(512), 0, s, a);
  else if (a.colp) hipLaunchKernelGGL((k_strips_bf16<1, 0>), dim3((unsigned)grid), dim3(512), 0, s, a);
  else hipLaunchKernelGGL((k_strips_bf16<0, 0>), dim3((unsigned)grid), dim3(512), 0, s, a);
}

// Measurement variants of the plain mode (see kAbl*); false if `ablation` is none of those built.
bool launch_strips_measure_bf16(const StripArgs& a, int ablation, hipStream_t s) {
  const dim3 grid((unsigned)(a.ntiles < 256 ? a.ntiles : 256)), block(512);
  switch (ablation) {
    case 0: hipLaunchKernelGGL((k_strips_bf16<0, kAblTimed>), grid, block, 0, s, a); return true;
    case 1: hipLaunchKernelGGL((k_strips_bf16<0, kAblTimed | 1>), grid, block, 0, s, a); return true;
    case 2: hipLaunchKernelGGL((k_strips_bf16<0, kAblTimed | 2>), grid, block, 0, s, a); return true;
    case 3: hipLaunchKernelGGL((k_strips_bf16<0, kAblTimed | 3>), grid, block, 0, s, a); return true;
    case 4: hipLaunchKernelGGL((k_strips_bf16<0, kAblTimed | 4>), grid, block, 0, s, a); return true;
    case 7: hipLaunchKernelGGL((k_strips_bf16<0, kAblTimed | 7>), grid, block, 0, s, a); return true;
    default: return false;
  }
}

}  // namespace fc
