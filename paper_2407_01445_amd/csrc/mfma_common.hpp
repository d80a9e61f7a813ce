// Types and device helpers shared by the MFMA translation units of libfastclip (gfx950, wave64).
#pragma once
#include "fc_internal.hpp"

namespace fc {


typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
typedef short v4s __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4s lds_v4s;

constexpr int BK = 32;                       // contraction depth of one LDS stage
constexpr int kOpBytes = 256 * BK * 2;       // one operand tile of a stage: 16 KiB
constexpr int kStageBytes = 2 * kOpBytes;    // 32 KiB
constexpr int kRingBytes = 5 * kStageBytes;  // 160 KiB: all of the LDS of a compute unit

#define FC_PIN() __builtin_amdgcn_sched_barrier(0)
#define FC_WAIT_VMCNT0() __builtin_amdgcn_s_waitcnt(0x0f70)
#define FC_WAIT_VMCNT8() __builtin_amdgcn_s_waitcnt(0x0f78)
#define FC_WAIT_VMCNT16() __builtin_amdgcn_s_waitcnt(0x4f70)
#define FC_WAIT_VMCNT20() __builtin_amdgcn_s_waitcnt(0x4f74)
#define FC_WAIT_VMCNT24() __builtin_amdgcn_s_waitcnt(0x4f78)

__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// 16 bytes per lane from global memory straight into LDS at lds_byte_addr + 16 * lane (wave-uniform address).
// Completion is tracked by vmcnt; the compiler does not see the LDS write, so every use below is fenced by an
// explicit s_waitcnt vmcnt + barrier.  M0 (the LDS base of the transfer) is written here and used by nothing else
// in these kernels.
// The source address is a wave-uniform base (kept in SGPRs) plus a per-lane 32-bit byte offset.
__device__ __forceinline__ void dma16(const void* uniform_base, uint32_t lane_byte_off, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_byte_off), "s"(uniform_base), "s"(__builtin_amdgcn_readfirstlane(lds_byte_addr))
               : "memory");
}
// Same for 4 bytes per lane (per-anchor scalars of the next tile).
__device__ __forceinline__ void dma4(const void* uniform_base, uint32_t lane_byte_off, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :
               : "v"(lane_byte_off), "s"(uniform_base), "s"(__builtin_amdgcn_readfirstlane(lds_byte_addr))
               : "memory");
}
__device__ __forceinline__ float bf2f(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }
__device__ __forceinline__ uint16_t f2bf(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }

// LDS has 64 banks of 4 bytes (256 bytes per cycle); a 16-byte-per-lane read is served 16 lanes at a time, an
// 8-byte-per-lane read 32 lanes at a time.
// LDS image of a K-contiguous operand tile (256 rows x 32 k, 64 bytes per row): 16-byte chunk c of row r sits at
// chunk position c ^ ((r >> 2) & 3): the 16 consecutive rows that one MFMA operand read touches per cycle then
// cover all 16 chunk slots of a 256-byte bank window.
__device__ __forceinline__ int rt_swz(int row) { return (row >> 2) & 3; }
__device__ __forceinline__ int rt_off(int row, int chunk) { return row * 64 + ((chunk ^ rt_swz(row)) << 4); }
// LDS image of a [32 k][256 n] tile of a row-major matrix (512 bytes per k row): 16-byte piece p of row k sits at
// piece position p ^ ((k & 3) << 2), so that the 4 rows x 64 bytes which a transposing read touches per cycle cover
// a whole bank window.
__device__ __forceinline__ int nt_swz(int k) { return (k & 3) << 2; }
__device__ __forceinline__ int nt_off(int k, int piece) { return k * 512 + ((piece ^ nt_swz(k)) << 4); }

// One accumulator element out of its AGPR at the point of use.  Left to itself the register allocator copies large
// parts of the accumulator block into VGPRs right after the main loop, which costs more VGPRs than there are.
__device__ __forceinline__ float acc_read(float in_agpr) {
  float x;
  asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(in_agpr));
  return x;
}
__device__ __forceinline__ bf16x8 join_halves(u32x2 lo, u32x2 hi) {
  const u32x4 r = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8, r);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  bf16x2 p;
  p[0] = (__bf16)lo;
  p[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, p);
}
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[4][4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
}

// Arguments of the strip kernels (Proc. 1: both b x B strips of one worker).
struct StripArgs {
  const bf16_t* anchors[2];     // first local row of the anchor side (image rows for strip 0, text rows for strip 1)
  const bf16_t* contrasts[2];   // row 0 of the contrast side (texts for strip 0, images for strip 1)
  int64_t ld_anchor[2], ld_contrast[2];
  const float* diag;            // s_pp per local anchor
  const float* kscale[2];       // log2(e) / tau of the anchor for each strip
  bf16_t* E[2];                 // Efrag per strip
  int64_t nCB;                  // column blocks (of 16) per anchor block in Efrag
  int64_t ldE;                  // contrast columns present in Efrag (multiple of 64, >= B)
  float* sums;                  // [4][nparts][bstride] out
  int nparts;
  int64_t bstride, b, B, d, off;
  int nAT, nCT, ntiles;
  // gathered state (Eqs. 3 / 5 / 7 over every global anchor), colp == nullptr otherwise
  const float* colp;            // [2][nCT][4][256]: per strip and contrast column j: log2(e)/tau_j, s_jj log2(e)/tau_j,
                                // c_j (0 where column j takes no part), unused
  bf16_t* F[2];                 // second stored strip c_j l(j, p_r), fragment order, nCBF column blocks per anchor block
  int64_t nCBF;
  // the whole batch is local and every tile is whole: only strip 0 is formed, l2(j, p) of the text anchors goes to
  // F[0] and their sums are taken down the columns
  int square;
  uint64_t* cycles;             // measurement variants only: [workgroup][wave 0 | wave 4][4] counters, else nullptr
};

// Which tiles go to the persistent kernel (unguarded direct-to-LDS loads), which to the guarded one.  The persistent
// kernel needs 256 rows of each operand to EXIST, not to be wanted: a last anchor tile with fewer than 256 local
// anchors is computed on the global rows that follow the local ones (off + a0 + 256 <= B) and what it produces for
// them lands in padding (strip rows and per-anchor slots beyond b) that nothing reads.  Only a tile whose rows would
// run past the end of the global batch, or a width that is not whole 64-deep stages, needs the guarded kernel.
// First local anchor of anchor tile `at`.  Tiles start every 256 anchors, except that a last tile with fewer than 256
// anchors left is moved back to end exactly at b when the 32-anchor blocks of the stored strips allow it (b >= 256,
// b % 32 == 0): it then recomputes some anchors of the tile before it - to the same bits, every anchor's values and
// sums depend on its row and on the contrast tile only - and is a whole tile on every worker, also the last one.
// Not when the similarity matrix is formed once (square): there the tiles also sum down their columns over the anchors,
// and an anchor computed twice would be counted twice.
__host__ __device__ __forceinline__ int64_t strip_anchor_first(const StripArgs& a, int at, bool square) {
  const int64_t a0 = (int64_t)at * 256;
  return (!square && a0 + 256 > a.b && a.b >= 256 && a.b % 32 == 0) ? a.b - 256 : a0;
}
__host__ __device__ __forceinline__ bool strip_tile_is_interior(const StripArgs& a, int64_t a0, int64_t c0) {
  return (a.off + a0 + 256 <= a.B) && (c0 + 256 <= a.B) && (a.d % 64 == 0) && (a.d >= 128);
}

// ----------------------------------------------------------------------------------------------------------------
// Epilogue of one wave of a strip tile whose accumulators are NI x NJ blocks of 32 x 32: accumulator (ti, tj, v) of
// lane (lr, hk) is contrast c0 + cw + ti 32 + 8 (v >> 2) + 4 hk + (v & 3), anchor a0 + aw + tj 32 + lr (c0 / a0: first
// contrast / anchor of the workgroup's tile, cw / aw: the wave's offset inside it; a0 + aw is a multiple of 32, c0 + cw
// of 16).  t = (s - s_pp) log2(e)/tau, l = 2^t; l goes to the fragment-ordered strip, the sums of l and of (s - s_pp) l
// over the wave's contrasts to sred_w[quantity][anchor inside the tile].  sk / sdiag: log2(e)/tau and s_pp of the
// tile's anchors.  GUARD: zero outside the batch and on the anchor's own column (B_{i-} excludes i).
template <bool GUARD, int NI, int NJ>
__device__ __forceinline__ void strip_epilogue(const StripArgs& a, f32x16 (&acc)[NI][NJ], const float* sk,
                                               const float* sdiag, float (*sred_w)[256], int strip, int64_t a0,
                                               int64_t c0, int cw, int aw, int lane) {
  const int lr = lane & 31, hk = lane >> 5;
  bf16_t* __restrict__ E = a.E[strip];
  // fragment (ab, cb) of this lane: E + ((ab nCB + cb) 64 + lane) 8; ab and cb are wave-uniform
  const int64_t ab0 = (a0 + aw) >> 5, cb0 = (c0 + cw) >> 4;
  const int B = (int)a.B, b = (int)a.b, off = (int)a.off;   // all below 2^24
  // gathered state: column parameters of this tile (log2(e)/tau_j, s_jj log2(e)/tau_j, c_j), second strip F
  const float* __restrict__ colp = a.colp ? a.colp + ((int64_t)strip * a.nCT + (c0 >> 8)) * 1024 : nullptr;
  bf16_t* __restrict__ F = a.F[strip];
#pragma unroll
  for (int tj = 0; tj < NJ; ++tj) {
    const int al = aw + tj * 32 + lr;
    const float kk = sk[al], dk = sdiag[al] * kk;   // log2(e)/tau and s_pp log2(e)/tau of this anchor
    const int anchor = (int)a0 + al;
    // 4 independent partial sums per quantity: a dependent VALU op issues only every ~36 cycles on a lone
    // wavefront, so one serial accumulation chain per sum would dominate this phase
    float sgv[4] = {0.f, 0.f, 0.f, 0.f}, stv[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ti = 0; ti < NI; ++ti) {
      const int crow = (int)c0 + cw + ti * 32 + 4 * hk;
      // groups of 4 accumulators (v = 4 g + q <-> contrast crow + 8 g + q), pinned apart to keep live ranges short
      uint32_t pk[8], pf[8];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float sv[4], t[4], e[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) sv[q] = acc_read(acc[ti][tj][4 * g + q]);
#pragma unroll
        for (int q = 0; q < 4; ++q) t[q] = fmaf(sv[q], kk, -dk);
#pragma unroll
        for (int q = 0; q < 4; ++q) e[q] = __builtin_amdgcn_exp2f(t[q]);
        if (colp) {   // wave-uniform
          const int cl = ((int)c0 & 255) + cw + ti * 32 + 4 * hk + 8 * g;   // column inside the 256-column parameter tile
          const float4 ck = *(const float4*)(colp + cl), cd = *(const float4*)(colp + 256 + cl),
                       cc = *(const float4*)(colp + 512 + cl);
          const float ckq[4] = {ck.x, ck.y, ck.z, ck.w}, cdq[4] = {cd.x, cd.y, cd.z, cd.w},
                      ccq[4] = {cc.x, cc.y, cc.z, cc.w};
          float f[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            f[q] = ccq[q] * __builtin_amdgcn_exp2f(fmaf(sv[q], ckq[q], -cdq[q]));
            if (GUARD) f[q] = anchor < b ? f[q] : 0.f;
          }
          pf[2 * g] = pack_bf16x2(f[0], f[1]);
          pf[2 * g + 1] = pack_bf16x2(f[2], f[3]);
        }
        if (GUARD) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int c = crow + 8 * g + q;
            const bool ok = (c < B) && (anchor < b) && (c != off + anchor);
            e[q] = ok ? e[q] : 0.f;
          }
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
        const int64_t cb = cb0 + 2 * ti + j;
        bf16_t* frag = E + ((ab0 + tj) * a.nCB + cb) * 512;   // wave-uniform
        const u32x4 w = {pk[4 * j], pk[4 * j + 1], pk[4 * j + 2], pk[4 * j + 3]};
        if (!GUARD || 16 * cb < a.ldE) *(u32x4*)(frag + lane * 8) = w;
        if (colp && (!GUARD || 16 * cb < a.ldE)) {
          const u32x4 wf = {pf[4 * j], pf[4 * j + 1], pf[4 * j + 2], pf[4 * j + 3]};
          *(u32x4*)(F + (((ab0 + tj) * a.nCBF + cb) * 64 + lane) * 8) = wf;
        }
      }
      FC_PIN();
    }
    const float sgl = (sgv[0] + sgv[1]) + (sgv[2] + sgv[3]);
    const float stl = (stv[0] + stv[1]) + (stv[2] + stv[3]);
    const float sg = sgl + __shfl_xor(sgl, 32);
    const float st = stl + __shfl_xor(stl, 32);
    if (hk == 0) {
      sred_w[0][al] = sg;
      sred_w[1][al] = kk > 0.f ? st * __builtin_amdgcn_rcpf(kk) : 0.f;   // sum of (s - s_pp) l
    }
  }
}

// Sum of v[i] over the 32 lanes that share (lane >> 5), for 16 values at once: each step halves the number of values
// a lane carries (the lower half of a lane pair keeps the first half of the values, the upper half the second), so
// 16 values cost 16 exchanges instead of 80.  On return v[0] of lane l is the total of value number (l & 31) >> 1.
template <int HALF, int MASK>
__device__ __forceinline__ void lanes32_halve(float (&v)[16], int lane) {
  const bool upper = (lane & MASK) != 0;
#pragma unroll
  for (int i = 0; i < HALF; ++i) {
    const float send = upper ? v[i] : v[i + HALF];
    const float keep = upper ? v[i + HALF] : v[i];
    v[i] = keep + __shfl_xor(send, MASK);
  }
}
__device__ __forceinline__ void lanes32_sum(float (&v)[16], int lane) {
  lanes32_halve<8, 16>(v, lane);
  lanes32_halve<4, 8>(v, lane);
  lanes32_halve<2, 4>(v, lane);
  lanes32_halve<1, 2>(v, lane);
  v[0] += __shfl_xor(v[0], 1);
}

void launch_strips_interior_bf16(const StripArgs& a, hipStream_t s);   // kernels_strips.hip
bool launch_strips_measure_bf16(const StripArgs& a, int ablation, hipStream_t s);   // kernels_strips.hip

}  // namespace fc
