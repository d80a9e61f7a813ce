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
__host__ __device__ __forceinline__ int64_t strip_anchor_first(const StripArgs& a, int at) {
  const int64_t a0 = (int64_t)at * 256;
  return (a0 + 256 > a.b && a.b >= 256 && a.b % 32 == 0) ? a.b - 256 : a0;
}
__host__ __device__ __forceinline__ bool strip_tile_is_interior(const StripArgs& a, int64_t a0, int64_t c0) {
  return (a.off + a0 + 256 <= a.B) && (c0 + 256 <= a.B) && (a.d % 64 == 0) && (a.d >= 128);
}

void launch_strips_interior_bf16(const StripArgs& a, hipStream_t s);   // kernels_strips.hip

}  // namespace fc
