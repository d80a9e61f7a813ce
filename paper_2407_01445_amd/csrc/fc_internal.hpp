// Internal declarations shared by the translation units of libfastclip (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fastclip.h"

namespace fc {

typedef uint16_t bf16_t;  // raw bf16 bits in memory

constexpr int kTileContrasts = 256;  // contrast rows per workgroup tile of the strip kernel
constexpr int kMaxSplit = 64;

// State kernel: threads per anchor side that share the work of adding up that side's partial sums (a power of two up to
// 32, a quarter of the partial sums at most so that every thread has four loads of each quantity in flight); a block
// of 256 threads then finishes 128 / lanes anchors.
static inline int state_lanes(int nparts) {
  int lanes = 1;
  while (lanes < 32 && lanes * 8 <= nparts) lanes *= 2;
  return lanes;
}
static inline int state_blocks(int64_t b, int nparts) {
  const int per_block = 128 / state_lanes(nparts);
  return (int)((b + per_block - 1) / per_block);
}

static inline size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

// One split's partial result of the contraction is kept as whole 256 x 256 tiles, each laid out as
// [64 groups of 4 rows][256 columns][4 rows] (tile = (n / 256) * tiles_m + m / 256): floats per tile, and per split
// for b rows of width d.
constexpr size_t kPartialTileFloats = 256 * 256;
__host__ __device__ static inline size_t partial_split_floats(int64_t b, int64_t d) {
  return (size_t)((b + 255) / 256) * (size_t)((d + 255) / 256) * kPartialTileFloats;
}

// Where everything lives inside the caller's workspace (byte offsets, 256-byte aligned).
struct Layout {
  int64_t B, b, off, d, N;
  int bf16;          // 1: MFMA path, 0: fp32 accuracy path
  int nparts;        // partial row sums per anchor and quantity written by the strip phase
  int64_t bstride;   // anchors padded to whole tiles of 256 (stride of the per-anchor arrays)
  int64_t ldE;       // contrast columns of the stored exp strips (MFMA path: multiple of 64; fp32 path: B)
  int nsplit;        // split of the contraction over its column range
  int64_t kslice;    // 32-deep stages per split
  int nstate_blocks; // scalar partials: one per block of the state kernel, or per diagonal block of the fused fold
  int fused_state;   // 1: MFMA path, few anchors and few partial sums: the fold kernel runs the state phase itself
  int gathered;      // 1: contrast-side estimator over every global anchor (FASTCLIP_GATHERED_STATE and b < B)
  int fine;          // 1: MFMA path on fine tiles (kernels_fine.hip): 128 x 128 strip tiles, 64 x 64 output tiles of the
                     //    contraction; nparts counts 128-column tiles, nsplit / kslice count 64-deep stages, and with one
                     //    split there are no partial results
  int t128;          // 1: MFMA path on 128 x 128 tiles (kernels_tiles128.hip); nparts counts 128-column tiles, nsplit /
                     //    kslice count 32-deep stages, and with one split there are no partial results
  int square;        // 1: MFMA path, b == B: the similarity matrix is formed once (F[0] holds
                     //    l2(j, p) in the layout of E[0] until the fold transposes it into E[1])
  int64_t ncol;      // gathered: entries per column-parameter array (B rounded up to whole 256-column tiles)
  size_t diag, tau1, tau2, k1, k2;   // float[bstride]
  size_t uold1, uold2;               // float[bstride]: u^t of the batch's samples (gathered with the temperatures)
  size_t sums;                       // float[4][nparts][bstride]: sum e1, sum x1 e1, sum e2, sum x2 e2
  size_t c1, c2, dcoef;              // float[bstride]
  size_t red;                        // double[nstate_blocks][2]
  size_t E[2];                       // fp32 path: float [b][ldE]; MFMA path: fragment-ordered bf16 strips
  size_t Opart[2];                   // float [nsplit][partial_split_floats(b, d)]   (MFMA path)
  // gathered: per global row j (= contrast column of the strips) and side s, in tiles of 256 columns
  // [s][tile][4][256]: log2(e)/tau_j, s_jj log2(e)/tau_j, c_j (0 for local rows and beyond B), unused.
  // Side 0 describes the text anchors j (l2(j, .), weights of d_img), side 1 the image anchors (l1(j, .), d_txt).
  size_t colp;
  size_t F[2];                       // gathered: the second stored strip c_j l(j, p_r), same form as E, folded into E
                                     // after the state phase (MFMA path) or summed directly (fp32 path)
  size_t total;
};

fastclip_status validate(const fastclip_config* cfg, const fastclip_buffers* bufs);
void make_layout(const fastclip_config& cfg, Layout* L);

// ---- kernel launchers (each enqueues on `s` and returns; errors are read by the caller
//      through hipGetLastError) -----------------------------------------------------------
// Proc. "parameter_update" for a temperature, as the kernels take it (bias corrections formed on the host).
struct TauUpd {
  int optimizer;      // 0: no update
  float lr, beta1, beta2, eps, corr1, corr2, tau_min, drop_below, drop_factor;
  int64_t stride;     // elements between consecutive samples in the per-sample arrays
};
fastclip_status validate_tau_update(int32_t version, const fastclip_tau_update* upd, const fastclip_tau_state* st);
TauUpd make_tau_upd(const fastclip_tau_update& upd);

struct StepCtx {
  fastclip_config cfg;
  fastclip_buffers buf;
  Layout L;
  char* ws;
  hipStream_t s;
  TauUpd tau_upd;            // optimizer == 0 unless called through fastclip_step_update_tau
  fastclip_tau_state tau_st;
};

void launch_prep(const StepCtx& c);            // s_ii, temperature gather / broadcast
void launch_prep_cols(const StepCtx& c);       // gathered: s_jj, temperature and coefficient of every global anchor
void launch_strips_f32(const StepCtx& c);      // accuracy path: exp strips + row sums
void launch_strips_bf16(const StepCtx& c);     // MFMA path: exp strips + row sums
void launch_state(const StepCtx& c);           // Eq. 1, coefficients, scalar partials
void launch_state_phase(const fastclip_config& cfg, const fastclip_buffers& buf, const TauUpd& upd,
                        const fastclip_tau_state& tst, const float* sums, float* coef, double* red, int nblocks,
                        hipStream_t s);    // the state phase on its own, one partial sum per anchor and quantity
bool state_records_are_canonical(const float* u_img, const float* u_txt, const fastclip_tau_state& t, int64_t stride);
void launch_grad_f32(const StepCtx& c);        // accuracy path: gradients + scalars
void launch_fold_bf16(const StepCtx& c);       // MFMA path: local contrast-side weights folded into the strips
void launch_contract_bf16(const StepCtx& c);   // MFMA path: strips x X contractions
void launch_strips_fine_bf16(const StepCtx& c);    // MFMA path, fine tiles: exp strips + row sums
void launch_contract_fine_bf16(const StepCtx& c);  // MFMA path, fine tiles: contractions, outputs and scalars
void launch_strips_t128_bf16(const StepCtx& c);    // MFMA path, 128 x 128 tiles: exp strips + row sums
void launch_contract_t128_bf16(const StepCtx& c);  // MFMA path, 128 x 128 tiles: contractions, outputs and scalars
void launch_norm_backward_bf16(const StepCtx& c);  // MFMA path: gradients through the L2 normalisation, if asked for
void launch_finalize_bf16(const StepCtx& c);   // MFMA path: combine + scalars

void launch_normalize_rows(const void* raw, int raw_bf16, int64_t ld_raw, int64_t b, int64_t d, void* unit, int unit_bf16,
                           int64_t ld_unit, float* norm, hipStream_t s);
void launch_record_rmw(const int64_t* idx, int64_t n, float* rec, int64_t stride, hipStream_t s);    // measurement only
bool launch_strips_measure(const StepCtx& c, int ablation, uint64_t* cycles);   // measurement only; false: not applicable
void launch_mfma_ceiling(int workgroups, int iters, uint64_t* out, float* sink, hipStream_t s);   // measurement only

void launch_state_flat(const int64_t* idx, int64_t n, int64_t stride, float gamma, float M,
                       const float* sum_img, const float* sum_txt, float* u_img, float* u_txt,
                       float* u_new_img, float* u_new_txt, hipStream_t s);
void launch_check_indices(const int64_t* idx, int64_t b, int64_t N, void* ws, hipStream_t s);
void launch_tau_scalar(const TauUpd& u, const fastclip_tau_state& st, const float* d_tau, hipStream_t s);
void launch_tau_sparse(const TauUpd& u, const fastclip_tau_state& st, const int64_t* idx, int64_t b,
                       const float* d_tau_img, const float* d_tau_txt, hipStream_t s);

}  // namespace fc
