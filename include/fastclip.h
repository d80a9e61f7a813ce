/*
 * fastclip.h - C ABI of the MI355X (gfx950) FCCO global-contrastive-loss step.
 *
 * One call of fastclip_step() is one worker's share of one FastCLIP iteration:
 * Alg. 1 line 6 (the mini-batch contrastive terms g1, g2 of Proc. 1), line 7 (the
 * moving-average update of the per-sample estimators u, Eq. 1), line 9 (the gradient
 * estimator of Proc. 2, Eqs. 2-7, here with respect to the local embedding rows) and the
 * gradient half of line 12 (the temperature gradients, Eqs. 8-10).
 *
 * Conventions
 *   - Every pointer in fastclip_buffers and every `workspace` is DEVICE memory owned by
 *     the caller.  The library never allocates, frees, or keeps state between calls.
 *   - `stream` is a hipStream_t passed as void*.  All work is enqueued on it; no call
 *     synchronises except where stated.  Outputs are valid once the stream has reached
 *     the end of the call.
 *   - Host-checkable errors are reported before anything is launched and leave every
 *     buffer untouched.
 *   - Matrices are row-major.  B = rows of the gathered global batch, b = local anchors,
 *     which are the global rows off .. off+b-1; M = B-1.  Local anchor r is dataset sample
 *     idx[r].  Similarities are plain dot products of the rows as given (the caller
 *     normalises); gradients are with respect to those rows.
 */
#ifndef FASTCLIP_H
#define FASTCLIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FASTCLIP_OK = 0,
  FASTCLIP_ERR_NULL = 1,        /* a required pointer is NULL */
  FASTCLIP_ERR_SHAPE = 2,       /* B<2, b<1, off<0, off+b>B, d<1, ld<d, N<1, b>N, state_stride outside [1,64], bad struct_size, unknown flag */
  FASTCLIP_ERR_VALUE = 3,       /* gamma not in (0,1], eps<0, NaN scalar, unknown version or dtype */
  FASTCLIP_ERR_WORKSPACE = 4,   /* workspace_bytes smaller than fastclip_workspace_bytes() */
  FASTCLIP_ERR_UNSUPPORTED = 5, /* bf16 path: d or a row stride not a multiple of 8, a matrix base not
                                   16-byte aligned, B + b or a row stride above 2^22; any path: B, b or d
                                   above 2^24, a row stride above 2^30, d_img / d_txt not 16-byte aligned */
  FASTCLIP_ERR_LAUNCH = 6,      /* the HIP runtime reported an error */
  FASTCLIP_ERR_INDEX = 7        /* fastclip_check_indices: out-of-range or repeated index */
} fastclip_status;

/* Temperature scheme / loss (Sec. 4 "The Temperature Parameter Updates"):
 *   V0  GCL without its leading tau, learnable global tau      (Eqs. 4, 5, 8)
 *   V1  GCL, constant global tau                               (Eqs. 2, 3)
 *   V2  RGCL, one learnable tau per sample and side            (Eqs. 6, 7, 9)
 *   V3  RGCL-g, learnable global tau                           (Eqs. 2, 3, 10)          */
typedef enum { FASTCLIP_V0 = 0, FASTCLIP_V1 = 1, FASTCLIP_V2 = 2, FASTCLIP_V3 = 3 } fastclip_version_t;

/* Embedding storage type.  F32: accuracy path (fp32 rows; dot products, the sums over the contrasts, the gradient
 * sums, the logarithms and the sums behind loss and d_tau are carried in fp64; what is stored between the phases
 * - exponentials, row sums, u, coefficients - and every output is fp32).
 * BF16: MFMA path (bf16 rows, fp32 accumulation; exp values are rounded to bf16 only
 * where they are operands of the gradient contractions). */
typedef enum { FASTCLIP_F32 = 0, FASTCLIP_BF16 = 1 } fastclip_dtype;

/* fastclip_config.flags.
 * FASTCLIP_GATHERED_STATE: the caller supplies u^{t+1} of EVERY row of the global batch as
 * gathered from all workers (Alg. 1 line 8; u_glob_img / u_glob_txt, and for V2 the rows'
 * temperatures tau_glob_img / tau_glob_txt).  The contrast-side estimator (Eq. 3, 5, 7) then
 * runs over every global anchor i, so that d_img / d_txt are worker k's complete
 * G_{w,a,k} + G_{w,b,k} with respect to its rows; without the flag only the anchors i in B_k
 * enter it.  A worker obtains the arrays by running the step of its own anchors first
 * (u_new_img / u_new_txt) and gathering; on a single GPU holding the whole batch (b == B) the
 * flag changes nothing and the arrays are not read. */
#define FASTCLIP_GATHERED_STATE 1
/* FASTCLIP_FINE_TILES (opt-in, bf16 path without gathered state, fewer than 192 large strip tiles): an older form of the
 * small-tile path: strips on 128 x 128 tiles staged through registers, contraction on 64 x 64 output tiles finished in
 * place when the column range needs no split.  Kept because its contraction is the faster one where the whole batch is
 * local and small (b = B = 1024); the library never chooses it by itself.  Same results up to summation order. */
#define FASTCLIP_FINE_TILES 2
/* FASTCLIP_SINGLE_PASS (bf16 path, b == B): form the similarity matrix ONCE whatever the batch size: with the whole batch
 * local the text strip is the transpose of the image strip, so every dot product yields both exponentials (Proc. 1 with
 * k = K = 1).  Without the flag the library does so when it pays (more 256 x 256 tiles than compute units) and forms the
 * two strips separately below that, where twice the workgroups finish sooner.  Same results up to summation order.
 * Ignored when b < B or on the fp32 path. */
#define FASTCLIP_SINGLE_PASS 4
/* Tile size of the bf16 path.  By default the library chooses: batches whose 256 x 256 strip tiles would occupy at most
 * half of the compute units (2 ceil(b/256) ceil(B/256) <= 128; not with gathered state, not in the single-pass form) run
 * the strip phase on 128 x 128 tiles and the contraction on 128 x 128 output tiles - four times as many workgroups, two
 * per compute unit, and an output tile whose column range needs no split is finished in place (no partial results, no
 * finalize kernel); everything else runs on 256 x 256 tiles.  FASTCLIP_TILES_128 asks for the small tiles wherever they
 * apply (up to 191 large tiles), FASTCLIP_TILES_256 for the large ones always; both together are an error.  Same results
 * up to summation order. */
#define FASTCLIP_TILES_128 8
#define FASTCLIP_TILES_256 16

typedef struct {
  uint32_t struct_size;      /* sizeof(fastclip_config) */
  int32_t  version;          /* fastclip_version_t */
  int32_t  emb_dtype;        /* fastclip_dtype */
  int32_t  flags;            /* 0 or an OR of the FASTCLIP_* flags above; any other bit is an error */
  int64_t  B, b, off, d;     /* global rows, local anchors, first local row, embedding width */
  int64_t  ld_img, ld_txt;   /* row strides of img_glob / txt_glob in elements, >= d */
  int64_t  N;                /* samples in the state arrays */
  int64_t  state_stride;     /* elements between the entries of consecutive samples in EVERY per-sample state array
                                (u_img, u_txt, tau_img, tau_txt; with fastclip_step_update_tau also the temperatures'
                                moments).  1: dense arrays of N floats.  S > 1: the arrays are fields of N records of
                                S floats each (pass the address of the field in record 0), so that everything the
                                method keeps for a sample lies in one memory line and one line is moved per
                                sample instead of one per array.  1 <= S <= 64 */
  float    gamma;            /* inner learning rate of Eq. 1, in (0, 1] */
  float    eps;              /* the small constant inside log(eps + g) */
  float    rho;              /* RGCL / RGCL-g hyper-parameter (V2, V3) */
  float    tau_grad_scale;   /* V2: factor in front of Eq. 9 (the paper prints 1/|S|) */
} fastclip_config;

typedef struct {
  const void*    img_glob;   /* [B, ld_img] image embeddings of the global batch */
  const void*    txt_glob;   /* [B, ld_txt] text embeddings of the global batch */
  const int64_t* idx;        /* [b] dataset indices of the local anchors, in [0,N), distinct */
  float*         u_img;      /* [N] in/out: u_1 of Eq. 1.  A stored 0.0f means "never visited":
                                the first visit stores g whatever gamma is */
  float*         u_txt;      /* [N] in/out: u_2 */
  const float*   tau;        /* [1] global temperature, read on the device (V0, V1, V3) */
  const float*   tau_img;    /* [N] per-sample temperatures tau_1 (V2); never written */
  const float*   tau_txt;    /* [N] per-sample temperatures tau_2 (V2) */
  float*         d_img;      /* [b, d] out: gradient w.r.t. the local image rows, fully overwritten */
  float*         d_txt;      /* [b, d] out: gradient w.r.t. the local text rows */
  float*         loss;       /* [1] out: local-batch objective with g replaced by u^{t+1} */
  float*         d_tau;      /* [1] out: Eq. 8 (V0) / Eq. 10 (V3); required for V0 and V3 */
  float*         d_tau_img;  /* [b] out, batch order: Eq. 9 first line (V2) */
  float*         d_tau_txt;  /* [b] out: Eq. 9 second line (V2) */
  float*         g_img;      /* [b] out, optional (NULL to skip): g_1 of Proc. 1 */
  float*         g_txt;      /* [b] out, optional: g_2 */
  float*         u_new_img;  /* [b] out, optional: u_1^{t+1} of the local anchors in batch order
                                (what a multi-worker caller would All_Gather, Alg. 1 line 8) */
  float*         u_new_txt;  /* [b] out, optional */
  const float*   u_glob_img; /* [B] FASTCLIP_GATHERED_STATE: u_1^{t+1} of every global row, > 0 (or eps > 0);
                                the entries of the local rows off .. off+b-1 are ignored (this call's own
                                new values are used).  Never written */
  const float*   u_glob_txt; /* [B] likewise u_2^{t+1} */
  const float*   tau_glob_img; /* [B] FASTCLIP_GATHERED_STATE with V2: tau_1 of every global row (local entries
                                  ignored); NULL otherwise */
  const float*   tau_glob_txt; /* [B] likewise tau_2 */
  const float*   norm_img;   /* [b] optional (both or neither): the rows of img_glob / txt_glob are L2-normalised encoder
                                outputs (cosine similarity, Sec. 3) and norm_img[r] is the norm that local image row r
                                had before.  d_img / d_txt are then gradients with respect to the rows BEFORE
                                normalisation: (d - e (e . d)) / norm, e = the normalised row as given */
  const float*   norm_txt;   /* [b] likewise for the local text rows */
} fastclip_buffers;

/* Bytes of device workspace fastclip_step needs for this configuration; 0 if the
 * configuration is invalid.  Pure host function. */
size_t fastclip_workspace_bytes(const fastclip_config* cfg);

/* How the library will run this configuration (pure host function; FASTCLIP_OK or the status fastclip_validate(cfg, NULL)
 * gives, then *plan is untouched).  For callers that want to know which kernels a profile will show and for the
 * benchmark's labels; nothing in it has to be passed back. */
typedef struct {
  int32_t tile;          /* rows of a strip tile on the bf16 path: 256, 128, or 64 for FASTCLIP_FINE_TILES (whose strip tiles
                            are 128 x 128 and output tiles 64 x 64); 0 on the fp32 path */
  int32_t single_pass;   /* 1: b == B and the similarity matrix is formed once */
  int32_t gathered;      /* 1: the contrast side runs over every global anchor (flag set and b < B) */
  int32_t fused_state;   /* 1: the state phase runs inside the fold kernel (few anchors, few partial sums) */
  int32_t nsplit;        /* splits of the contraction's column range; 1 on the small-tile paths: tiles finished in place */
  int32_t nparts;        /* partial sums per anchor and quantity that the strip phase leaves to the state phase */
} fastclip_plan;
fastclip_status fastclip_describe(const fastclip_config* cfg, fastclip_plan* plan);

/* Validate a configuration (and, if bufs != NULL, the pointers it requires) exactly as
 * fastclip_step does, without launching anything.  Pure host function. */
fastclip_status fastclip_validate(const fastclip_config* cfg, const fastclip_buffers* bufs);

/* The step (Alg. 1 lines 6, 7, 9 and the gradient of line 12; Proc. 1, Eq. 1, Proc. 2,
 * Eqs. 2-10).  Preconditions that cannot be checked without a device round trip and are
 * therefore the caller's: idx values distinct and in range (see fastclip_check_indices),
 * temperatures >= 0.023 for unit-norm rows so that exp((s - s_ii)/tau) stays finite in fp32.
 * `workspace` must be 256-byte aligned.  Asynchronous on `stream`. */
fastclip_status fastclip_step(const fastclip_config* cfg, const fastclip_buffers* bufs,
                              void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or hold a workspace of their own (code under HIP graph capture,
 * serving loops, harnesses that forbid hipMalloc): the same step as fastclip_step, same kernels, same results, with
 * its workspace in a static array of FASTCLIP_STATIC_SCRATCH_BYTES of device memory that is part of the library's
 * code object.  Every GPU the library runs on holds one such array from the first kernel launch until the process
 * ends.  The call allocates and frees nothing (no hipMalloc / hipFree, no allocating library routine); on its first
 * call on a device it looks the array's device address up (hipGetSymbolAddress) and keeps it.
 *   - A configuration whose fastclip_workspace_bytes() exceeds FASTCLIP_STATIC_SCRATCH_BYTES is refused with
 *     FASTCLIP_ERR_WORKSPACE before anything is launched (64 MiB holds the paper's own shapes: up to 640 local
 *     anchors of a global batch of 5120 at width 512, and 1024 x 1024 x 512 or 256 of 8192 x 512).
 *   - All calls on one GPU share that GPU's array, whatever their stream: calls that overlap in time on one GPU race
 *     on it.  Calls that follow each other on one stream, or are ordered by events, are safe.  The array keeps the
 *     last call's contents; the step reads nothing from its workspace that it has not written in the same call, so
 *     nothing needs clearing in between.
 *   - The current device must be the one `stream` belongs to.
 * Errors, outputs and asynchrony are those of fastclip_step. */
#define FASTCLIP_STATIC_SCRATCH_BYTES (64u << 20)
fastclip_status fastclip_step_static(const fastclip_config* cfg, const fastclip_buffers* bufs, void* stream);

/* The forward half of the cosine similarity of Sec. 3: the b raw encoder rows of one worker become the unit rows
 * e / |e| that fastclip_step takes and the norms |e| that it takes as norm_img / norm_txt to return gradients with
 * respect to the raw rows.  A worker calls it on its own b image rows and b text rows with `unit` pointing at its slice
 * (row off) of img_glob / txt_glob, before the rows are gathered.
 *   raw   [b, ld_raw] device, raw_dtype FASTCLIP_F32 or FASTCLIP_BF16;  unit  [b, ld_unit] device out, unit_dtype likewise
 *         (the emb_dtype of the step that follows);  norm  [b] device out, fp32.
 * The squares are summed in fp64; each element is divided in fp32 and rounded once to unit_dtype.  A row of zeros
 * yields a row of zeros and norm 0 (the step's gradient through such a row is not defined).  unit may be raw itself
 * (same type and stride): rows are then normalised in place.  Asynchronous on `stream`; b == 0 does nothing. */
fastclip_status fastclip_normalize_rows(const void* raw, int32_t raw_dtype, int64_t ld_raw, int64_t b, int64_t d,
                                        void* unit, int32_t unit_dtype, int64_t ld_unit, float* norm, void* stream);

/* Same step, but brackets every kernel with HIP events on `stream`, synchronises, and
 * writes the duration of each phase in milliseconds to phase_ms[0 .. FASTCLIP_N_PHASES-1]
 * (host memory; phases that a path does not run are reported as 0).  Measurement aid:
 * it creates and destroys events and blocks the calling thread. */
#define FASTCLIP_N_PHASES 8
#define FASTCLIP_PHASE_PREP 0      /* s_ii and temperature gather */
#define FASTCLIP_PHASE_STRIPS 1    /* similarity strips + exp + row sums (Proc. 1) */
#define FASTCLIP_PHASE_STATE 2     /* Eq. 1 update / scatter, coefficients, scalars (0 where the bf16 path runs it inside the next phase) */
#define FASTCLIP_PHASE_LOCAL 3     /* bf16 path: contrast-side weights of Eqs. 3/5/7 folded into the stored strips (+ the state phase for small batches) */
#define FASTCLIP_PHASE_CONTRACT 4  /* gradient contractions of Eqs. 2-7 */
#define FASTCLIP_PHASE_FINALIZE 5  /* split sums, scaling, diagonal terms, loss and tau gradient */
fastclip_status fastclip_step_timed(const fastclip_config* cfg, const fastclip_buffers* bufs,
                                    void* workspace, size_t workspace_bytes, void* stream,
                                    float* phase_ms);
const char* fastclip_phase_name(int phase);

/* Measurement aid, not part of the step: what the matrix cores deliver in the launch shape of the strip kernel when
 * nothing else is in the way.  `workgroups` workgroups of 8 wavefronts (two per SIMD, 128 accumulator registers each)
 * issue iters x 8 independent MFMAs 32x32x16 bf16 on pseudo-random register operands: no memory traffic, no LDS, no
 * barrier.  The kernel is launched twice, the second launch is timed with HIP events on `stream`; the call creates and
 * destroys two events, allocates a few KiB of host memory, SYNCHRONISES the stream and copies the wavefronts' counters
 * back.  ms: duration of the timed launch.  stats[0] = flop of that launch, stats[1] = mean shader cycles of a
 * wavefront's loop, stats[2] = shader clock in GHz while the loops ran (cycles over the 100 MHz wall clock),
 * stats[3] = cycles per MFMA as one wavefront sees them (64 = two wavefronts sharing a SIMD at the nominal 32).
 * workspace: workgroups x 128 + 2048 bytes of device memory, 256-byte aligned. */
fastclip_status fastclip_measure_mfma_ceiling(int32_t workgroups, int32_t iters, void* workspace,
                                              size_t workspace_bytes, void* stream, float* ms, double* stats);

/* Measurement aid, not part of the step: the whole-tile strip kernel (plain mode: bf16, every 256 x 256 tile whole, no
 * gathered state, not the single-pass form of b == B) with parts of it compiled out and per-wavefront cycle counters,
 * so that what bounds the kernel can be measured again after any change to it.  ablation: 0 the complete kernel;
 * 1 without the global -> LDS operand requests; 2 without the LDS operand reads of the main loop; 3 without both;
 * 4 without the epilogue (exponentials, sums, stores); 7 MFMAs and barriers only.  Every variant but 0 computes
 * nonsense and LEAVES THE WORKSPACE'S STRIPS AND SUMS UNDEFINED.  The call runs the prep kernel, launches the variant
 * once untimed and `reps` times between two HIP events, SYNCHRONISES the stream and reads the counters back (it creates
 * and destroys two events and allocates a few KiB of host memory).  workspace: fastclip_workspace_bytes(cfg) + 16 KiB.
 * ms: mean duration of a launch.  stats[0] / stats[1]: mean cycles from kernel entry to exit of the older / younger
 * wavefront of a SIMD; stats[2]: of which between a tile's last stage and the next tile (the epilogue and its
 * barriers); stats[3]: 64-deep stages per workgroup; stats[4]: shader clock in GHz while the kernel ran;
 * stats[5]: workgroups.  FASTCLIP_ERR_UNSUPPORTED where the layout is not the plain whole-tile one. */
fastclip_status fastclip_measure_strips(const fastclip_config* cfg, const fastclip_buffers* bufs, void* workspace,
                                        size_t workspace_bytes, void* stream, int32_t ablation, int32_t reps, float* ms,
                                        double* stats);

/* Measurement aid, not part of the step: the access pattern of the state phase on 32-byte records with nothing else in
 * the way.  For each of the n distinct indices idx[i] in [0, N) the first 32 bytes of record idx[i] (records of
 * record_floats floats, a multiple of 8, 32-byte aligned) are read, changed by one multiply-add per word and written
 * back, 16 bytes per lane by two neighbouring lanes: what the memory system delivers for random whole-sector
 * read-modify-writes, against which the state kernel's rate is read.  CHANGES the records.  Asynchronous on `stream`. */
fastclip_status fastclip_measure_record_rmw(const int64_t* idx, int64_t n, int64_t N, float* records,
                                            int64_t record_floats, void* stream);

/* ---- temperature update (Alg. 1 line 12: Proc. "temperature_update" with Proc. "parameter_update", weight decay 0) ----
 * V1 keeps tau.  V0 / V3 step the global tau with d_tau (Eq. 8 / Eq. 10).  V2 steps tau_1[idx[r]], tau_2[idx[r]] with
 * d_tau_img[r], d_tau_txt[r] (Eq. 9) and touches no other entry.  After the step the temperature is projected onto
 * tau >= tau_min (the constraint tau >= tau_0 of the objectives).  lr_drop_below / lr_drop_factor: the learning rate is
 * multiplied by lr_drop_factor for a temperature that is below lr_drop_below before the step (Sec. 4 / App. B: a third
 * once tau < 0.03 for V3); set lr_drop_below = 0 to switch that off. */
typedef enum {
  FASTCLIP_TAU_SGDM = 1,   /* m = beta1 m + G;  tau -= lr m                         (beta1 = momentum) */
  FASTCLIP_TAU_LAMB = 2,   /* with the layer factor alpha = 1 prescribed for tau: identical to AdamW */
  FASTCLIP_TAU_LION = 3,   /* c = beta1 m + (1-beta1) G;  m = beta2 m + (1-beta2) G;  tau -= lr sign(c) */
  FASTCLIP_TAU_ADAMW = 4   /* m, v moments with bias correction 1 - beta^step;  tau -= lr m^ / (sqrt(v^) + eps) */
} fastclip_tau_optimizer;

typedef struct {             /* host scalars */
  uint32_t struct_size;      /* sizeof(fastclip_tau_update) */
  int32_t  optimizer;        /* fastclip_tau_optimizer */
  int64_t  step;             /* t + 1 >= 1: exponent of the bias corrections */
  float    lr, beta1, beta2, eps;
  float    tau_min;
  float    lr_drop_below, lr_drop_factor;
  int32_t  state_stride;     /* V2: elements between consecutive samples in the [N] arrays of fastclip_tau_state
                                (see fastclip_config.state_stride); 0 or 1 = dense */
} fastclip_tau_update;

typedef struct {             /* DEVICE memory owned by the caller, updated in place */
  float* tau;                /* [1]  V0, V3 */
  float* m;                  /* [1]  first-moment / momentum state of tau */
  float* v;                  /* [1]  second-moment state (AdamW, LAMB; may be NULL otherwise) */
  float* tau_img;            /* [N]  V2: tau_1 */
  float* tau_txt;            /* [N]  V2: tau_2 */
  float* m_img;  float* v_img;   /* [N] states of tau_1 (v_* may be NULL for SGDM / LION) */
  float* m_txt;  float* v_txt;   /* [N] states of tau_2 */
} fastclip_tau_state;

/* The update alone, from gradients that a previous fastclip_step wrote (a caller with several workers averages
 * d_tau over the workers in between; d_tau_img / d_tau_txt need no averaging).  d_tau: [1] device (V0, V3);
 * d_tau_img, d_tau_txt: [b] device, batch order, with idx [b] (V2).  Asynchronous on `stream`; V1 returns
 * FASTCLIP_OK and does nothing. */
fastclip_status fastclip_temperature_update(int32_t version, const fastclip_tau_update* upd,
                                            const fastclip_tau_state* state, const int64_t* idx, int64_t b,
                                            int64_t N, const float* d_tau, const float* d_tau_img,
                                            const float* d_tau_txt, void* stream);

/* fastclip_step followed by the temperature update of the same iteration, for a single worker (no averaging of
 * d_tau in between).  For V2 the update is part of the state phase: the kernel that gathers u by idx and scatters
 * u^{t+1} also steps tau_1, tau_2 and their moments at the same indices.  bufs->tau (V0, V3) must be state->tau,
 * bufs->tau_img / tau_txt (V2) must be state->tau_img / tau_txt; the step itself uses the temperatures as they were
 * before the call, and every output of fastclip_step is produced as usual. */
fastclip_status fastclip_step_update_tau(const fastclip_config* cfg, const fastclip_buffers* bufs,
                                         const fastclip_tau_update* upd, const fastclip_tau_state* state,
                                         void* workspace, size_t workspace_bytes, void* stream);

/* The state phase of fastclip_step on its own (Alg. 1 line 7, the per-anchor half of lines 9 and 12: Eq. 1 by dataset
 * index, the coefficients of Eqs. 2-7, Eq. 9, loss and Eqs. 8 / 10, and with upd / state the temperature update of the
 * same samples), for cfg->b anchors whose sums over the contrasts are given.  It runs the kernel and the per-anchor code
 * that the step runs for this phase, and exists to measure that code against the HBM roofline on many indices and to
 * test it alone.
 *   cfg    used: version, emb_dtype (FASTCLIP_F32 selects the fp64 logarithms of the accuracy path), B (only through
 *          M = B - 1; b may exceed it here), b <= 2^24 anchors, N, state_stride, gamma, eps, rho, tau_grad_scale
 *   bufs   used: idx, u_img, u_txt (updated in place), tau or tau_img / tau_txt, loss, d_tau or d_tau_img / d_tau_txt,
 *          and the optional g_img, g_txt, u_new_img, u_new_txt; the embedding pointers are not read
 *   upd, state   both NULL: no temperature update; otherwise as for fastclip_step_update_tau
 *   sums   [4][b] device, read only: per anchor the sum of l1, of (s - s_ii) l1, of l2, of (s - s_ii) l2 over B_{i-}
 *   coef   [3][b] device, out: c_1, c_2 (the factors 1 / (|B_k| |B_i-| (eps + u^{t+1})) of Eqs. 2-7, divided by tau for
 *          V0) and c_1 M g_1 + c_2 M g_2
 * Records: when the eight per-sample arrays of V2 with the temperature update are the fields
 * {u_img, tau_img, m_img, v_img, u_txt, tau_txt, m_txt, v_txt}, in this order, of records of state_stride floats with
 * state_stride a multiple of 8 and u_img 32-byte aligned, every sample is read and written as whole 32-byte sectors
 * (16 bytes per side and lane); fastclip_step_update_tau takes the same path.  Any other layout is moved field by field.
 * workspace: fastclip_state_phase_workspace_bytes(b) bytes, 256-byte aligned.  Asynchronous on `stream`. */
size_t fastclip_state_phase_workspace_bytes(int64_t b);
fastclip_status fastclip_state_phase(const fastclip_config* cfg, const fastclip_buffers* bufs,
                                     const fastclip_tau_update* upd, const fastclip_tau_state* state,
                                     const float* sums, float* coef, void* workspace, size_t workspace_bytes,
                                     void* stream);

/* Eq. 1 alone, for n anchors whose exp-sums are already known (the state phase of
 * fastclip_step run on its own; used to measure the gather/update/scatter kernel on many
 * indices).  sum_img[r] / sum_txt[r] hold M * g_1 / M * g_2 of anchor r (device, [n]);
 * u_img/u_txt [N] are updated in place at idx; u_new_img / u_new_txt [n] receive the new
 * values in batch order.  M = the divisor |B_{i-}|.  Asynchronous on `stream`.  idx holds n distinct values
 * in [0, N) (not checked on the device); n > N cannot satisfy that and returns FASTCLIP_ERR_SHAPE. */
fastclip_status fastclip_state_update(const int64_t* idx, int64_t n, int64_t N, float gamma, float M,
                                      const float* sum_img, const float* sum_txt,
                                      float* u_img, float* u_txt,
                                      float* u_new_img, float* u_new_txt, void* stream);
/* The same with u_img / u_txt as fields of N records of state_stride floats (fastclip_config.state_stride):
 * sample i is u_img[i * state_stride], u_txt[i * state_stride].  With both fields in one record a sample costs one
 * memory line instead of two. */
fastclip_status fastclip_state_update_strided(const int64_t* idx, int64_t n, int64_t N, int64_t state_stride,
                                              float gamma, float M, const float* sum_img, const float* sum_txt,
                                              float* u_img, float* u_txt, float* u_new_img, float* u_new_txt,
                                              void* stream);

/* Debug aid: checks on the device that idx[0..b) are distinct and inside [0, N).
 * Needs fastclip_check_indices_workspace_bytes(b) bytes of workspace.  SYNCHRONISES the
 * stream.  Returns FASTCLIP_OK or FASTCLIP_ERR_INDEX. */
size_t fastclip_check_indices_workspace_bytes(int64_t b);
fastclip_status fastclip_check_indices(const int64_t* idx, int64_t b, int64_t N,
                                       void* workspace, size_t workspace_bytes, void* stream);

/* Cosine schedule of the inner learning rate (Sec. 4 "The Inner LR Schedule"):
 * epoch = t / iters_per_epoch; 0.5 (1 + cos(pi epoch / decay_epochs)) (1 - gamma_min) + gamma_min
 * while epoch < decay_epochs, gamma_min afterwards.  Pure host function. */
float fastclip_gamma_cosine(int64_t t, int64_t iters_per_epoch, int64_t decay_epochs, float gamma_min);

const char* fastclip_status_string(fastclip_status s);

/* Text of the HIP error behind the most recent FASTCLIP_ERR_LAUNCH on the calling thread
 * ("no error" if there was none).  The string is static; pure host function. */
const char* fastclip_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FASTCLIP_H */
