// C ABI of libfastclip: argument validation, workspace carving, launch sequences.
// The arithmetic lives in the kernel translation units; nothing here runs on the CPU
// except checks, address arithmetic and the gamma schedule.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "fc_internal.hpp"

namespace fc {

static bool bad_float(float x) { return !(x == x) || isinf(x); }

static thread_local hipError_t g_last_hip_error = hipSuccess;
// Reads and clears the runtime's error state; remembers a failure for fastclip_last_hip_error.
static fastclip_status launch_status() {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return FASTCLIP_OK;
  g_last_hip_error = e;
  return FASTCLIP_ERR_LAUNCH;
}
static fastclip_status hip_failed(hipError_t e) {
  g_last_hip_error = e;
  return FASTCLIP_ERR_LAUNCH;
}

fastclip_status validate(const fastclip_config* cfg, const fastclip_buffers* bufs) {
  if (!cfg) return FASTCLIP_ERR_NULL;
  if (cfg->struct_size != sizeof(fastclip_config) || (cfg->flags & ~(FASTCLIP_GATHERED_STATE | FASTCLIP_FINE_TILES | FASTCLIP_SINGLE_PASS | FASTCLIP_TILES_128 | FASTCLIP_TILES_256)))
    return FASTCLIP_ERR_SHAPE;
  if (cfg->B < 2 || cfg->b < 1 || cfg->off < 0 || cfg->off + cfg->b > cfg->B || cfg->d < 1 ||
      cfg->ld_img < cfg->d || cfg->ld_txt < cfg->d || cfg->N < 1 || cfg->b > cfg->N || cfg->state_stride < 1 ||
      cfg->state_stride > 64)
    return FASTCLIP_ERR_SHAPE;
  if ((cfg->flags & FASTCLIP_TILES_128) && (cfg->flags & FASTCLIP_TILES_256)) return FASTCLIP_ERR_VALUE;
  if (cfg->version < FASTCLIP_V0 || cfg->version > FASTCLIP_V3) return FASTCLIP_ERR_VALUE;
  if (cfg->emb_dtype != FASTCLIP_F32 && cfg->emb_dtype != FASTCLIP_BF16) return FASTCLIP_ERR_VALUE;
  if (bad_float(cfg->gamma) || bad_float(cfg->eps) || bad_float(cfg->rho) || bad_float(cfg->tau_grad_scale))
    return FASTCLIP_ERR_VALUE;
  if (!(cfg->gamma > 0.0f && cfg->gamma <= 1.0f) || cfg->eps < 0.0f) return FASTCLIP_ERR_VALUE;
  const int64_t lim = (int64_t)1 << 24;
  if (cfg->B > lim || cfg->b > lim || cfg->d > lim || cfg->ld_img > ((int64_t)1 << 30) ||
      cfg->ld_txt > ((int64_t)1 << 30))
    return FASTCLIP_ERR_UNSUPPORTED;
  if (cfg->emb_dtype == FASTCLIP_BF16 && (cfg->d % 8 || cfg->ld_img % 8 || cfg->ld_txt % 8))
    return FASTCLIP_ERR_UNSUPPORTED;
  // the MFMA kernels address a tile panel (256 rows, or 8 anchor blocks of the stored strips) with 32-bit byte
  // offsets per lane
  const int64_t lim22 = (int64_t)1 << 22;
  if (cfg->emb_dtype == FASTCLIP_BF16 && (cfg->B + cfg->b > lim22 || cfg->ld_img > lim22 || cfg->ld_txt > lim22))
    return FASTCLIP_ERR_UNSUPPORTED;
  if (bufs) {
    if (!bufs->img_glob || !bufs->txt_glob || !bufs->idx || !bufs->u_img || !bufs->u_txt ||
        !bufs->d_img || !bufs->d_txt || !bufs->loss)
      return FASTCLIP_ERR_NULL;
    if (cfg->version == FASTCLIP_V2) {
      if (!bufs->tau_img || !bufs->tau_txt || !bufs->d_tau_img || !bufs->d_tau_txt) return FASTCLIP_ERR_NULL;
    } else {
      if (!bufs->tau) return FASTCLIP_ERR_NULL;
      if ((cfg->version == FASTCLIP_V0 || cfg->version == FASTCLIP_V3) && !bufs->d_tau) return FASTCLIP_ERR_NULL;
    }
    if ((bufs->norm_img == nullptr) != (bufs->norm_txt == nullptr)) return FASTCLIP_ERR_NULL;
    if ((cfg->flags & FASTCLIP_GATHERED_STATE) && cfg->b < cfg->B) {   // b == B: no remote anchors, arrays not read
      if (!bufs->u_glob_img || !bufs->u_glob_txt) return FASTCLIP_ERR_NULL;
      if (cfg->version == FASTCLIP_V2 && (!bufs->tau_glob_img || !bufs->tau_glob_txt)) return FASTCLIP_ERR_NULL;
    }
    if (cfg->emb_dtype == FASTCLIP_BF16 &&
        (((uintptr_t)bufs->img_glob & 15) || ((uintptr_t)bufs->txt_glob & 15)))
      return FASTCLIP_ERR_UNSUPPORTED;
    if (((uintptr_t)bufs->d_img & 15) || ((uintptr_t)bufs->d_txt & 15)) return FASTCLIP_ERR_UNSUPPORTED;
  }
  return FASTCLIP_OK;
}

fastclip_status validate_tau_update(int32_t version, const fastclip_tau_update* upd, const fastclip_tau_state* st) {
  if (!upd || !st) return FASTCLIP_ERR_NULL;
  if (upd->struct_size != sizeof(fastclip_tau_update) || upd->state_stride < 0 || upd->state_stride > 64)
    return FASTCLIP_ERR_SHAPE;
  if (version < FASTCLIP_V0 || version > FASTCLIP_V3) return FASTCLIP_ERR_VALUE;
  if (upd->optimizer < FASTCLIP_TAU_SGDM || upd->optimizer > FASTCLIP_TAU_ADAMW) return FASTCLIP_ERR_VALUE;
  const float f[7] = {upd->lr, upd->beta1, upd->beta2, upd->eps, upd->tau_min, upd->lr_drop_below, upd->lr_drop_factor};
  for (float x : f)
    if (bad_float(x)) return FASTCLIP_ERR_VALUE;
  if (upd->step < 1 || upd->lr < 0.0f || upd->eps < 0.0f || upd->beta1 < 0.0f || upd->beta1 >= 1.0f ||
      upd->beta2 < 0.0f || upd->beta2 >= 1.0f || upd->lr_drop_factor < 0.0f)
    return FASTCLIP_ERR_VALUE;
  const bool two = upd->optimizer == FASTCLIP_TAU_ADAMW || upd->optimizer == FASTCLIP_TAU_LAMB;
  if (version == FASTCLIP_V2) {
    if (!st->tau_img || !st->tau_txt || !st->m_img || !st->m_txt) return FASTCLIP_ERR_NULL;
    if (two && (!st->v_img || !st->v_txt)) return FASTCLIP_ERR_NULL;
  } else if (version != FASTCLIP_V1) {
    if (!st->tau || !st->m || (two && !st->v)) return FASTCLIP_ERR_NULL;
  }
  return FASTCLIP_OK;
}

TauUpd make_tau_upd(const fastclip_tau_update& upd) {
  TauUpd u;
  u.optimizer = upd.optimizer;
  u.lr = upd.lr; u.beta1 = upd.beta1; u.beta2 = upd.beta2; u.eps = upd.eps;
  // bias corrections 1 / (1 - beta^step) of Proc. "parameter_update", in double on the host
  u.corr1 = (float)(1.0 / (1.0 - pow((double)upd.beta1, (double)upd.step)));
  u.corr2 = (float)(1.0 / (1.0 - pow((double)upd.beta2, (double)upd.step)));
  u.tau_min = upd.tau_min; u.drop_below = upd.lr_drop_below; u.drop_factor = upd.lr_drop_factor;
  u.stride = upd.state_stride > 1 ? upd.state_stride : 1;
  return u;
}

void make_layout(const fastclip_config& cfg, Layout* L) {
  memset(L, 0, sizeof(*L));
  L->B = cfg.B; L->b = cfg.b; L->off = cfg.off; L->d = cfg.d; L->N = cfg.N;
  L->bf16 = cfg.emb_dtype == FASTCLIP_BF16;
  L->bstride = (int64_t)round_up((size_t)cfg.b, kTileContrasts);   // whole anchor tiles: the strip kernel works on 256 rows
  L->gathered = (cfg.flags & FASTCLIP_GATHERED_STATE) && cfg.b < cfg.B;
  L->ncol = (int64_t)round_up((size_t)cfg.B, kTileContrasts);
  // forming the similarity matrix once halves the MFMA work of the strip phase but doubles the epilogue of every
  // tile: it pays once the tiles outnumber the compute units (below that one tile's latency is the phase's time)
  const int64_t bt = (cfg.B + kTileContrasts - 1) / kTileContrasts;
  L->square = L->bf16 && cfg.b == cfg.B && (2 * bt * bt > 256 || (cfg.flags & FASTCLIP_SINGLE_PASS));
  // Fine tiles (opt-in) where 256 x 256 tiles would leave most of the chip idle: fewer large strip tiles than three
  // quarters of the compute units (one per compute unit is what the large-tile kernels are built for).
  const int64_t big_tiles = 2 * ((cfg.b + 255) / 256) * ((cfg.B + 255) / 256);
  L->fine = (cfg.flags & FASTCLIP_FINE_TILES) && L->bf16 && !L->gathered && !L->square && big_tiles < 192;
  // 128 x 128 tiles: asked for (wherever a quarter of the large tiles' workgroups would still not fill the chip), or
  // chosen when the large tiles would occupy at most half of the compute units (measured: b = 128 .. 1024 of
  // B = 1024 .. 8192 at width 512 are 4 - 22 % faster, b = 640 of 5120, 120 large tiles, breaks even)
  const bool small_ok = L->bf16 && !L->gathered && !L->square && !L->fine && !(cfg.flags & FASTCLIP_TILES_256);
  L->t128 = small_ok && ((cfg.flags & FASTCLIP_TILES_128) ? big_tiles < 192 : big_tiles <= 128);
  size_t at = 0;
  auto take = [&](size_t bytes) { size_t o = at; at += round_up(bytes, 256); return o; };
  const size_t fb = sizeof(float) * (size_t)L->bstride;
  if (L->t128) {
    L->nparts = (int)((cfg.B + 127) / 128);
    L->ldE = (int64_t)round_up((size_t)cfg.B, 64);
    // Split of the contraction over its column range, in 32-deep stages.  Cost model in units of one stage time of a
    // workgroup that has its compute unit to itself (0.65 us: a stage is the latency of its instructions, not its MFMA
    // time); measured on b = 128 .. 1024 of B = 1024 .. 8192 at width 512.  Up to 256 workgroups run one per compute
    // unit; a second one on a compute unit stretches both by 1.45; beyond 512 they run in rounds.  A tile's start and end
    // cost 4; with more than one split the finalize kernel costs 5 + 0.42 per MiB of partial results it reads.  One split
    // needs no finalize kernel (the tile is finished in place).
    const int64_t stages = L->ldE / 32;
    const int64_t tiles = ((cfg.b + 127) / 128) * ((cfg.d + 127) / 128) * 2;
    const double tile_mib = 128.0 * 128.0 * 4.0 / (1024.0 * 1024.0);
    int64_t best = 1;
    double best_cost = 0.0;
    for (int64_t ns = 1; ns <= kMaxSplit && ns <= stages; ++ns) {
      const int64_t slice = (stages + ns - 1) / ns;
      const int64_t used = (stages + slice - 1) / slice;
      if (used != ns) continue;                                     // every split must get at least one stage
      const int64_t wgs = tiles * ns;
      const double stretch = wgs <= 256 ? 1.0 : (wgs <= 512 ? 1.0 + 0.45 * (double)(wgs - 256) / 256.0
                                                            : 1.45 * (double)((wgs + 511) / 512));
      const double cost = stretch * (double)slice + 4.0 + (ns > 1 ? 5.0 + 0.42 * tile_mib * (double)wgs : 0.0);
      if (ns == 1 || cost < best_cost) { best = ns; best_cost = cost; }
    }
    L->nsplit = (int)best;
    L->kslice = (stages + best - 1) / best;
  } else if (L->fine) {
    L->nparts = (int)((cfg.B + 127) / 128);
    L->ldE = (int64_t)round_up((size_t)cfg.B, 64);
    // Split of the contraction over its column range, in 64-deep stages.  Cost model in units of one stage time: rounds
    // of 512 workgroups (two per compute unit) x (slice + 6 for the tile's start and end), and with more than one split
    // the finalize kernel: 27 for its launch + 0.02 per split and output tile.  One split needs no finalize kernel.
    const int64_t stages = L->ldE / 64;
    const int64_t tiles = ((cfg.b + 63) / 64) * ((cfg.d + 63) / 64) * 2;
    int64_t best = 1;
    double best_cost = 0.0;
    for (int64_t ns = 1; ns <= kMaxSplit && ns <= stages; ++ns) {
      const int64_t slice = (stages + ns - 1) / ns;
      const int64_t used = (stages + slice - 1) / slice;
      if (used != ns) continue;                                     // every split must get at least one stage
      const int64_t rounds = (tiles * ns + 511) / 512;
      const double cost = (double)rounds * (double)(slice + 6) + (ns > 1 ? 27.0 + 0.02 * (double)tiles * (double)ns : 0.0);
      if (ns == 1 || cost < best_cost) { best = ns; best_cost = cost; }
    }
    L->nsplit = (int)best;
    L->kslice = (stages + best - 1) / best;
  } else if (L->bf16) {
    L->nparts = (int)((cfg.B + kTileContrasts - 1) / kTileContrasts);
    L->ldE = (int64_t)round_up((size_t)cfg.B, 64);
    // Split of the contraction over its column range.  A workgroup owns one 256 x 256 output tile of one side and
    // `slice` stages; the 256 compute units take the workgroups in rounds.  Cost model in units of one stage time:
    // rounds x (slice + 12 for writing the partial tile) + 0.05 per split and output tile for the finalize pass that
    // adds the partial results up.
    const int64_t stages = L->ldE / 32;
    const int64_t tiles = ((cfg.b + 255) / 256) * ((cfg.d + 255) / 256) * 2;
    int64_t max_split = stages / 8;
    if (max_split > kMaxSplit) max_split = kMaxSplit;
    if (max_split < 1) max_split = 1;
    int64_t best = 1;
    double best_cost = 0.0;
    for (int64_t ns = 1; ns <= max_split; ++ns) {
      const int64_t slice = (stages + ns - 1) / ns;
      const int64_t used = (stages + slice - 1) / slice;          // splits that really get stages
      const int64_t rounds = (tiles * used + 255) / 256;
      const double cost = (double)rounds * (double)(slice + 12) + 0.05 * (double)tiles * (double)used;
      if (ns == 1 || cost < best_cost) { best = ns; best_cost = cost; }
    }
    L->kslice = (stages + best - 1) / best;
    L->nsplit = (int)((stages + L->kslice - 1) / L->kslice);
  } else {
    L->nparts = 1;
    L->ldE = cfg.B;
    L->nsplit = 0;
    L->kslice = 0;
  }
  // Every 64 x 64 block of the fold needs the coefficients of 128 anchor sides.  Forming them inside the fold saves a
  // launch, but every block then sums those anchors' partial sums again (b^2 / 32 anchor sides x nparts floats in
  // all, against 2 b x nparts once): worth it only while that stays small.
  L->fused_state = L->bf16 && L->nparts <= 64 &&
                   (double)cfg.b * (double)cfg.b / 32.0 * (double)L->nparts * 4.0 <= 2.0 * 1024 * 1024;
  L->nstate_blocks = L->fused_state ? (int)((cfg.b + 63) / 64) : state_blocks(cfg.b, L->nparts);
  L->diag = take(fb); L->tau1 = take(fb); L->tau2 = take(fb); L->k1 = take(fb); L->k2 = take(fb);
  L->uold1 = take(fb); L->uold2 = take(fb);
  L->sums = take(fb * 4 * (size_t)L->nparts);
  L->c1 = take(fb); L->c2 = take(fb); L->dcoef = take(fb);
  L->red = take(sizeof(double) * 2 * (size_t)L->nstate_blocks);
  const size_t esz = L->bf16 ? sizeof(bf16_t) : sizeof(float);
  if (L->bf16) {
    // fragment-ordered strips: anchors padded to whole 256-row tiles
    const size_t rows = round_up((size_t)cfg.b, 256);
    for (int s = 0; s < 2; ++s) L->E[s] = take(esz * rows * (size_t)L->ldE);
    if (L->t128) {     // [nsplit][2 sides][b to 128][d to 128] floats, only with more than one split
      if (L->nsplit > 1)
        L->Opart[0] = take(sizeof(float) * (size_t)L->nsplit * 2 * round_up((size_t)cfg.b, 128) * round_up((size_t)cfg.d, 128));
    } else if (L->fine) {     // [nsplit][2 sides][b to 64][d to 64] floats, only with more than one split
      if (L->nsplit > 1)
        L->Opart[0] = take(sizeof(float) * (size_t)L->nsplit * 2 * round_up((size_t)cfg.b, 64) * round_up((size_t)cfg.d, 64));
    } else {
      for (int s = 0; s < 2; ++s)
        L->Opart[s] = take(sizeof(float) * (size_t)L->nsplit * partial_split_floats(cfg.b, cfg.d));
    }
  } else {
    for (int s = 0; s < 2; ++s) L->E[s] = take(esz * (size_t)cfg.b * (size_t)L->ldE);
  }
  if (L->square) L->F[0] = take(esz * round_up((size_t)cfg.b, 256) * (size_t)L->ldE);
  if (L->gathered) {
    L->colp = take(sizeof(float) * 2 * 4 * (size_t)L->ncol);
    if (L->bf16) {
      const size_t rows = round_up((size_t)cfg.b, 256);
      for (int s = 0; s < 2; ++s) L->F[s] = take(esz * rows * (size_t)L->ldE);
    } else {
      for (int s = 0; s < 2; ++s) L->F[s] = take(esz * (size_t)cfg.b * (size_t)L->ldE);
    }
  }
  L->total = at;
}

static fastclip_status run_step(const fastclip_config* cfg, const fastclip_buffers* bufs, void* workspace,
                                size_t workspace_bytes, void* stream, float* phase_ms,
                                const fastclip_tau_update* upd = nullptr, const fastclip_tau_state* tst = nullptr) {
  fastclip_status st = validate(cfg, bufs);
  if (st != FASTCLIP_OK) return st;
  if (!bufs) return FASTCLIP_ERR_NULL;
  StepCtx c;
  c.cfg = *cfg;
  c.buf = *bufs;
  memset(&c.tau_upd, 0, sizeof(c.tau_upd));
  memset(&c.tau_st, 0, sizeof(c.tau_st));
  if (upd || tst) {
    st = validate_tau_update(cfg->version, upd, tst);
    if (st != FASTCLIP_OK) return st;
    // the step must read the very temperatures that the update writes
    if (cfg->version == FASTCLIP_V2 ? (tst->tau_img != bufs->tau_img || tst->tau_txt != bufs->tau_txt)
                                    : (cfg->version != FASTCLIP_V1 && tst->tau != bufs->tau))
      return FASTCLIP_ERR_VALUE;
    // ... laid out as the step's own state arrays are
    if (cfg->version == FASTCLIP_V2 && (upd->state_stride > 1 ? upd->state_stride : 1) != cfg->state_stride)
      return FASTCLIP_ERR_VALUE;
    if (cfg->version != FASTCLIP_V1) { c.tau_upd = make_tau_upd(*upd); c.tau_st = *tst; }
  }
  make_layout(*cfg, &c.L);
  if (!workspace) return FASTCLIP_ERR_NULL;
  if (workspace_bytes < c.L.total || ((uintptr_t)workspace & 255)) return FASTCLIP_ERR_WORKSPACE;
  c.ws = (char*)workspace;
  c.s = (hipStream_t)stream;
  (void)hipGetLastError();

  hipEvent_t ev[FASTCLIP_N_PHASES + 1];
  int nev = 0;
  int phase_of[FASTCLIP_N_PHASES];
  auto mark = [&](int phase) {
    if (!phase_ms) return;
    if (nev == 0) { (void)hipEventCreate(&ev[0]); (void)hipEventRecord(ev[0], c.s); nev = 1; }
    if (phase >= 0) { (void)hipEventCreate(&ev[nev]); (void)hipEventRecord(ev[nev], c.s); phase_of[nev - 1] = phase; ++nev; }
  };
  mark(-1);
  launch_prep(c);
  if (c.L.gathered) launch_prep_cols(c);
  mark(FASTCLIP_PHASE_PREP);
  if (c.L.t128) {
    launch_strips_t128_bf16(c);           mark(FASTCLIP_PHASE_STRIPS);
    if (!c.L.fused_state) { launch_state(c); mark(FASTCLIP_PHASE_STATE); }
    launch_fold_bf16(c);                  mark(FASTCLIP_PHASE_LOCAL);   // with fused_state: the state phase as well
    launch_contract_t128_bf16(c);         mark(FASTCLIP_PHASE_CONTRACT);  // outputs and scalars included
    launch_norm_backward_bf16(c);
  } else if (c.L.fine) {
    launch_strips_fine_bf16(c);           mark(FASTCLIP_PHASE_STRIPS);
    if (!c.L.fused_state) { launch_state(c); mark(FASTCLIP_PHASE_STATE); }
    launch_fold_bf16(c);                  mark(FASTCLIP_PHASE_LOCAL);   // with fused_state: the state phase as well
    launch_contract_fine_bf16(c);         mark(FASTCLIP_PHASE_CONTRACT);  // outputs and scalars included
    launch_norm_backward_bf16(c);
  } else if (c.L.bf16) {
    launch_strips_bf16(c);                mark(FASTCLIP_PHASE_STRIPS);
    if (!c.L.fused_state) { launch_state(c); mark(FASTCLIP_PHASE_STATE); }
    launch_fold_bf16(c);                  mark(FASTCLIP_PHASE_LOCAL);   // with fused_state: the state phase as well
    launch_contract_bf16(c);              mark(FASTCLIP_PHASE_CONTRACT);
    launch_finalize_bf16(c);
    launch_norm_backward_bf16(c);
  } else {
    launch_strips_f32(c);                 mark(FASTCLIP_PHASE_STRIPS);
    launch_state(c);                      mark(FASTCLIP_PHASE_STATE);
    launch_grad_f32(c);
  }
  // global temperature: stepped once its gradient is complete (V2 was stepped in the state phase)
  if (c.tau_upd.optimizer && c.cfg.version != FASTCLIP_V2) launch_tau_scalar(c.tau_upd, c.tau_st, c.buf.d_tau, c.s);
  mark(FASTCLIP_PHASE_FINALIZE);
  fastclip_status rc = launch_status();
  if (phase_ms) {
    for (int i = 0; i < FASTCLIP_N_PHASES; ++i) phase_ms[i] = 0.0f;
    const hipError_t es = hipStreamSynchronize(c.s);
    if (es != hipSuccess) rc = hip_failed(es);
    for (int i = 0; i + 1 < nev; ++i) {
      float ms = 0.0f;
      if (rc == FASTCLIP_OK && hipEventElapsedTime(&ms, ev[i], ev[i + 1]) == hipSuccess) phase_ms[phase_of[i]] += ms;
    }
    for (int i = 0; i < nev; ++i) (void)hipEventDestroy(ev[i]);
  }
  return rc;
}

// ---- fastclip_step_static: the step's workspace in device memory that the library's code object brings along -------
// One array per GPU (every device that loads the code object holds its own copy at its own address, until the process
// ends).  In host code the array's name is only a handle for hipGetSymbolAddress: the address that kernels and memory
// calls need is looked up once per device, with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[FASTCLIP_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device i, nullptr until first used there

static fastclip_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_failed(e);
  if (dev < 0 || dev >= kMaxDevices) return FASTCLIP_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_failed(e != hipSuccess ? e : hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return FASTCLIP_OK;
}

}  // namespace fc

extern "C" {

fastclip_status fastclip_step_static(const fastclip_config* cfg, const fastclip_buffers* bufs, void* stream) {
  const fastclip_status st = fc::validate(cfg, bufs);
  if (st != FASTCLIP_OK) return st;
  fc::Layout L;
  fc::make_layout(*cfg, &L);
  if (L.total > (size_t)FASTCLIP_STATIC_SCRATCH_BYTES) return FASTCLIP_ERR_WORKSPACE;
  void* ws = nullptr;
  const fastclip_status sp = fc::static_scratch(&ws);
  if (sp != FASTCLIP_OK) return sp;
  return fc::run_step(cfg, bufs, ws, (size_t)FASTCLIP_STATIC_SCRATCH_BYTES, stream, nullptr);
}

size_t fastclip_workspace_bytes(const fastclip_config* cfg) {
  if (fc::validate(cfg, nullptr) != FASTCLIP_OK) return 0;
  fc::Layout L;
  fc::make_layout(*cfg, &L);
  return L.total;
}

fastclip_status fastclip_describe(const fastclip_config* cfg, fastclip_plan* plan) {
  if (!plan) return FASTCLIP_ERR_NULL;
  const fastclip_status st = fc::validate(cfg, nullptr);
  if (st != FASTCLIP_OK) return st;
  fc::Layout L;
  fc::make_layout(*cfg, &L);
  plan->tile = !L.bf16 ? 0 : (L.t128 ? 128 : (L.fine ? 64 : 256));
  plan->single_pass = L.square;
  plan->gathered = L.gathered;
  plan->fused_state = L.fused_state;
  plan->nsplit = L.nsplit;
  plan->nparts = L.nparts;
  return FASTCLIP_OK;
}

fastclip_status fastclip_validate(const fastclip_config* cfg, const fastclip_buffers* bufs) {
  return fc::validate(cfg, bufs);
}

fastclip_status fastclip_step(const fastclip_config* cfg, const fastclip_buffers* bufs, void* workspace,
                              size_t workspace_bytes, void* stream) {
  return fc::run_step(cfg, bufs, workspace, workspace_bytes, stream, nullptr);
}

fastclip_status fastclip_step_timed(const fastclip_config* cfg, const fastclip_buffers* bufs, void* workspace,
                                    size_t workspace_bytes, void* stream, float* phase_ms) {
  if (!phase_ms) return FASTCLIP_ERR_NULL;
  return fc::run_step(cfg, bufs, workspace, workspace_bytes, stream, phase_ms);
}

fastclip_status fastclip_step_update_tau(const fastclip_config* cfg, const fastclip_buffers* bufs,
                                         const fastclip_tau_update* upd, const fastclip_tau_state* state,
                                         void* workspace, size_t workspace_bytes, void* stream) {
  if (!upd || !state) return FASTCLIP_ERR_NULL;
  return fc::run_step(cfg, bufs, workspace, workspace_bytes, stream, nullptr, upd, state);
}

// blocks of the state phase on its own: one per 128 anchors up to eight per compute unit of the largest part
static int state_phase_blocks(int64_t b) {
  const int tiles = fc::state_blocks(b, 1);
  return tiles < 2048 ? tiles : 2048;
}

size_t fastclip_state_phase_workspace_bytes(int64_t b) {
  if (b < 1 || b > ((int64_t)1 << 24)) return 0;
  return fc::round_up(sizeof(double) * 2 * (size_t)state_phase_blocks(b), 256);
}

fastclip_status fastclip_state_phase(const fastclip_config* cfg, const fastclip_buffers* bufs,
                                     const fastclip_tau_update* upd, const fastclip_tau_state* state,
                                     const float* sums, float* coef, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  // the phase sees the batch only through M = B - 1 and its b anchors: none of the matrix limits of the step apply
  if (!cfg) return FASTCLIP_ERR_NULL;
  if (cfg->struct_size != sizeof(fastclip_config) || cfg->B < 2 || cfg->b < 1 || cfg->N < 1 || cfg->b > cfg->N ||
      cfg->state_stride < 1 || cfg->state_stride > 64)
    return FASTCLIP_ERR_SHAPE;
  if (cfg->version < FASTCLIP_V0 || cfg->version > FASTCLIP_V3 ||
      (cfg->emb_dtype != FASTCLIP_F32 && cfg->emb_dtype != FASTCLIP_BF16))
    return FASTCLIP_ERR_VALUE;
  if (fc::bad_float(cfg->gamma) || fc::bad_float(cfg->eps) || fc::bad_float(cfg->rho) ||
      fc::bad_float(cfg->tau_grad_scale) || !(cfg->gamma > 0.0f && cfg->gamma <= 1.0f) || cfg->eps < 0.0f)
    return FASTCLIP_ERR_VALUE;
  if (cfg->b > ((int64_t)1 << 24) || cfg->B > ((int64_t)1 << 24)) return FASTCLIP_ERR_UNSUPPORTED;
  fastclip_status st = FASTCLIP_OK;
  if (!bufs || !sums || !coef || !workspace) return FASTCLIP_ERR_NULL;
  if (!bufs->idx || !bufs->u_img || !bufs->u_txt || !bufs->loss) return FASTCLIP_ERR_NULL;
  if (cfg->version == FASTCLIP_V2) {
    if (!bufs->tau_img || !bufs->tau_txt || !bufs->d_tau_img || !bufs->d_tau_txt) return FASTCLIP_ERR_NULL;
  } else {
    if (!bufs->tau) return FASTCLIP_ERR_NULL;
    if (cfg->version != FASTCLIP_V1 && !bufs->d_tau) return FASTCLIP_ERR_NULL;
  }
  if ((upd == nullptr) != (state == nullptr)) return FASTCLIP_ERR_NULL;
  fc::TauUpd tu;
  memset(&tu, 0, sizeof(tu));
  fastclip_tau_state ts;
  memset(&ts, 0, sizeof(ts));
  if (upd) {
    st = fc::validate_tau_update(cfg->version, upd, state);
    if (st != FASTCLIP_OK) return st;
    if (cfg->version == FASTCLIP_V2 ? (state->tau_img != bufs->tau_img || state->tau_txt != bufs->tau_txt)
                                    : (cfg->version != FASTCLIP_V1 && state->tau != bufs->tau))
      return FASTCLIP_ERR_VALUE;
    if (cfg->version == FASTCLIP_V2 && (upd->state_stride > 1 ? upd->state_stride : 1) != cfg->state_stride)
      return FASTCLIP_ERR_VALUE;
    if (cfg->version != FASTCLIP_V1) { tu = fc::make_tau_upd(*upd); ts = *state; }
  }
  if (workspace_bytes < fastclip_state_phase_workspace_bytes(cfg->b) || ((uintptr_t)workspace & 255))
    return FASTCLIP_ERR_WORKSPACE;
  (void)hipGetLastError();
  fc::launch_state_phase(*cfg, *bufs, tu, ts, sums, coef, (double*)workspace, state_phase_blocks(cfg->b),
                         (hipStream_t)stream);
  if (tu.optimizer && cfg->version != FASTCLIP_V2) fc::launch_tau_scalar(tu, ts, bufs->d_tau, (hipStream_t)stream);
  return fc::launch_status();
}

fastclip_status fastclip_temperature_update(int32_t version, const fastclip_tau_update* upd,
                                            const fastclip_tau_state* state, const int64_t* idx, int64_t b,
                                            int64_t N, const float* d_tau, const float* d_tau_img,
                                            const float* d_tau_txt, void* stream) {
  const fastclip_status st = fc::validate_tau_update(version, upd, state);
  if (st != FASTCLIP_OK) return st;
  if (version == FASTCLIP_V1) return FASTCLIP_OK;
  (void)hipGetLastError();
  const fc::TauUpd u = fc::make_tau_upd(*upd);
  if (version == FASTCLIP_V2) {
    if (!idx || !d_tau_img || !d_tau_txt) return FASTCLIP_ERR_NULL;
    if (b < 0 || N < 1 || b > N || b > ((int64_t)1 << 31) - 1024) return FASTCLIP_ERR_SHAPE;
    if (b == 0) return FASTCLIP_OK;
    fc::launch_tau_sparse(u, *state, idx, b, d_tau_img, d_tau_txt, (hipStream_t)stream);
  } else {
    if (!d_tau) return FASTCLIP_ERR_NULL;
    fc::launch_tau_scalar(u, *state, d_tau, (hipStream_t)stream);
  }
  return fc::launch_status();
}

fastclip_status fastclip_measure_mfma_ceiling(int32_t workgroups, int32_t iters, void* workspace,
                                              size_t workspace_bytes, void* stream, float* ms, double* stats) {
  if (!workspace || !ms || !stats) return FASTCLIP_ERR_NULL;
  if (workgroups < 1 || workgroups > 4096 || iters < 1 || iters > (1 << 24)) return FASTCLIP_ERR_SHAPE;
  const size_t need = (size_t)workgroups * 8 * 2 * sizeof(uint64_t) + 512 * sizeof(float);
  if (workspace_bytes < need || ((uintptr_t)workspace & 255)) return FASTCLIP_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  uint64_t* out = (uint64_t*)workspace;
  float* sink = (float*)((char*)workspace + (size_t)workgroups * 8 * 2 * sizeof(uint64_t));
  (void)hipGetLastError();
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return fc::hip_failed(e);
  e = hipEventCreate(&e1);
  if (e != hipSuccess) { (void)hipEventDestroy(e0); return fc::hip_failed(e); }
  fc::launch_mfma_ceiling(workgroups, iters, out, sink, s);     // untimed: first launch of the kernel
  (void)hipEventRecord(e0, s);
  fc::launch_mfma_ceiling(workgroups, iters, out, sink, s);
  (void)hipEventRecord(e1, s);
  fastclip_status rc = fc::launch_status();
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) rc = fc::hip_failed(e);
  *ms = 0.f;
  if (rc == FASTCLIP_OK && hipEventElapsedTime(ms, e0, e1) != hipSuccess) rc = FASTCLIP_ERR_LAUNCH;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != FASTCLIP_OK) return rc;
  // per-wave counters of the timed launch: mean shader cycles and mean 100 MHz ticks of a wave's loop
  const size_t nw = (size_t)workgroups * 8;
  uint64_t* host = (uint64_t*)malloc(nw * 2 * sizeof(uint64_t));
  if (!host) return FASTCLIP_ERR_LAUNCH;
  e = hipMemcpy(host, out, nw * 2 * sizeof(uint64_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) { free(host); return fc::hip_failed(e); }
  double cyc = 0.0, ticks = 0.0;
  for (size_t i = 0; i < nw; ++i) { cyc += (double)host[2 * i]; ticks += (double)host[2 * i + 1]; }
  free(host);
  cyc /= (double)nw; ticks /= (double)nw;
  stats[0] = (double)workgroups * 8.0 * (double)iters * 8.0 * 32768.0;   // flop of the timed launch
  stats[1] = cyc;                                                       // shader cycles per wave
  stats[2] = ticks > 0.0 ? cyc / (ticks * 10.0) : 0.0;                  // GHz while the loop ran (ticks of 10 ns)
  stats[3] = cyc / ((double)iters * 8.0);                               // cycles per MFMA as one wave sees them
  return FASTCLIP_OK;
}

fastclip_status fastclip_measure_strips(const fastclip_config* cfg, const fastclip_buffers* bufs, void* workspace,
                                        size_t workspace_bytes, void* stream, int32_t ablation, int32_t reps, float* ms,
                                        double* stats) {
  if (!ms || !stats) return FASTCLIP_ERR_NULL;
  fastclip_status st = fc::validate(cfg, bufs);
  if (st != FASTCLIP_OK) return st;
  if (!bufs || !workspace) return FASTCLIP_ERR_NULL;
  if (reps < 1 || reps > 1000) return FASTCLIP_ERR_SHAPE;
  fc::StepCtx c;
  c.cfg = *cfg;
  c.buf = *bufs;
  memset(&c.tau_upd, 0, sizeof(c.tau_upd));
  memset(&c.tau_st, 0, sizeof(c.tau_st));
  fc::make_layout(*cfg, &c.L);
  const size_t ncyc = (size_t)256 * 2 * 4;
  if (workspace_bytes < c.L.total + ncyc * sizeof(uint64_t) || ((uintptr_t)workspace & 255)) return FASTCLIP_ERR_WORKSPACE;
  if (!c.L.bf16 || c.L.fine || c.L.t128 || c.L.square || c.L.gathered) return FASTCLIP_ERR_UNSUPPORTED;
  c.ws = (char*)workspace;
  c.s = (hipStream_t)stream;
  uint64_t* cycles = (uint64_t*)(c.ws + c.L.total);
  (void)hipGetLastError();
  hipError_t e = hipMemsetAsync(cycles, 0, ncyc * sizeof(uint64_t), c.s);
  if (e != hipSuccess) return fc::hip_failed(e);
  fc::launch_prep(c);                                   // s_ii and the temperatures that the epilogue reads
  if (!fc::launch_strips_measure(c, ablation, cycles)) return FASTCLIP_ERR_UNSUPPORTED;   // untimed first launch
  hipEvent_t e0, e1;
  e = hipEventCreate(&e0);
  if (e != hipSuccess) return fc::hip_failed(e);
  e = hipEventCreate(&e1);
  if (e != hipSuccess) { (void)hipEventDestroy(e0); return fc::hip_failed(e); }
  (void)hipEventRecord(e0, c.s);
  for (int i = 0; i < reps; ++i) (void)fc::launch_strips_measure(c, ablation, cycles);
  (void)hipEventRecord(e1, c.s);
  fastclip_status rc = fc::launch_status();
  e = hipStreamSynchronize(c.s);
  if (e != hipSuccess) rc = fc::hip_failed(e);
  *ms = 0.f;
  if (rc == FASTCLIP_OK && hipEventElapsedTime(ms, e0, e1) != hipSuccess) rc = FASTCLIP_ERR_LAUNCH;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != FASTCLIP_OK) return rc;
  *ms /= (float)reps;
  uint64_t* host = (uint64_t*)malloc(ncyc * sizeof(uint64_t));
  if (!host) return FASTCLIP_ERR_LAUNCH;
  e = hipMemcpy(host, cycles, ncyc * sizeof(uint64_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) { free(host); return fc::hip_failed(e); }
  // counters of the last launch: [workgroup][older | younger wave of SIMD 0][total cycles, epilogue cycles, 10 ns ticks, -]
  double tot[2] = {0.0, 0.0}, epi[2] = {0.0, 0.0}, ticks = 0.0;
  int used = 0;
  for (int w = 0; w < 256; ++w) {
    if (!host[(w * 2) * 4]) continue;
    ++used;
    for (int y = 0; y < 2; ++y) { tot[y] += (double)host[(w * 2 + y) * 4]; epi[y] += (double)host[(w * 2 + y) * 4 + 1]; }
    ticks += (double)host[(w * 2) * 4 + 2];
  }
  free(host);
  if (!used) return FASTCLIP_ERR_LAUNCH;
  const double tiles_per_wg = 2.0 * (double)((cfg->b + 255) / 256) * (double)((cfg->B + 255) / 256) / (double)used;
  stats[0] = tot[0] / used;                                 // cycles of the older wave of a SIMD, kernel entry to exit
  stats[1] = tot[1] / used;                                 // ... of the younger wave
  stats[2] = epi[0] / used;                                 // of which between the last stage of a tile and the next tile
  stats[3] = tiles_per_wg * (double)(cfg->d / 64);          // 64-deep stages per workgroup
  stats[4] = ticks > 0.0 ? tot[0] / (ticks * 10.0) : 0.0;   // shader clock in GHz while the kernel ran
  stats[5] = (double)used;                                  // workgroups
  return FASTCLIP_OK;
}

fastclip_status fastclip_normalize_rows(const void* raw, int32_t raw_dtype, int64_t ld_raw, int64_t b, int64_t d,
                                        void* unit, int32_t unit_dtype, int64_t ld_unit, float* norm, void* stream) {
  if (!raw || !unit || !norm) return FASTCLIP_ERR_NULL;
  if (b < 0 || d < 1 || ld_raw < d || ld_unit < d) return FASTCLIP_ERR_SHAPE;
  if ((raw_dtype != FASTCLIP_F32 && raw_dtype != FASTCLIP_BF16) || (unit_dtype != FASTCLIP_F32 && unit_dtype != FASTCLIP_BF16))
    return FASTCLIP_ERR_VALUE;
  if (b > ((int64_t)1 << 31) - 1024 || d > ((int64_t)1 << 24) || ld_raw > ((int64_t)1 << 30) || ld_unit > ((int64_t)1 << 30))
    return FASTCLIP_ERR_UNSUPPORTED;
  if (raw == unit && (raw_dtype != unit_dtype || ld_raw != ld_unit)) return FASTCLIP_ERR_VALUE;
  if (b == 0) return FASTCLIP_OK;
  (void)hipGetLastError();
  fc::launch_normalize_rows(raw, raw_dtype == FASTCLIP_BF16, ld_raw, b, d, unit, unit_dtype == FASTCLIP_BF16, ld_unit, norm,
                            (hipStream_t)stream);
  return fc::launch_status();
}

fastclip_status fastclip_measure_record_rmw(const int64_t* idx, int64_t n, int64_t N, float* records,
                                            int64_t record_floats, void* stream) {
  if (!idx || !records) return FASTCLIP_ERR_NULL;
  if (n < 0 || N < 1 || n > N || n > ((int64_t)1 << 30) || record_floats < 8 || record_floats % 8 ||
      record_floats > 64)
    return FASTCLIP_ERR_SHAPE;
  if ((uintptr_t)records & 31) return FASTCLIP_ERR_UNSUPPORTED;
  if (n == 0) return FASTCLIP_OK;
  (void)hipGetLastError();
  fc::launch_record_rmw(idx, n, records, record_floats, (hipStream_t)stream);
  return fc::launch_status();
}

const char* fastclip_phase_name(int phase) {
  switch (phase) {
    case FASTCLIP_PHASE_PREP: return "prep";
    case FASTCLIP_PHASE_STRIPS: return "strips";
    case FASTCLIP_PHASE_STATE: return "state";
    case FASTCLIP_PHASE_LOCAL: return "local";
    case FASTCLIP_PHASE_CONTRACT: return "contract";
    case FASTCLIP_PHASE_FINALIZE: return "finalize";
    default: return "unused";
  }
}

fastclip_status fastclip_state_update(const int64_t* idx, int64_t n, int64_t N, float gamma, float M,
                                      const float* sum_img, const float* sum_txt, float* u_img, float* u_txt,
                                      float* u_new_img, float* u_new_txt, void* stream) {
  return fastclip_state_update_strided(idx, n, N, 1, gamma, M, sum_img, sum_txt, u_img, u_txt, u_new_img, u_new_txt,
                                       stream);
}

fastclip_status fastclip_state_update_strided(const int64_t* idx, int64_t n, int64_t N, int64_t state_stride,
                                              float gamma, float M, const float* sum_img, const float* sum_txt,
                                              float* u_img, float* u_txt, float* u_new_img, float* u_new_txt,
                                              void* stream) {
  if (!idx || !sum_img || !sum_txt || !u_img || !u_txt || !u_new_img || !u_new_txt) return FASTCLIP_ERR_NULL;
  // the indices are distinct values in [0, N), so there cannot be more than N of them
  if (n < 0 || N < 1 || n > N || n > ((int64_t)1 << 31) - 1024 || state_stride < 1 || state_stride > 64)
    return FASTCLIP_ERR_SHAPE;
  if (fc::bad_float(gamma) || fc::bad_float(M) || !(gamma > 0.0f && gamma <= 1.0f) || !(M > 0.0f))
    return FASTCLIP_ERR_VALUE;
  if (n == 0) return FASTCLIP_OK;
  (void)hipGetLastError();
  fc::launch_state_flat(idx, n, state_stride, gamma, M, sum_img, sum_txt, u_img, u_txt, u_new_img, u_new_txt,
                        (hipStream_t)stream);
  return fc::launch_status();
}

static size_t table_slots(int64_t b) {
  size_t s = 64;
  while (s < (size_t)b * 2) s <<= 1;
  return s;
}

size_t fastclip_check_indices_workspace_bytes(int64_t b) {
  if (b < 0 || b > ((int64_t)1 << 28)) return 0;
  return 256 + table_slots(b) * sizeof(int64_t);
}

fastclip_status fastclip_check_indices(const int64_t* idx, int64_t b, int64_t N, void* workspace,
                                       size_t workspace_bytes, void* stream) {
  if (!idx || !workspace) return FASTCLIP_ERR_NULL;
  if (b < 0 || N < 1 || b > ((int64_t)1 << 28)) return FASTCLIP_ERR_SHAPE;
  if (workspace_bytes < fastclip_check_indices_workspace_bytes(b) || ((uintptr_t)workspace & 255))
    return FASTCLIP_ERR_WORKSPACE;
  if (b == 0) return FASTCLIP_OK;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();
  fc::launch_check_indices(idx, b, N, workspace, s);
  int flag = 0;
  if (fc::launch_status() != FASTCLIP_OK) return FASTCLIP_ERR_LAUNCH;
  hipError_t e = hipMemcpyAsync(&flag, workspace, sizeof(int), hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return fc::hip_failed(e);
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fc::hip_failed(e);
  return flag ? FASTCLIP_ERR_INDEX : FASTCLIP_OK;
}

float fastclip_gamma_cosine(int64_t t, int64_t iters_per_epoch, int64_t decay_epochs, float gamma_min) {
  if (iters_per_epoch < 1) iters_per_epoch = 1;
  if (t < 0) t = 0;
  const int64_t epoch = t / iters_per_epoch;
  if (decay_epochs < 1 || epoch >= decay_epochs) return gamma_min;
  const double c = cos(M_PI * (double)epoch / (double)decay_epochs);
  return (float)(0.5 * (1.0 + c) * (1.0 - (double)gamma_min) + (double)gamma_min);
}

const char* fastclip_last_hip_error(void) { return hipGetErrorString(fc::g_last_hip_error); }

const char* fastclip_status_string(fastclip_status s) {
  switch (s) {
    case FASTCLIP_OK: return "ok";
    case FASTCLIP_ERR_NULL: return "a required pointer is NULL";
    case FASTCLIP_ERR_SHAPE: return "invalid shape or struct_size";
    case FASTCLIP_ERR_VALUE: return "invalid scalar, version or dtype";
    case FASTCLIP_ERR_WORKSPACE: return "workspace too small or misaligned";
    case FASTCLIP_ERR_UNSUPPORTED: return "unsupported size or alignment";
    case FASTCLIP_ERR_LAUNCH: return "HIP runtime error";
    case FASTCLIP_ERR_INDEX: return "index out of range or repeated";
    default: return "unknown status";
  }
}

}  // extern "C"
