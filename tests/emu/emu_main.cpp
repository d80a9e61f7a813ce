// Runs fastclip_step of the CPU build of libfastclip's sources on one case file and writes the outputs.  Every buffer is
// its own exact-size allocation, so that AddressSanitizer sees any access outside it; the matrices end with the last
// row's d elements.  Test infrastructure (see hip/hip_runtime.h).
#include <hip/hip_runtime.h>
#include "fastclip.h"

thread_local dim3 threadIdx, blockIdx;
dim3 blockDim, gridDim;
namespace emu {
thread_local Block* t_block;
thread_local Wave* t_wave;
thread_local int t_lane;
uintptr_t g_lds_hi;
static int g_marker;

// a pool of OS threads that plays the threads of one workgroup at a time
struct Pool {
  std::vector<std::thread> th;
  std::mutex m;
  std::condition_variable start, done;
  unsigned gen = 0;
  int nactive = 0, remaining = 0;
  bool quit = false;
  std::function<void(int)> work;
  void worker(int i) {
    unsigned seen = 0;
    for (;;) {
      {
        std::unique_lock<std::mutex> l(m);
        start.wait(l, [&] { return quit || (gen != seen && i < nactive); });
        if (quit) return;
        seen = gen;
      }
      work(i);
      std::unique_lock<std::mutex> l(m);
      if (--remaining == 0) done.notify_all();
    }
  }
  void run(int n, const std::function<void(int)>& w) {
    while ((int)th.size() < n) { const int i = (int)th.size(); th.emplace_back([this, i] { worker(i); }); }
    std::unique_lock<std::mutex> l(m);
    work = w; nactive = n; remaining = n; ++gen;
    start.notify_all();
    done.wait(l, [&] { return remaining == 0; });
    nactive = 0;
  }
  ~Pool() {
    { std::unique_lock<std::mutex> l(m); quit = true; start.notify_all(); }
    for (auto& t : th) t.join();
  }
};
static Pool g_pool;

void launch(dim3 grid, dim3 block, const std::function<void()>& body) {
  gridDim = grid; blockDim = block;
  const int nthreads = (int)(block.x * block.y * block.z), nwaves = (nthreads + 63) / 64;
  for (unsigned bz = 0; bz < grid.z; ++bz)
    for (unsigned by = 0; by < grid.y; ++by)
      for (unsigned bx = 0; bx < grid.x; ++bx) {
        Block blk;
        blk.waves = std::vector<Wave>(nwaves);
        blk.bar.reset(nthreads);
        for (int w = 0; w < nwaves; ++w) blk.waves[w].bar.reset(nthreads - 64 * w < 64 ? nthreads - 64 * w : 64);
        g_pool.run(nthreads, [&](int t) {
          threadIdx = dim3(t % block.x, (t / block.x) % block.y, t / (block.x * block.y));
          blockIdx = dim3(bx, by, bz);
          t_block = &blk; t_wave = &blk.waves[t / 64]; t_lane = t % 64;
          body();
          t_wave->bar.leave();      // a finished thread takes no part in later barriers
          t_block->bar.leave();
        });
      }
}
}  // namespace emu

template <typename T> static T* rd(FILE* f, size_t n) {
  T* p = (T*)malloc(n * sizeof(T) ? n * sizeof(T) : 1);
  if (fread(p, sizeof(T), n, f) != n) { fprintf(stderr, "short read\n"); exit(2); }
  return p;
}
// outputs and workspace start as NaN bit patterns; with EMU_UNINIT set they stay uninitialised (for MemorySanitizer)
template <typename T> static T* nan_buf(size_t n) {
  T* p = (T*)malloc(n * sizeof(T) ? n * sizeof(T) : 1);
  if (!getenv("EMU_UNINIT")) memset(p, 0xff, n * sizeof(T));
  return p;
}

// case file: 12 int64 {version, emb_dtype, flags, B, b, off, d, ld_img, ld_txt, N, state_stride, has_glob},
// 5 float {gamma, eps, rho, tau, tau_grad_scale}, img, txt (each (B - 1) ld + d elements), idx [b], u_img, u_txt [N],
// V2: tau_img, tau_txt [N], has_glob: u_glob_img, u_glob_txt [B] and for V2 tau_glob_img, tau_glob_txt [B].
// With a third argument "tau" the file goes on with 2 int64 {optimizer, step}, 7 float {lr, beta1, beta2, eps, tau_min,
// lr_drop_below, lr_drop_factor}, then V2: m_img, v_img, m_txt, v_txt [N], else m, v [1], and fastclip_step_update_tau
// runs instead of fastclip_step; with state_stride 8 the eight per-sample arrays of V2 are packed into records
// {u_1, tau_1, m_1, v_1, u_2, tau_2, m_2, v_2} first (the layout the library moves as 16-byte words).
// The small entry points on one file: "misc" <in> <out>.  In: 6 int64 {b, d, ld_raw, ld_unit, N, n}, 2 float {gamma, M},
// raw fp32 rows ((b - 1) ld_raw + d), idx [n], sum_img, sum_txt [n], u_img, u_txt [N].  Runs fastclip_normalize_rows
// (fp32 -> bf16), fastclip_check_indices on idx and on idx with its last entry repeated, fastclip_state_update.
// Out: norm [b], unit rows as raw bf16 bits ((b - 1) ld_unit + d, 2 bytes each), 2 int32 statuses, u_img, u_txt [N],
// u_new_img, u_new_txt [n].
static int run_misc(const char* fin, const char* fout) {
  FILE* f = fopen(fin, "rb");
  if (!f) return 2;
  int64_t h[6];
  float p[2];
  if (fread(h, 8, 6, f) != 6 || fread(p, 4, 2, f) != 2) return 2;
  const int64_t b = h[0], d = h[1], ld_raw = h[2], ld_unit = h[3], N = h[4], n = h[5];
  float* raw = rd<float>(f, (size_t)(b - 1) * ld_raw + d);
  int64_t* idx = rd<int64_t>(f, n);
  float *sum_img = rd<float>(f, n), *sum_txt = rd<float>(f, n), *u_img = rd<float>(f, N), *u_txt = rd<float>(f, N);
  fclose(f);
  const size_t n_unit = (size_t)(b - 1) * ld_unit + d;
  uint16_t* unit = nan_buf<uint16_t>(n_unit);
  float* norm = nan_buf<float>(b);
  if (fastclip_normalize_rows(raw, FASTCLIP_F32, ld_raw, b, d, unit, FASTCLIP_BF16, ld_unit, norm, nullptr) != FASTCLIP_OK)
    return 4;
  const size_t wsb = fastclip_check_indices_workspace_bytes(n);
  void* ws = nullptr;
  if (posix_memalign(&ws, 256, wsb)) return 2;
  int32_t st[2];
  st[0] = (int32_t)fastclip_check_indices(idx, n, N, ws, wsb, nullptr);
  int64_t* dup = (int64_t*)malloc(sizeof(int64_t) * n);
  memcpy(dup, idx, sizeof(int64_t) * n);
  if (n > 1) dup[n - 1] = dup[0];
  st[1] = (int32_t)fastclip_check_indices(dup, n, N, ws, wsb, nullptr);
  float *u_new_img = nan_buf<float>(n), *u_new_txt = nan_buf<float>(n);
  if (fastclip_state_update(idx, n, N, p[0], p[1], sum_img, sum_txt, u_img, u_txt, u_new_img, u_new_txt, nullptr) != FASTCLIP_OK)
    return 4;
  FILE* o = fopen(fout, "wb");
  if (!o) return 2;
  fwrite(norm, 4, b, o); fwrite(unit, 2, n_unit, o); fwrite(st, 4, 2, o);
  fwrite(u_img, 4, N, o); fwrite(u_txt, 4, N, o); fwrite(u_new_img, 4, n, o); fwrite(u_new_txt, 4, n, o);
  fclose(o);
  return 0;
}

int main(int argc, char** argv) {
  emu::g_lds_hi = (uintptr_t)&emu::g_marker & ~(uintptr_t)0xffffffffull;
  if (argc == 4 && !strcmp(argv[1], "misc")) return run_misc(argv[2], argv[3]);
  if (argc < 3) return 2;
  FILE* f = fopen(argv[1], "rb");
  if (!f) return 2;
  int64_t h[12];
  float p[5];
  if (fread(h, 8, 12, f) != 12 || fread(p, 4, 5, f) != 5) return 2;
  fastclip_config cfg;
  memset(&cfg, 0, sizeof(cfg));
  cfg.struct_size = sizeof(cfg);
  cfg.version = (int32_t)h[0]; cfg.emb_dtype = (int32_t)h[1]; cfg.flags = (int32_t)h[2];
  cfg.B = h[3]; cfg.b = h[4]; cfg.off = h[5]; cfg.d = h[6]; cfg.ld_img = h[7]; cfg.ld_txt = h[8]; cfg.N = h[9];
  cfg.state_stride = h[10];
  cfg.gamma = p[0]; cfg.eps = p[1]; cfg.rho = p[2]; cfg.tau_grad_scale = p[4];
  const size_t esz = cfg.emb_dtype == FASTCLIP_BF16 ? 2 : 4;
  const size_t n_img = (size_t)(cfg.B - 1) * cfg.ld_img + cfg.d, n_txt = (size_t)(cfg.B - 1) * cfg.ld_txt + cfg.d;
  fastclip_buffers b;
  memset(&b, 0, sizeof(b));
  b.img_glob = rd<char>(f, n_img * esz);
  b.txt_glob = rd<char>(f, n_txt * esz);
  b.idx = rd<int64_t>(f, cfg.b);
  b.u_img = rd<float>(f, cfg.N); b.u_txt = rd<float>(f, cfg.N);
  float* tau = (float*)malloc(4); *tau = p[3]; b.tau = tau;
  if (cfg.version == FASTCLIP_V2) { b.tau_img = rd<float>(f, cfg.N); b.tau_txt = rd<float>(f, cfg.N); }
  if (h[11]) {
    b.u_glob_img = rd<float>(f, cfg.B); b.u_glob_txt = rd<float>(f, cfg.B);
    if (cfg.version == FASTCLIP_V2) { b.tau_glob_img = rd<float>(f, cfg.B); b.tau_glob_txt = rd<float>(f, cfg.B); }
  }
  const bool with_tau = argc > 3 && !strcmp(argv[3], "tau");
  const bool v2_ = cfg.version == FASTCLIP_V2;
  fastclip_tau_update upd;
  fastclip_tau_state tst;
  memset(&upd, 0, sizeof(upd));
  memset(&tst, 0, sizeof(tst));
  float* rec = nullptr;
  const int64_t S = cfg.state_stride;
  if (with_tau) {
    int64_t ih[2];
    float fp[7];
    if (fread(ih, 8, 2, f) != 2 || fread(fp, 4, 7, f) != 7) return 2;
    upd.struct_size = sizeof(upd); upd.optimizer = (int32_t)ih[0]; upd.step = ih[1];
    upd.lr = fp[0]; upd.beta1 = fp[1]; upd.beta2 = fp[2]; upd.eps = fp[3]; upd.tau_min = fp[4];
    upd.lr_drop_below = fp[5]; upd.lr_drop_factor = fp[6]; upd.state_stride = (int32_t)S;
    if (v2_) {
      tst.m_img = rd<float>(f, cfg.N); tst.v_img = rd<float>(f, cfg.N);
      tst.m_txt = rd<float>(f, cfg.N); tst.v_txt = rd<float>(f, cfg.N);
      tst.tau_img = (float*)b.tau_img; tst.tau_txt = (float*)b.tau_txt;
    } else {
      tst.tau = tau; tst.m = rd<float>(f, 1); tst.v = rd<float>(f, 1);
    }
  }
  if (S > 1) {          // pack the per-sample arrays into records (canonical field order), exact-size allocation
    if (S < 8 || !v2_ || !with_tau) { fprintf(stderr, "records: V2 with the temperature update and stride >= 8 only\n"); return 3; }
    rec = (float*)malloc(sizeof(float) * cfg.N * S);
    float* src[8] = {b.u_img, tst.tau_img, tst.m_img, tst.v_img, b.u_txt, tst.tau_txt, tst.m_txt, tst.v_txt};
    for (int64_t n = 0; n < cfg.N; ++n)
      for (int64_t k = 0; k < S; ++k) rec[n * S + k] = k < 8 ? src[k][n] : 7.5f;
    for (int k = 0; k < 8; ++k) free(src[k]);
    b.u_img = rec + 0; tst.tau_img = rec + 1; tst.m_img = rec + 2; tst.v_img = rec + 3;
    b.u_txt = rec + 4; tst.tau_txt = rec + 5; tst.m_txt = rec + 6; tst.v_txt = rec + 7;
    b.tau_img = tst.tau_img; b.tau_txt = tst.tau_txt;
  }
  fclose(f);
  b.d_img = nan_buf<float>(cfg.b * cfg.d); b.d_txt = nan_buf<float>(cfg.b * cfg.d);
  b.loss = nan_buf<float>(1); b.d_tau = nan_buf<float>(1);
  b.d_tau_img = nan_buf<float>(cfg.b); b.d_tau_txt = nan_buf<float>(cfg.b);
  b.g_img = nan_buf<float>(cfg.b); b.g_txt = nan_buf<float>(cfg.b);
  b.u_new_img = nan_buf<float>(cfg.b); b.u_new_txt = nan_buf<float>(cfg.b);
  const size_t need = fastclip_workspace_bytes(&cfg);
  if (!need) { fprintf(stderr, "invalid config\n"); return 3; }
  void* ws = nullptr;
  if (posix_memalign(&ws, 256, need)) return 2;
  if (!getenv("EMU_UNINIT")) memset(ws, 0xff, need);
  const fastclip_status st = with_tau ? fastclip_step_update_tau(&cfg, &b, &upd, &tst, ws, need, nullptr)
                                      : fastclip_step(&cfg, &b, ws, need, nullptr);
  if (st != FASTCLIP_OK) { fprintf(stderr, "fastclip_step: %d\n", (int)st); return 4; }
  FILE* o = fopen(argv[2], "wb");
  if (!o) return 2;
  const bool v2 = cfg.version == FASTCLIP_V2, has_tau = cfg.version == FASTCLIP_V0 || cfg.version == FASTCLIP_V3;
  fwrite(b.d_img, 4, cfg.b * cfg.d, o); fwrite(b.d_txt, 4, cfg.b * cfg.d, o);
  fwrite(b.loss, 4, 1, o);
  if (has_tau) fwrite(b.d_tau, 4, 1, o);
  if (v2) { fwrite(b.d_tau_img, 4, cfg.b, o); fwrite(b.d_tau_txt, 4, cfg.b, o); }
  fwrite(b.g_img, 4, cfg.b, o); fwrite(b.g_txt, 4, cfg.b, o);
  fwrite(b.u_new_img, 4, cfg.b, o); fwrite(b.u_new_txt, 4, cfg.b, o);
  auto field = [&](const float* p) {      // a per-sample array, dense or a field of the records
    for (int64_t n = 0; n < cfg.N; ++n) fwrite(p + n * S, 4, 1, o);
  };
  field(b.u_img); field(b.u_txt);
  if (with_tau) {
    if (v2) { field(tst.tau_img); field(tst.tau_txt); field(tst.m_img); field(tst.v_img); field(tst.m_txt); field(tst.v_txt); }
    else if (has_tau) { fwrite(tst.tau, 4, 1, o); fwrite(tst.m, 4, 1, o); fwrite(tst.v, 4, 1, o); }
  }
  if (rec) {                               // bytes of the records that belong to no field stay as they were
    for (int64_t n = 0; n < cfg.N; ++n)
      for (int64_t k = 8; k < S; ++k)
        if (rec[n * S + k] != 7.5f) { fprintf(stderr, "record padding touched\n"); return 5; }
  }
  fclose(o);
  return 0;
}
