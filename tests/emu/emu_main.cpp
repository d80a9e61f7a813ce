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
// V2: tau_img, tau_txt [N], has_glob: u_glob_img, u_glob_txt [B] and for V2 tau_glob_img, tau_glob_txt [B]
int main(int argc, char** argv) {
  emu::g_lds_hi = (uintptr_t)&emu::g_marker & ~(uintptr_t)0xffffffffull;
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
  const fastclip_status st = fastclip_step(&cfg, &b, ws, need, nullptr);
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
  fwrite(b.u_img, 4, cfg.N, o); fwrite(b.u_txt, 4, cfg.N, o);
  fclose(o);
  return 0;
}
