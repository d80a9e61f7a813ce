// CPU stand-in for the HIP runtime and for the gfx950 builtins that libfastclip's sources use, so that the very
// sources of the kernels can be compiled for the host and run under AddressSanitizer (or the thread / memory
// sanitizers): every GPU thread is an OS thread, the threads of a workgroup run together, workgroups run one after
// another.  Wave-wide operations (MFMA, transposing LDS reads, lane exchanges) meet in a per-wave buffer; direct-to-LDS
// loads copy at once.  Test infrastructure only: nothing of the product is built from this.
#pragma once
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <condition_variable>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __shared__ static
#define __launch_bounds__(...)

struct dim3 { unsigned x, y, z; dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {} };
struct float4 { float x, y, z, w; };
struct float2 { float x, y; };
struct uint4 { uint32_t x, y, z, w; };
struct uint2 { uint32_t x, y; };
static inline float4 make_float4(float x, float y, float z, float w) { return float4{x, y, z, w}; }

typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidSymbol = 13 };
typedef void* hipStream_t;
typedef void* hipEvent_t;
enum { hipMemcpyDeviceToHost = 2 };
static inline hipError_t hipGetLastError() { return hipSuccess; }
static inline const char* hipGetErrorString(hipError_t) { return "emu"; }
static inline hipError_t hipEventCreate(hipEvent_t* e) { *e = nullptr; return hipSuccess; }
static inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
static inline hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
static inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }
static inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
static inline hipError_t hipMemcpy(void* d, const void* s, size_t n, int) { memcpy(d, s, n); return hipSuccess; }
static inline hipError_t hipMemcpyAsync(void* d, const void* s, size_t n, int, hipStream_t) { memcpy(d, s, n); return hipSuccess; }
static inline hipError_t hipMemsetAsync(void* d, int v, size_t n, hipStream_t) { memset(d, v, n); return hipSuccess; }
static inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
#define HIP_SYMBOL(x) (&(x))
static inline hipError_t hipGetSymbolAddress(void** p, const void* sym) { *p = (void*)sym; return hipSuccess; }
#define __align__(n) __attribute__((aligned(n)))

namespace emu {
// barrier whose number of participants shrinks when a thread leaves (a finished wave takes no part in s_barrier)
struct Barrier {
  std::mutex m; std::condition_variable cv; int active = 0, waiting = 0; unsigned gen = 0;
  void reset(int n) { active = n; waiting = 0; }
  void wait() {
    std::unique_lock<std::mutex> l(m);
    const unsigned g = gen;
    if (++waiting == active) { waiting = 0; ++gen; cv.notify_all(); return; }
    cv.wait(l, [&] { return gen != g; });
  }
  void leave() {
    std::unique_lock<std::mutex> l(m);
    --active;
    if (active > 0 && waiting == active) { waiting = 0; ++gen; cv.notify_all(); }
  }
};
struct Wave { Barrier bar; alignas(64) unsigned char buf[2][64][64]; };
struct Block { Barrier bar; std::vector<Wave> waves; };
extern thread_local Block* t_block;
extern thread_local Wave* t_wave;
extern thread_local int t_lane;
extern uintptr_t g_lds_hi;      // upper 32 bits shared by every static (LDS) object of the image
}  // namespace emu

extern thread_local dim3 threadIdx, blockIdx;
extern dim3 blockDim, gridDim;

#define __syncthreads() emu::t_block->bar.wait()
#define __builtin_amdgcn_s_barrier() emu::t_block->bar.wait()
#define __builtin_amdgcn_s_waitcnt(x) ((void)0)
#define __builtin_amdgcn_sched_barrier(x) ((void)0)
#define __builtin_amdgcn_readfirstlane(x) (x)
#define __builtin_amdgcn_exp2f(x) exp2f(x)
#define __builtin_amdgcn_rcpf(x) (1.0f / (x))
#define __fmul_rn(a, b) ((a) * (b))
static inline float __uint_as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static inline uint64_t wall_clock64() { return 0; }
static inline unsigned long long atomicCAS(unsigned long long* p, unsigned long long cmp, unsigned long long val) {
  __atomic_compare_exchange_n(p, &cmp, val, false, __ATOMIC_SEQ_CST, __ATOMIC_SEQ_CST);
  return cmp;
}

template <typename T>
static inline T __shfl_xor(T v, int mask) {
  emu::Wave* w = emu::t_wave;
  memcpy(w->buf[0][emu::t_lane], &v, sizeof(T));
  w->bar.wait();
  T r;
  memcpy(&r, w->buf[0][emu::t_lane ^ mask], sizeof(T));
  w->bar.wait();
  return r;
}

// 16 (or 4) bytes per lane from base + off into LDS at lds32 + bytes * lane, at once
static inline void emu_dma(const void* base, uint32_t off, uint32_t lds32, int bytes) {
  char* dst = (char*)(emu::g_lds_hi | (uintptr_t)lds32) + (size_t)bytes * emu::t_lane;
  memcpy(dst, (const char*)base + off, bytes);
}

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 emu_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float emu_f32x16;
static inline float emu_bf2f(__bf16 x) { uint16_t b; memcpy(&b, &x, 2); return __uint_as_float((uint32_t)b << 16); }
// D = A B + C, 32 x 32 x 16: lane (i, h) gives A[i][8h .. 8h+7] and B[8h .. 8h+7][i]; D[8 (v >> 2) + 4 h + (v & 3)][i] in v
static inline emu_f32x16 __builtin_amdgcn_mfma_f32_32x32x16_bf16(emu_bf16x8 a, emu_bf16x8 b, emu_f32x16 c, int, int, int) {
  emu::Wave* w = emu::t_wave;
  const int lane = emu::t_lane;
  memcpy(w->buf[0][lane], &a, 16);
  memcpy(w->buf[1][lane], &b, 16);
  w->bar.wait();
  const int n = lane & 31, h = lane >> 5;
  for (int v = 0; v < 16; ++v) {
    const int row = 8 * (v >> 2) + 4 * h + (v & 3);
    float s = 0.f;
    for (int k = 0; k < 16; ++k) {
      __bf16 x, y;
      memcpy(&x, w->buf[0][row + 32 * (k >> 3)] + 2 * (k & 7), 2);
      memcpy(&y, w->buf[1][n + 32 * (k >> 3)] + 2 * (k & 7), 2);
      s += emu_bf2f(x) * emu_bf2f(y);
    }
    c[v] += s;
  }
  w->bar.wait();
  return c;
}
typedef short emu_v4s __attribute__((ext_vector_type(4)));
// groups of 16 lanes: lane s reads 4 values (a row piece); lane L receives value (L & 3) of the lanes 4 e + (L >> 2)
static inline emu_v4s emu_ds_read_tr16_b64(uintptr_t p32) {
  emu::Wave* w = emu::t_wave;
  const int lane = emu::t_lane;
  const char* src = (const char*)(emu::g_lds_hi | (uintptr_t)(uint32_t)p32);
  memcpy(w->buf[0][lane], src, 8);
  w->bar.wait();
  const int g = lane & ~15, L = lane & 15;
  emu_v4s r;
  for (int e = 0; e < 4; ++e) {
    short v;
    memcpy(&v, w->buf[0][g + 4 * e + (L >> 2)] + 2 * (L & 3), 2);
    r[e] = v;
  }
  w->bar.wait();
  return r;
}
#define __builtin_amdgcn_ds_read_tr16_b64_v4i16(p) emu_ds_read_tr16_b64((uintptr_t)(p))

namespace emu { void launch(dim3 grid, dim3 block, const std::function<void()>& body); }
#define hipLaunchKernelGGL(kern, grid, block, shmem, stream, ...) emu::launch((grid), (block), [&] { kern(__VA_ARGS__); })
