// Minimal CPU stand-in for the parts of the HIP runtime and device language that libsttm uses.
// TEST INFRASTRUCTURE ONLY: it lets the kernels be compiled with g++ and run on host threads (one OS
// thread per GPU thread of a workgroup, workgroups one after the other), so that hangs, out-of-bounds
// accesses and races can be hunted with timeouts, AddressSanitizer and gdb without a GPU.
// Wavefront collectives (__shfl*, __ballot, wave barrier) assume the 64 lanes of a wavefront call them
// together, exactly as the kernels themselves require on the GPU.
#pragma once
#include <pthread.h>
#include <stdint.h>
#include <string.h>
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <tuple>
#include <utility>
#include <vector>

#define STTM_HOST_EMULATION 1
#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __shared__ static
#define __launch_bounds__(...)
#define __restrict__
#define __align__(n) alignas(n)
#define HIP_SYMBOL(x) (x)

struct dim3 {
  unsigned x, y, z;
  dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
struct float4 { float x, y, z, w; };
struct uint4 { unsigned x, y, z, w; };
struct uint2 { unsigned x, y; };
struct int4 { int x, y, z, w; };
inline float4 make_float4(float a, float b, float c, float d) { return {a, b, c, d}; }
inline uint4 make_uint4(unsigned a, unsigned b, unsigned c, unsigned d) { return {a, b, c, d}; }
inline uint2 make_uint2(unsigned a, unsigned b) { return {a, b}; }
inline int4 make_int4(int a, int b, int c, int d) { return {a, b, c, d}; }

namespace hip_emul {
extern thread_local dim3 t_threadIdx, t_blockIdx;
extern dim3 g_blockDim, g_gridDim;
struct Wave {
  pthread_barrier_t bar;
  uint64_t slot[64];
};
extern thread_local Wave* t_wave;
extern pthread_barrier_t g_block_bar;
extern float g_dynamic_lds[];
inline void wave_sync() { pthread_barrier_wait(&t_wave->bar); }
inline uint64_t exchange(uint64_t v, int src_lane) {
  const int lane = t_threadIdx.x & 63;
  t_wave->slot[lane] = v;
  wave_sync();
  const uint64_t r = t_wave->slot[src_lane & 63];
  wave_sync();
  return r;
}
void launch(dim3 grid, dim3 block, void (*body)(void*), void* closure);
}  // namespace hip_emul

#define threadIdx (hip_emul::t_threadIdx)
#define blockIdx (hip_emul::t_blockIdx)
#define blockDim (hip_emul::g_blockDim)
#define gridDim (hip_emul::g_gridDim)

inline void __syncthreads() { pthread_barrier_wait(&hip_emul::g_block_bar); }
#define __builtin_amdgcn_fence(order, scope) __atomic_thread_fence(__ATOMIC_SEQ_CST)
#define __builtin_amdgcn_wave_barrier() hip_emul::wave_sync()
#define __builtin_amdgcn_readfirstlane(x) (x)  // only applied to values that are the same in every lane

inline float __uint_as_float(unsigned u) { float f; memcpy(&f, &u, 4); return f; }
inline unsigned __float_as_uint(float f) { unsigned u; memcpy(&u, &f, 4); return u; }
inline int __popcll(unsigned long long v) { return __builtin_popcountll(v); }
inline int __ffsll(long long v) { return __builtin_ffsll(v); }
using std::max;
using std::min;

template <class T> inline T __shfl(T v, int src, int = 64) {
  uint64_t raw = 0;
  memcpy(&raw, &v, sizeof(T));
  raw = hip_emul::exchange(raw, src);
  T r;
  memcpy(&r, &raw, sizeof(T));
  return r;
}
template <class T> inline T __shfl_xor(T v, int mask, int = 64) {
  return __shfl(v, (int)(hip_emul::t_threadIdx.x & 63) ^ mask);
}
template <class T> inline T __shfl_up(T v, int delta, int = 64) {
  const int lane = hip_emul::t_threadIdx.x & 63;
  return __shfl(v, lane >= delta ? lane - delta : lane);
}
template <class T> inline T __shfl_down(T v, int delta, int = 64) {
  const int lane = hip_emul::t_threadIdx.x & 63;
  return __shfl(v, lane + delta < 64 ? lane + delta : lane);
}
inline unsigned long long __ballot(int pred) {
  const int lane = hip_emul::t_threadIdx.x & 63;
  hip_emul::t_wave->slot[lane] = pred ? 1 : 0;
  hip_emul::wave_sync();
  unsigned long long m = 0;
  for (int l = 0; l < 64; ++l) m |= (unsigned long long)(hip_emul::t_wave->slot[l] & 1) << l;
  hip_emul::wave_sync();
  return m;
}

template <class T> inline T atomicAdd(T* p, T v) { return __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST); }
inline unsigned atomicMax(unsigned* p, unsigned v) {
  unsigned old = __atomic_load_n(p, __ATOMIC_SEQ_CST);
  while (old < v && !__atomic_compare_exchange_n(p, &old, v, false, __ATOMIC_SEQ_CST, __ATOMIC_SEQ_CST)) {}
  return old;
}
inline unsigned long long atomicMax(unsigned long long* p, unsigned long long v) {
  unsigned long long old = __atomic_load_n(p, __ATOMIC_SEQ_CST);
  while (old < v && !__atomic_compare_exchange_n(p, &old, v, false, __ATOMIC_SEQ_CST, __ATOMIC_SEQ_CST)) {}
  return old;
}
inline int atomicMax(int* p, int v) {
  int old = __atomic_load_n(p, __ATOMIC_SEQ_CST);
  while (old < v && !__atomic_compare_exchange_n(p, &old, v, false, __ATOMIC_SEQ_CST, __ATOMIC_SEQ_CST)) {}
  return old;
}
template <class T> inline T atomicExch(T* p, T v) { return __atomic_exchange_n(p, v, __ATOMIC_SEQ_CST); }
inline void __threadfence() { __atomic_thread_fence(__ATOMIC_SEQ_CST); }
inline int atomicMin(int* p, int v) {
  int old = __atomic_load_n(p, __ATOMIC_SEQ_CST);
  while (old > v && !__atomic_compare_exchange_n(p, &old, v, false, __ATOMIC_SEQ_CST, __ATOMIC_SEQ_CST)) {}
  return old;
}

// ---- half precision (what <hip/hip_fp16.h> provides on the GPU), bit-exact conversions ---------------
struct __half { unsigned short x; };
inline __half __ushort_as_half(unsigned short u) { return __half{u}; }
inline unsigned short __half_as_ushort(__half h) { return h.x; }
inline float __half2float(__half h) {
  const unsigned s = (h.x >> 15) & 1u, e = (h.x >> 10) & 31u, m = h.x & 1023u;
  unsigned u;
  if (e == 0) {
    if (m == 0) { u = s << 31; }
    else {  // subnormal: value = m * 2^-24
      float f = (float)m * 5.9604644775390625e-08f;
      return s ? -f : f;
    }
  } else if (e == 31) {
    u = (s << 31) | 0x7f800000u | (m << 13);
  } else {
    u = (s << 31) | ((e + 112u) << 23) | (m << 13);
  }
  float f;
  __builtin_memcpy(&f, &u, 4);
  return f;
}
inline __half __float2half_rn(float f) {  // round to nearest even
  unsigned u;
  __builtin_memcpy(&u, &f, 4);
  const unsigned s = (u >> 16) & 0x8000u;
  const unsigned a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return __half{(unsigned short)(s | 0x7e00u)};           // NaN
  if (a >= 0x47800000u) return __half{(unsigned short)(s | 0x7c00u)};          // >= 65536 (rounds to inf); inf
  if (a < 0x33000000u) return __half{(unsigned short)s};                       // < 2^-25: zero
  if (a < 0x38800000u) {                                                        // subnormal half
    const float af = f < 0 ? -f : f;
    const float scaled = af * 16777216.0f;                                      // / 2^-24: exact
    unsigned q = (unsigned)scaled;
    const float rem = scaled - (float)q;
    if (rem > 0.5f || (rem == 0.5f && (q & 1u))) ++q;
    return __half{(unsigned short)(s | q)};
  }
  unsigned r = a - 0x38000000u;                                                 // rebias exponent
  const unsigned lsb = (r >> 13) & 1u;
  r += 0xfffu + lsb;
  r >>= 13;
  if (r >= 0x7c00u) r = 0x7c00u;
  return __half{(unsigned short)(s | r)};
}

// ---- host API subset -------------------------------------------------------------------------------
typedef int hipError_t;
constexpr hipError_t hipSuccess = 0;
typedef void* hipStream_t;
typedef void* hipEvent_t;
enum hipMemcpyKind { hipMemcpyHostToDevice, hipMemcpyDeviceToHost, hipMemcpyDeviceToDevice };
inline const char* hipGetErrorString(hipError_t) { return "emulated"; }
inline hipError_t hipGetDeviceCount(int* n) { *n = 1; return hipSuccess; }
inline hipError_t hipSetDevice(int) { return hipSuccess; }
template <class T> inline hipError_t hipGetSymbolAddress(void** p, T& sym) { *p = (void*)&sym; return hipSuccess; }
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
inline hipError_t hipMemcpyAsync(void* d, const void* s, size_t n, hipMemcpyKind, hipStream_t) {
  memcpy(d, s, n);
  return hipSuccess;
}
inline hipError_t hipMemsetAsync(void* d, int v, size_t n, hipStream_t) { memset(d, v, n); return hipSuccess; }
inline hipError_t hipEventCreate(hipEvent_t* e) { *e = nullptr; return hipSuccess; }
inline hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }

template <class... P, class... A>
inline void hip_emul_launch(void (*k)(P...), dim3 grid, dim3 block, size_t, hipStream_t, A... args) {
  std::tuple<P...> t(static_cast<P>(args)...);
  struct C { void (*k)(P...); std::tuple<P...>* t; } c{k, &t};
  hip_emul::launch(grid, block, [](void* p) {
    C* cc = static_cast<C*>(p);
    std::apply(cc->k, *cc->t);
  }, &c);
}
#define hipLaunchKernelGGL(kernel, grid, block, lds, stream, ...) \
  hip_emul_launch(kernel, grid, block, lds, stream, __VA_ARGS__)
