// Shared declarations of the HIP kernels behind libsttm (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

// Dynamic LDS of a kernel. (The second form serves the host-thread build used by the CPU tests.)
#ifndef STTM_HOST_EMULATION
#define STTM_DYNAMIC_LDS(T, name) extern __shared__ T name[]
#else
#define STTM_DYNAMIC_LDS(T, name) T* name = reinterpret_cast<T*>(hip_emul::g_dynamic_lds)
#endif

// Keeps the instruction scheduler from moving anything across this point (used where hoisting the next batch of
// loads above the work on the current one would cost more registers than the overlap is worth).
#ifndef STTM_HOST_EMULATION
#define STTM_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
#else
#define STTM_SCHED_FENCE() ((void)0)
#endif

namespace sttm {

constexpr int kWave = 64;
constexpr int kMaxLevels = 6;  // P <= 32  =>  levels 0..5

// Problem geometry, passed by value to every kernel.
struct Geo {
  int B, T, H, W, D;
  int P;         // padded power-of-two grid side
  int L;         // root level = log2(P / R)
  int R;         // root nodes per side
  int HW;        // valid cells per frame
  int F;         // frames = B*T
  int NN;        // pyramid nodes per frame (levels 0..L of the P x P grid)
  int lvl_base[kMaxLevels + 1];
  int dtype;     // 0 = f32, 1 = bf16, 2 = f16
  int vec;       // channels per lane per 16-byte load: 4 (f32) / 8 (bf16, f16)
  int cch;       // channels per chunk = 64 * vec (one wavefront spans one chunk of a token row)
  int nC;        // chunks per row = ceil(D / cch)
  int N;         // B*T*H*W
};

// First node index of a level: sum over the finer levels k of (P >> k)^2 = 4 (P^2 - (P >> lvl)^2) / 3. Computed, not
// looked up: with a per-lane level the table in the kernel arguments would cost a memory access each time.
__host__ __device__ inline int level_base(const Geo& g, int lvl) {
  const int q = g.P >> lvl;
  return (g.P * g.P - q * q) * 4 / 3;
}

__host__ __device__ inline int node_index(const Geo& g, int lvl, int by, int bx) {
  return level_base(g, lvl) + by * (g.P >> lvl) + bx;
}

__host__ __device__ inline bool node_exists(const Geo& g, int lvl, int by, int bx) {
  return (by << lvl) < g.H && (bx << lvl) < g.W;
}

// Decodes a per-frame node index into (level, by, bx).
__host__ __device__ inline void node_decode(const Geo& g, int idx, int& lvl, int& by, int& bx) {
  lvl = 0;
  while (lvl < g.L && idx >= level_base(g, lvl + 1)) ++lvl;
  const int r = idx - level_base(g, lvl);
  const int sh = __builtin_ctz((unsigned)g.P) - lvl;  // the level's grid side is a power of two
  by = r >> sh;
  bx = r & ((1 << sh) - 1);
}

// ---- the packed dot product of the target -----------------------------------------------------------------
// c + a.lo * b.lo + a.hi * b.hi on the two 16-bit values each register holds (v_dot2c_f32_bf16, v_dot2_f32_f16: the
// products of two 16-bit values are exact in fp32), and a pair of constants handed over as register contents the
// compiler cannot look into: written as literals, the bf16 pair (1, 0) = 0x00003f80 is encoded as the inline operand
// "1.0", which the instruction does not read as this pair. These three are all that differs in the host-thread
// build of the tests; everything built on them is the same code in both.
#ifndef STTM_HOST_EMULATION
__device__ inline float dot2_bf16(uint32_t a, uint32_t b, float c) {
  typedef __bf16 pair __attribute__((ext_vector_type(2)));
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(pair, a), __builtin_bit_cast(pair, b), c, false);
}
__device__ inline float dot2_f16(uint32_t a, uint32_t b, float c) {
  typedef _Float16 pair __attribute__((ext_vector_type(2)));
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(pair, a), __builtin_bit_cast(pair, b), c, false);
}
template <uint32_t LO, uint32_t HI>
__device__ inline void opaque_pairs(uint32_t& lo, uint32_t& hi) {
  asm volatile("s_mov_b32 %0, %2\n\ts_mov_b32 %1, %3" : "=s"(lo), "=s"(hi) : "i"(LO), "i"(HI));
}
#else
inline float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return fmaf(__uint_as_float(a & 0xffff0000u), __uint_as_float(b & 0xffff0000u),
              fmaf(__uint_as_float(a << 16), __uint_as_float(b << 16), c));
}
inline float dot2_f16(uint32_t a, uint32_t b, float c) {
  return fmaf(__half2float(__ushort_as_half((unsigned short)(a >> 16))),
              __half2float(__ushort_as_half((unsigned short)(b >> 16))),
              fmaf(__half2float(__ushort_as_half((unsigned short)(a & 0xffffu))),
                   __half2float(__ushort_as_half((unsigned short)(b & 0xffffu))), c));
}
template <uint32_t LO, uint32_t HI>
inline void opaque_pairs(uint32_t& lo, uint32_t& hi) { lo = LO; hi = HI; }
#endif

// ---- feature row access: one lane owns `VEC` consecutive channels ------------------------------------
template <int DT> struct Row;  // DT: 0 = f32, 1 = bf16, 2 = f16

template <> struct Row<0> {
  static constexpr int VEC = 4;
  typedef float4 Raw;
  typedef float Elem;
  __device__ static inline Raw zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
  __device__ static inline void unpack(const Raw& r, float (&x)[4]) {
    x[0] = r.x; x[1] = r.y; x[2] = r.z; x[3] = r.w;
  }
  // this lane's share of the dot product of two rows
  __device__ static inline float dot(const Raw& a, const Raw& b) {
    return fmaf(a.x, b.x, fmaf(a.y, b.y, fmaf(a.z, b.z, a.w * b.w)));
  }
  // S += the row's channels
  __device__ static inline void add_row(const Raw& r, float (&S)[4]) {
    S[0] += r.x; S[1] += r.y; S[2] += r.z; S[3] += r.w;
  }
};

template <> struct Row<1> {
  static constexpr int VEC = 8;
  typedef uint4 Raw;
  typedef uint16_t Elem;
  __device__ static inline Raw zero() { return make_uint4(0u, 0u, 0u, 0u); }
  __device__ static inline void unpack(const Raw& r, float (&x)[8]) {
    x[0] = __uint_as_float(r.x << 16); x[1] = __uint_as_float(r.x & 0xffff0000u);
    x[2] = __uint_as_float(r.y << 16); x[3] = __uint_as_float(r.y & 0xffff0000u);
    x[4] = __uint_as_float(r.z << 16); x[5] = __uint_as_float(r.z & 0xffff0000u);
    x[6] = __uint_as_float(r.w << 16); x[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  // Straight from the packed pairs: one instruction multiplies two pairs and adds both products to the running
  // fp32 sum, so nothing has to be unpacked.
  __device__ static inline float dot(const Raw& a, const Raw& b) {
    return dot2_bf16(a.w, b.w, dot2_bf16(a.z, b.z, dot2_bf16(a.y, b.y, dot2_bf16(a.x, b.x, 0.f))));
  }
  // S += the row's channels: the same instruction against the constant pairs (1, 0) and (0, 1) widens a channel and
  // adds it in one step (multiplying the other channel by zero: exact for every finite value, and where a value is an
  // infinity or a NaN in the other element of the pair spills over, into a sum that is undefined then anyway).
  __device__ static inline void add_row(const Raw& r, float (&S)[8]) {
    uint32_t klo, khi;
    opaque_pairs<0x3f80u, 0x3f800000u>(klo, khi);
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      S[2 * j] = dot2_bf16(w[j], klo, S[2 * j]);
      S[2 * j + 1] = dot2_bf16(w[j], khi, S[2 * j + 1]);
    }
  }
};

template <> struct Row<2> {
  static constexpr int VEC = 8;
  typedef uint4 Raw;
  typedef uint16_t Elem;
  __device__ static inline Raw zero() { return make_uint4(0u, 0u, 0u, 0u); }
  __device__ static inline float lo(uint32_t w) { return __half2float(__ushort_as_half((unsigned short)(w & 0xffffu))); }
  __device__ static inline float hi(uint32_t w) { return __half2float(__ushort_as_half((unsigned short)(w >> 16))); }
  __device__ static inline void unpack(const Raw& r, float (&x)[8]) {
    x[0] = lo(r.x); x[1] = hi(r.x); x[2] = lo(r.y); x[3] = hi(r.y);
    x[4] = lo(r.z); x[5] = hi(r.z); x[6] = lo(r.w); x[7] = hi(r.w);
  }
  __device__ static inline float dot(const Raw& a, const Raw& b) {
    return dot2_f16(a.w, b.w, dot2_f16(a.z, b.z, dot2_f16(a.y, b.y, dot2_f16(a.x, b.x, 0.f))));
  }
  // S += the row's channels (see Row<1>::add_row)
  __device__ static inline void add_row(const Raw& r, float (&S)[8]) {
    uint32_t klo, khi;
    opaque_pairs<0x3c00u, 0x3c000000u>(klo, khi);
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      S[2 * j] = dot2_f16(w[j], klo, S[2 * j]);
      S[2 * j + 1] = dot2_f16(w[j], khi, S[2 * j + 1]);
    }
  }
};

// 16-byte accesses for data that is touched once (the gather's rows and its output): marked non-temporal so that
// they do not displace what later kernels want to find in the caches.
#ifndef STTM_HOST_EMULATION
typedef unsigned int sttm_u32x4 __attribute__((ext_vector_type(4)));
typedef float sttm_f32x4 __attribute__((ext_vector_type(4)));
__device__ inline uint4 load_once(const uint4* p) {
  const sttm_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const sttm_u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ inline float4 load_once(const float4* p) {
  const sttm_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const sttm_f32x4*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ inline void store_once(uint4* p, const uint4& v) {
  sttm_u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<sttm_u32x4*>(p));
}
__device__ inline void store_once(float4* p, const float4& v) {
  sttm_f32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<sttm_f32x4*>(p));
}
#else
template <class T> inline T load_once(const T* p) { return *p; }
template <class T> inline void store_once(T* p, const T& v) { *p = v; }
#endif

__device__ inline uint32_t f32_to_f16_rne(float f) { return (uint32_t)__half_as_ushort(__float2half_rn(f)); }

__device__ inline uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Two fp32 values rounded to nearest even and packed into one register (a in the low half): one conversion
// instruction of the target per pair (v_cvt_pk_bf16_f32 / v_cvt_pk_f16_f32); the host-thread build of the tests
// rounds in integer arithmetic.
#ifndef STTM_HOST_EMULATION
__device__ inline uint32_t pack2_bf16(float a, float b) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ inline uint32_t pack2_f16(float a, float b) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}
#else
inline uint32_t pack2_bf16(float a, float b) { return f32_to_bf16_rne(a) | (f32_to_bf16_rne(b) << 16); }
inline uint32_t pack2_f16(float a, float b) { return f32_to_f16_rne(a) | (f32_to_f16_rne(b) << 16); }
#endif

// cos(a, b) from the dot product and the two squared norms: clamped to <= 1, 0 for a zero norm.
__device__ inline float cosine_from(float dot, float na2, float nb2) {
  if (na2 == 0.f || nb2 == 0.f) return 0.f;
  float v = dot / (sqrtf(na2) * sqrtf(nb2));
  return v > 1.f ? 1.f : v;
}

// Monotone map float -> uint32 (order preserving for all non-NaN values).
__device__ inline uint32_t float_key(float v) {
  uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float key_float(uint32_t k) {
  uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(u);
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Orders LDS traffic between the lanes of one wavefront (no cross-wave synchronisation).
__device__ inline void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- budget search state (one per video and stage) ---------------------------------------------------
// Token count as a function of the threshold is K(tau) = base + sum_j w_j [v_j <= tau]; the search is an
// MSB-first radix select (11 + 11 + 10 bits) over the order-preserving integer image of v.
constexpr int kSelBins = 2048;
// What a search pass found, handed to the next launch so that it does not have to derive it again.
struct SelFound {
  unsigned long long budget;  // target - base
  unsigned long long acc;     // weight of the keys below the prefix
  unsigned prefix;            // leading digits of the searched key found so far
  int rc;                     // 0 = searching, 1 = everything fits (tau = 1), 2 = the base alone exceeds the target
};
// The level-0 histogram is fed by hundreds of workgroups whose values fall into a handful of bins; it is kept
// in kSelCopies copies, one per accelerator die (workgroups go to the dies round-robin by their index), so that
// the hot counters stay in one die's L2 instead of travelling between the dies with every atomic.
constexpr int kSelCopies = 8;
struct SelState {
  unsigned hist0[kSelCopies][kSelBins];  // weight per leading digit over all elements; the copies add up
  unsigned hist[2][kSelBins];            // second and third digit under the found prefix
  unsigned lo_out;             // largest key whose leading 22 bits are below the found prefix (0 = none)
  unsigned pad0[3];
  SelFound found[2];           // after the first / second digit
  unsigned pad[16];
};

// One workgroup zeroes a state.
__device__ inline void sel_clear(SelState* st) {
  unsigned* p = reinterpret_cast<unsigned*>(st);
  for (int j = threadIdx.x; j < (int)(sizeof(SelState) / 4); j += blockDim.x) p[j] = 0;
}

// Adds w to hist[digit] for the lanes with valid set; every lane of the wavefront must call it. The two
// most frequent leading digits of the wavefront are combined before the atomic (real similarities sit in
// tight clusters, which would otherwise serialise on one LDS word); whatever is left goes through plain
// LDS atomics.
__device__ inline void wave_hist_add(unsigned* hist, bool valid, unsigned digit, unsigned w) {
  unsigned long long todo = __ballot(valid);
  for (int it = 0; it < 2 && todo; ++it) {
    const int leader = __ffsll((long long)todo) - 1;
    const unsigned d = __shfl(digit, leader, 64);
    const bool mine = valid && digit == d;
    const unsigned long long m = __ballot(mine);
    const unsigned sum = __popcll(__ballot(mine && (w & 1))) + 2u * __popcll(__ballot(mine && (w & 2)));
    if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[d], sum);
    todo &= ~m;
  }
  if ((todo >> (threadIdx.x & 63)) & 1ull) atomicAdd(&hist[digit], w);
}

// Adds a workgroup's LDS histogram of leading digits to the state's level-0 histogram (call after a barrier).
__device__ inline void sel_flush_level0(SelState* st, const unsigned* lds_hist) {
  unsigned* dst = st->hist0[blockIdx.x % kSelCopies];
  for (int j = threadIdx.x; j < kSelBins; j += blockDim.x)
    if (lds_hist[j]) atomicAdd(&dst[j], lds_hist[j]);
}

constexpr int kSelThreads = 256;

// Workgroup-wide (kSelThreads threads): the first bin of `hist` at which acc + running weight exceeds `budget`.
// Returns false when the whole histogram fits. All threads get the same answer.
// *below = largest non-empty bin before the found one, or -1.
// The histogram is the sum of COPIES arrays of kSelBins counters.
template <int COPIES>
__device__ inline bool sel_pick(const unsigned* __restrict__ hist, unsigned long long acc,
                                unsigned long long budget, unsigned* digit, unsigned long long* acc_out,
                                int* below) {
  __shared__ unsigned long long wsum[kSelThreads / 64];
  __shared__ unsigned s_digit;
  __shared__ unsigned long long s_acc;
  __shared__ int s_found, s_below;
  constexpr int PER = kSelBins / kSelThreads;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  unsigned h[PER];
  unsigned long long tot = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) h[j] = 0;
#pragma unroll
  for (int c = 0; c < COPIES; ++c)  // all loads at once
#pragma unroll
    for (int j = 0; j < PER; ++j) h[j] += hist[c * kSelBins + tid * PER + j];
#pragma unroll
  for (int j = 0; j < PER; ++j) tot += h[j];
  unsigned long long inc = tot;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned long long t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  if (tid == 0) { s_found = 0; s_below = -1; }
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  unsigned long long ex = acc + inc - tot;
  for (int w = 0; w < wave; ++w) ex += wsum[w];
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    if (ex <= budget && ex + h[j] > budget) {
      s_found = 1;
      s_digit = (unsigned)(tid * PER + j);
      s_acc = ex;
    }
    ex += h[j];
  }
  __syncthreads();
  const bool found = s_found != 0;
  if (found && below) {
    int mine = -1;  // largest non-empty bin below the found one: per thread, per wavefront, then one LDS atomic each
#pragma unroll
    for (int j = 0; j < PER; ++j)
      if (h[j] && tid * PER + j < (int)s_digit) mine = tid * PER + j;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mine = max(mine, __shfl_xor(mine, o, 64));
    if (lane == 0 && mine >= 0) atomicMax(&s_below, mine);
    __syncthreads();
    *below = s_below;
  }
  *digit = s_digit;
  *acc_out = s_acc;
  __syncthreads();
  return found;
}

// Last digit of a budget search, by a workgroup of kSelThreads threads: tau = midpoint between the searched key
// and the largest key below it. All threads get the value.
__device__ inline float sel_last_digit(const SelState* __restrict__ st) {
  const SelFound fd = st->found[1];
  float t = 1.f;
  if (fd.rc == 2) {
    t = -2.f;
  } else if (fd.rc == 0) {  // uniform over the workgroup
    unsigned d2;
    unsigned long long a2;
    int below;
    if (sel_pick<1>(st->hist[1], fd.acc, fd.budget, &d2, &a2, &below)) {
      const unsigned over = (fd.prefix << 10) | d2;
      const unsigned lo_key = below >= 0 ? ((fd.prefix << 10) | (unsigned)below) : st->lo_out;
      const float hi = key_float(over);
      const float lof = lo_key ? key_float(lo_key) : -2.f;
      t = 0.5f * (lof + hi);
      if (!(t < hi)) t = lof;
    }
  }
  return t;
}

// ---- launchers (defined in the .hip files; all asynchronous on `s`) ------------------------------------

// `sel`: the spatial search states [B]; cleared by the statistics pass, level 0 filled by the finalize kernel.
// `cell_dots`: 1 = also leave x_c(t) . x_c(t+1) of every cell in `part` (the temporal stage then skips those pairs);
// 2 = and S_n(t) . S_n(t+1) of every 2x2 and 4x4 block n.
void launch_pyramid_stats(const Geo& g, const void* feats, int cell_dots, float* part, float* nsum, SelState* sel,
                          hipStream_t s);
// Also works out the levels above an 8x8 unit from the stored unit sums (extends `part` and `nsum`).
void launch_spatial_finalize(const Geo& g, const float* part, float* partu, float* nsum, float* nrm2, float* sim, float* m,
                             uint32_t* sel_key, uint8_t* sel_w, SelState* sel, hipStream_t s);
// `pending` (may be NULL): the search states of a budget search whose last digit has not been resolved yet; the
// kernel then works the threshold out itself (and leaves it in `tau` for later readers) instead of reading `tau`.
void launch_spatial_decide(const Geo& g, const float* m, float* tau, const SelState* pending, int32_t* node_map,
                           uint8_t* node_level, hipStream_t s);
// `dirty`: the state has been searched since its statistics pass (levels 1-2 must be cleared first).
// `tau` == NULL: the last digit is left to the kernel that uses the threshold (see `pending` above).
void launch_select_spatial(const Geo& g, const uint32_t* keys, const uint8_t* weights, const int* target,
                           SelState* state, bool dirty, float* tau, hipStream_t s);
void launch_select_temporal(const Geo& g, const int32_t* node_map, const uint32_t* keys, const int* target,
                            SelState* state, bool dirty, float* tau, hipStream_t s);
inline size_t select_state_bytes(int B) { return (size_t)B * sizeof(SelState); }
// `sel`: the temporal search states [B]; cleared here, level 0 filled by launch_temporal_resolve.
// `skip_same`: 0 = every pair is computed here; 1 = pairs of two single cells are left out, 2 = also pairs of the same
// 2x2 or 4x4 block in both frames (their dot products are in the spatial pass's `part`).
// `items` (temporal_items_bytes() of them) / `item_count`: the work queue of the pass; the count must be zero on
// entry (launch_temporal_resolve leaves it so).
void launch_temporal_dots(const Geo& g, const void* feats, const uint8_t* node_level, const float* nsum,
                          int skip_same, float* pd_part, SelState* sel, void* items, int* item_count,
                          hipStream_t s);
size_t temporal_items_bytes(const Geo& g);
size_t temporal_count_bytes();
// The first pass works in 8x8-cell units (one wavefront per unit, chunk and frame) and leaves each unit's scalars
// as one block of kUnitScalars floats: per 4x4 tile 16 squared norms, 16 cell and 4 level-1 dot products, then the
// 4 level-2 dot products (padded to whole 128-byte lines), then per tile the 16 dot products of its cells with the
// same cells of the next frame, then per tile the dot products of its four 2x2 blocks and of the tile itself with the
// same blocks of the next frame (zeros unless asked for): part[f][chunk][unit][kUnitScalars].
constexpr int kUnitScalars = 256;
constexpr int kUnitCellDots = 160;
constexpr int kUnitNodeDots = 224;
// Offset of cell (y, x)'s cell-to-cell dot product inside its unit's block.
inline __host__ __device__ int unit_cell_dot_slot(int y, int x) {
  return kUnitCellDots + (((y >> 2) & 1) * 2 + ((x >> 2) & 1)) * 16 + (((y >> 1) & 1) * 2 + ((x >> 1) & 1)) * 4 +
         (y & 1) * 2 + (x & 1);
}
// Offset of the frame-to-frame dot product of the node at level 1 or 2 whose top-left cell is (y, x).
inline __host__ __device__ int unit_node_dot_slot(int lvl, int y, int x) {
  return kUnitNodeDots + (((y >> 2) & 1) * 2 + ((x >> 2) & 1)) * 8 + (lvl == 2 ? 4 : ((y >> 1) & 1) * 2 + ((x >> 1) & 1));
}
inline __host__ __device__ int unit_cols(const Geo& g) { return (g.W + 7) >> 3; }
inline __host__ __device__ int unit_rows(const Geo& g) { return (g.H + 7) >> 3; }
// fp32 sums of the pyramid nodes at levels >= 3: [F][nsum_nodes][D]
inline size_t nsum_nodes(const Geo& g) { return g.L >= 3 ? (size_t)(g.NN - g.lvl_base[3]) : 0; }
// `match`: destination rule (0 = top-left-most passing, 1 = the one under the top-left cell only, 2 = most similar).
// `cell_part`: the spatial pass's `part` when it holds frame-to-frame dot products (else NULL), `same_level`: of the
// same node in both frames up to this level (0 = single cells only, 2 = up to 4x4 blocks).
void launch_temporal_resolve(const Geo& g, int match, int same_level, const int32_t* node_map, const uint8_t* node_level,
                             const float* pd_part, const float* cell_part, const float* nrm2, float* sig, float* e,
                             uint32_t* sel_key, SelState* sel, int* item_count, hipStream_t s);
void launch_temporal_parent(const Geo& g, int match, const int32_t* node_map, const uint8_t* node_level,
                            const float* sig, float* tau, const SelState* pending, int32_t* parent, int32_t* ptr,
                            hipStream_t s);
void launch_roots(const Geo& g, int32_t* ptr_a, int32_t* ptr_b, const int32_t* node_map, int32_t* cluster_ids,
                  hipStream_t s);
void launch_node_levels(const Geo& g, const int32_t* node_map, uint8_t* node_level, hipStream_t s);

struct ReduceBuffers {
  int32_t* rank;        // [N]   exclusive count of roots before every cell
  int32_t* key_a;       // [N] sort ping
  int32_t* val_a;       // [N]
  int32_t* key_b;       // [N] sort pong
  int32_t* val_b;       // [N]
  int32_t* order;       // [N] sorted element list (live part first)
  int32_t* orow;        // [N] output row of every list position
  int32_t* hist;        // [tiles][digits] radix histogram of the running pass
  int32_t* tot;         // [digits] column totals (very large inputs)
  int32_t* gsum;        // [groups of tiles][digits] partial column sums (medium inputs)
  int32_t* tile_roots;  // [tiles]
  int32_t* tile_live;   // [tiles]
  int32_t* seg;         // [N+1] first list position of every output row
  int32_t* kdev;        // [4] number of clusters, length of the live list, length of the big-cluster list
  int32_t* zpos;        // [N] output row of every cluster rank under the Z-shaped scan
  int32_t* biglist;     // [big clusters][4] output row, first list position, end of the list, unused
  float* bigpart;       // [gather items][2][D] partial sums of clusters with more than 64 list slots
  int32_t* bigw;        // [gather items][2] member cells behind those partial sums
};
// node_map / node_level: the stage-1 partition, or both NULL (every cell is its own list element).
void launch_reduce_prepare(const Geo& g, const int32_t* cluster_ids, const int32_t* node_map,
                           const uint8_t* node_level, int64_t capacity, int32_t* out_ids, int64_t* offsets,
                           const ReduceBuffers& rb, bool zscan, hipStream_t s);
void launch_reduce_gather(const Geo& g, const void* feats, const float* nsum, const int32_t* node_map,
                          const uint8_t* node_level, int out_dtype, int64_t capacity, void* merged, int32_t* counts,
                          const ReduceBuffers& rb, bool zscan, hipStream_t s);
void launch_reduce_big(const Geo& g, const void* feats, const float* nsum, const int32_t* node_map,
                       const uint8_t* node_level, int out_dtype, int64_t capacity, void* merged, int32_t* counts,
                       const ReduceBuffers& rb, bool zscan, hipStream_t s);
// Position indices of the rows of the reduce call that has just run (its list, ranks and row map are still in `rb`).
void launch_positions(const Geo& g, const int32_t* cluster_ids, const int32_t* node_map, const uint8_t* node_level,
                      const int64_t* offsets,
                      int64_t capacity, const ReduceBuffers& rb, bool zscan, unsigned long long* possum,
                      unsigned* poscnt, int32_t* survived, int32_t* reassigned, float* merged_pos,
                      int32_t* root_tyxl, hipStream_t s);
size_t reduce_bigpart_floats(const Geo& g);
size_t reduce_bigw_entries(const Geo& g);
bool reduce_io_supported(int in_dtype, int out_dtype);
size_t reduce_biglist_entries(const Geo& g);
size_t reduce_hist_entries(int N);
size_t reduce_tiles(int N);
size_t reduce_gsum_entries();

}  // namespace sttm
