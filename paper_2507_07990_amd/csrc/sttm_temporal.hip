// Temporal stage (Sec. 3.3): similarities between every kept node of frame t and the kept nodes of
// frame t-1 it overlaps, directed edges with top-left priority, and the common root of every chain.
#include "sttm_dev.h"

namespace sttm {

__device__ inline void morton_decode(int z, int& dy, int& dx) {
  dx = 0; dy = 0;
#pragma unroll
  for (int b = 0; b < kMaxLevels; ++b) {
    dx |= ((z >> (2 * b)) & 1) << b;
    dy |= ((z >> (2 * b + 1)) & 1) << b;
  }
}

// Sum of the valid cells of the block [y0, y0+s) x [x0, x0+s) of one frame, for this lane's channels.
template <int DT>
__device__ inline void block_sum(const typename Row<DT>::Elem* fb, int D, int H, int W, int y0, int x0, int s,
                                 bool act, float (&S)[Row<DT>::VEC]) {
  typedef Row<DT> R;
  constexpr int VEC = R::VEC;
#pragma unroll
  for (int v = 0; v < VEC; ++v) S[v] = 0.f;
  const int y1 = min(y0 + s, H), x1 = min(x0 + s, W);
  for (int y = y0; y < y1; ++y) {
    int x = x0;
    for (; x + 4 <= x1; x += 4) {
      typename R::Raw r[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        r[j] = R::zero();
        if (act) r[j] = *reinterpret_cast<const typename R::Raw*>(fb + (size_t)(y * W + x + j) * D);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float t[VEC];
        R::unpack(r[j], t);
#pragma unroll
        for (int v = 0; v < VEC; ++v) S[v] += t[v];
      }
    }
    for (; x < x1; ++x) {
      typename R::Raw r = R::zero();
      if (act) r = *reinterpret_cast<const typename R::Raw*>(fb + (size_t)(y * W + x) * D);
      float t[VEC];
      R::unpack(r, t);
#pragma unroll
      for (int v = 0; v < VEC; ++v) S[v] += t[v];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// k_temporal_dots: grid (chunk, frame pair). The two frames' partitions are both quadtree cuts, so any
// two overlapping nodes are nested. The workgroup lists the "join" blocks (the coarser node of every
// overlap); a wavefront takes one join block, sums it in the frame where it is a single node, then
// walks the other frame's nodes inside it in Morton order, summing each and emitting the dot product.
// Output: pd_part[f][chunk][q] for q = top-left cell of the finer node of each overlapping pair.
// ------------------------------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void k_temporal_dots(Geo g, const void* __restrict__ feats_v,
                                                       const int32_t* __restrict__ node_map,
                                                       const uint8_t* __restrict__ node_level,
                                                       float* __restrict__ pd_part) {
  typedef Row<DT> R;
  constexpr int VEC = R::VEC;
  __shared__ uint8_t lvl_t[1024], lvl_p[1024];
  __shared__ int16_t heads[1024];
  __shared__ int ntask, next;
  const int chunk = blockIdx.x;
  const int pair = blockIdx.y;  // frame pairs of all videos: (b, t) with t >= 1
  const int b = pair / (g.T - 1), t = pair - b * (g.T - 1) + 1;
  const int f = b * g.T + t;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int H = g.H, W = g.W, HW = g.HW;
  if (threadIdx.x == 0) { ntask = 0; next = 0; }
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    lvl_t[c] = node_level[(size_t)f * HW + c];
    lvl_p[c] = node_level[(size_t)(f - 1) * HW + c];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    const int a = lvl_t[c], bb = lvl_p[c];
    const int rep = (a >= bb ? node_map[(size_t)f * HW + c] - f * HW
                             : node_map[(size_t)(f - 1) * HW + c] - (f - 1) * HW);
    if (rep == c) heads[atomicAdd(&ntask, 1)] = (int16_t)c;
  }
  __syncthreads();
  const int ch0 = chunk * g.cch + lane * VEC;
  const bool act = ch0 < g.D;
  const typename R::Elem* ft =
      reinterpret_cast<const typename R::Elem*>(feats_v) + (size_t)f * HW * g.D + (act ? ch0 : 0);
  const typename R::Elem* fp = ft - (size_t)HW * g.D;
  float* out = pd_part + (size_t)(f * g.nC + chunk) * HW;
  const int nt = ntask;
  while (true) {
    int ti = 0;
    if (lane == 0) ti = atomicAdd(&next, 1);
    ti = __shfl(ti, 0, 64);
    if (ti >= nt) break;
    const int c = heads[ti];
    const int a = lvl_t[c], bb = lvl_p[c];
    const bool coarse_is_t = a >= bb;
    const int lM = coarse_is_t ? a : bb;
    const int y0 = c / W, x0 = c - y0 * W;
    float SA[VEC];
    block_sum<DT>(coarse_is_t ? ft : fp, g.D, H, W, y0, x0, 1 << lM, act, SA);
    const typename R::Elem* fine = coarse_is_t ? fp : ft;
    const uint8_t* fine_lvl = coarse_is_t ? lvl_p : lvl_t;
    const int nz = 1 << (2 * lM);
    int z = 0;
    while (z < nz) {
      int dy, dx;
      morton_decode(z, dy, dx);
      const int y = y0 + dy, x = x0 + dx;
      if (y >= H || x >= W) { ++z; continue; }
      const int cb = y * W + x;
      const int lf = fine_lvl[cb];
      float SB[VEC];
      block_sum<DT>(fine, g.D, H, W, y, x, 1 << lf, act, SB);
      float d = 0.f;
#pragma unroll
      for (int v = 0; v < VEC; ++v) d = fmaf(SA[v], SB[v], d);
      d = wave_sum(d);
      if (lane == 0) out[cb] = d;
      z += 1 << (2 * lf);
    }
  }
  (void)wave;
}

void launch_temporal_dots(const Geo& g, const void* feats, const int32_t* node_map, const uint8_t* node_level,
                          float* pd_part, hipStream_t s) {
  if (g.T < 2) return;
  dim3 grid(g.nC, g.B * (g.T - 1)), block(256);
  if (g.dtype == 1)
    hipLaunchKernelGGL(k_temporal_dots<1>, grid, block, 0, s, g, feats, node_map, node_level, pd_part);
  else
    hipLaunchKernelGGL(k_temporal_dots<0>, grid, block, 0, s, g, feats, node_map, node_level, pd_part);
}

__device__ inline int node_idx_of(const Geo& g, int lvl, int y0, int x0) {
  return node_index(g, lvl, y0 >> lvl, x0 >> lvl);
}

// Per-frame view of the two partitions in LDS, shared by the two kernels below.
struct PairFrame {
  uint8_t lvl_t[1024], lvl_p[1024];
  int16_t rep_t[1024], rep_p[1024];
};

__device__ inline void load_pair_frame(const Geo& g, int f, const int32_t* node_map, const uint8_t* node_level,
                                       PairFrame& pf) {
  const int HW = g.HW;
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    pf.lvl_t[c] = node_level[(size_t)f * HW + c];
    pf.lvl_p[c] = node_level[(size_t)(f - 1) * HW + c];
    pf.rep_t[c] = (int16_t)(node_map[(size_t)f * HW + c] - f * HW);
    pf.rep_p[c] = (int16_t)(node_map[(size_t)(f - 1) * HW + c] - (f - 1) * HW);
  }
}

// ------------------------------------------------------------------------------------------------
// k_temporal_resolve: one workgroup per frame. Every overlapping (source n in frame t, destination d in
// frame t-1) pair lives at the top-left cell of the finer of the two nodes: the thread of that cell sums
// the per-chunk partial dots in chunk order, divides by the norms from the spatial stage and stores the
// similarity; e_n = max over n's destinations is collected with an integer max in LDS (order-free).
// Also writes the order-preserving integer image of e_n for the budget search (0 = not a candidate).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_temporal_resolve(Geo g, const int32_t* __restrict__ node_map,
                                                          const uint8_t* __restrict__ node_level,
                                                          const float* __restrict__ pd_part,
                                                          const float* __restrict__ nrm2,
                                                          float* __restrict__ sig, float* __restrict__ e,
                                                          uint32_t* __restrict__ sel_key) {
  __shared__ PairFrame pf;
  __shared__ unsigned ekey[1024];
  const int f = blockIdx.x, HW = g.HW, W = g.W;
  if (f % g.T == 0) {
    for (int c = threadIdx.x; c < HW; c += blockDim.x) sel_key[(size_t)f * HW + c] = 0;
    return;
  }
  load_pair_frame(g, f, node_map, node_level, pf);
  for (int c = threadIdx.x; c < HW; c += blockDim.x) ekey[c] = 0;
  __syncthreads();
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    const int a = pf.lvl_t[c], b = pf.lvl_p[c];
    const int n = pf.rep_t[c], d = pf.rep_p[c];
    if ((a <= b ? n : d) != c) continue;  // not the top-left cell of the finer node
    float dot = 0.f;
    for (int k = 0; k < g.nC; ++k) dot += pd_part[(size_t)(f * g.nC + k) * HW + c];
    const float nn = nrm2[(size_t)f * g.NN + node_idx_of(g, a, n / W, n % W)];
    const float nd = nrm2[(size_t)(f - 1) * g.NN + node_idx_of(g, b, d / W, d % W)];
    const float v = cosine_from(dot, nn, nd);
    sig[(size_t)f * HW + c] = v;
    if (v == v) atomicMax(&ekey[n], float_key(v));
  }
  __syncthreads();
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    const size_t i = (size_t)f * HW + c;
    if (pf.rep_t[c] != c) { sel_key[i] = 0; continue; }
    const unsigned k = ekey[c];                 // 0 only if every similarity was NaN
    e[i] = k ? key_float(k) : -2.f;
    sel_key[i] = k ? k : float_key(-2.f);
  }
}

void launch_temporal_resolve(const Geo& g, const int32_t* node_map, const uint8_t* node_level,
                             const float* pd_part, const float* nrm2, float* sig, float* e, uint32_t* sel_key,
                             hipStream_t s) {
  hipLaunchKernelGGL(k_temporal_resolve, dim3(g.F), dim3(256), 0, s, g, node_map, node_level, pd_part, nrm2, sig,
                     e, sel_key);
}

// ------------------------------------------------------------------------------------------------
// k_temporal_parent: directed edge of every kept node (Sec. 3.3): among the destinations whose similarity
// exceeds tau_T the one towards the top-left (smallest raster index; integer min in LDS). Also seeds the
// pointer-jumping array.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_temporal_parent(Geo g, const int32_t* __restrict__ node_map,
                                                         const uint8_t* __restrict__ node_level,
                                                         const float* __restrict__ sig,
                                                         const float* __restrict__ tau,
                                                         int32_t* __restrict__ parent, int32_t* __restrict__ ptr) {
  __shared__ PairFrame pf;
  __shared__ int par[1024];
  const int f = blockIdx.x, HW = g.HW;
  if (f % g.T == 0) {
    for (int c = threadIdx.x; c < HW; c += blockDim.x) {
      parent[(size_t)f * HW + c] = -1;
      ptr[(size_t)f * HW + c] = f * HW + c;
    }
    return;
  }
  load_pair_frame(g, f, node_map, node_level, pf);
  for (int c = threadIdx.x; c < HW; c += blockDim.x) par[c] = 0x7fffffff;
  __syncthreads();
  const float th = tau[f / g.T];
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    const int a = pf.lvl_t[c], b = pf.lvl_p[c];
    const int n = pf.rep_t[c], d = pf.rep_p[c];
    if ((a <= b ? n : d) != c) continue;
    if (sig[(size_t)f * HW + c] > th) atomicMin(&par[n], d);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    const int i = f * HW + c;
    int p = -1;
    if (pf.rep_t[c] == c && par[c] != 0x7fffffff) p = (f - 1) * HW + par[c];
    parent[i] = p;
    ptr[i] = p >= 0 ? p : i;
  }
}

void launch_temporal_parent(const Geo& g, const int32_t* node_map, const uint8_t* node_level, const float* sig,
                            const float* tau, int32_t* parent, int32_t* ptr, hipStream_t s) {
  hipLaunchKernelGGL(k_temporal_parent, dim3(g.F), dim3(256), 0, s, g, node_map, node_level, sig, tau, parent,
                     ptr);
}

// ------------------------------------------------------------------------------------------------
// Common root by pointer jumping (Sec. 3.3, "union-find in a vectorized form"): every edge points one
// frame back, so ceil(log2 T) doublings reach the root.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_root_jump(int n, const int32_t* __restrict__ src,
                                                   int32_t* __restrict__ dst) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[src[i]];
}

__global__ __launch_bounds__(256) void k_cluster_ids(int n, const int32_t* __restrict__ root,
                                                     const int32_t* __restrict__ node_map,
                                                     int32_t* __restrict__ cluster_ids) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) cluster_ids[i] = root[node_map[i]];
}

void launch_roots(const Geo& g, int32_t* ptr_a, int32_t* ptr_b, const int32_t* node_map, int32_t* cluster_ids,
                  hipStream_t s) {
  int rounds = 0;
  while ((1 << rounds) < g.T) ++rounds;
  dim3 grid((g.N + 255) / 256), block(256);
  int32_t* src = ptr_a;
  int32_t* dst = ptr_b;
  for (int r = 0; r < rounds; ++r) {
    hipLaunchKernelGGL(k_root_jump, grid, block, 0, s, g.N, src, dst);
    int32_t* tmp = src; src = dst; dst = tmp;
  }
  hipLaunchKernelGGL(k_cluster_ids, grid, block, 0, s, g.N, src, node_map, cluster_ids);
}

}  // namespace sttm
