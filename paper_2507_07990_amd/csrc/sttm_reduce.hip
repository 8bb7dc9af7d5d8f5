// Reduce stage (Sec. 3.1 / 3.3 / 3.4): one output token per cluster = mean of its member tokens, rows in
// ascending cluster id. Integer plumbing: rank of every root (prefix sum), member lists (stable radix
// sort of the cells by cluster id), then the one feature pass that gathers and averages.
#include "sttm_dev.h"

namespace sttm {

// ---- exclusive prefix sum over int32 -------------------------------------------------------------------
constexpr int kScanBlock = 256;
constexpr int kScanPer = 8;
constexpr int kScanTile = kScanBlock * kScanPer;  // 2048 elements per workgroup

size_t scan_blocks(int n) { return (size_t)(n + kScanTile - 1) / kScanTile; }

// MODE 0: input = in[i]; MODE 1: input = (in[i] == i) (root flags of a cluster map)
template <int MODE> __device__ inline int scan_input(const int32_t* in, int i) {
  return MODE == 0 ? in[i] : (in[i] == i ? 1 : 0);
}

__device__ inline int block_exclusive_scan(int v, int* total) {
  // 256 threads; returns the exclusive prefix of v within the workgroup
  __shared__ int wsum[kScanBlock / kWave];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kScanBlock / kWave; ++w) {
    if (w < wave) base += wsum[w];
    tot += wsum[w];
  }
  __syncthreads();
  *total = tot;
  return base + inc - v;
}

template <int MODE>
__global__ __launch_bounds__(kScanBlock) void k_scan_local(int n, const int32_t* in, int32_t* out,
                                                           int32_t* __restrict__ blocksum) {
  const int base = blockIdx.x * kScanTile + threadIdx.x * kScanPer;
  int v[kScanPer], s = 0;
#pragma unroll
  for (int j = 0; j < kScanPer; ++j) {
    v[j] = (base + j < n) ? scan_input<MODE>(in, base + j) : 0;
    s += v[j];
  }
  int total;
  int ex = block_exclusive_scan(s, &total);
#pragma unroll
  for (int j = 0; j < kScanPer; ++j) {
    if (base + j < n) out[base + j] = ex;
    ex += v[j];
  }
  if (threadIdx.x == 0) blocksum[blockIdx.x] = total;
}

// One workgroup scans the per-block totals in place (exclusive), sequentially over tiles.
__global__ __launch_bounds__(kScanBlock) void k_scan_tops(int nb, int32_t* __restrict__ blocksum,
                                                          int32_t* __restrict__ grand_total) {
  int carry = 0;
  for (int t0 = 0; t0 < nb; t0 += kScanBlock) {
    const int i = t0 + threadIdx.x;
    const int v = i < nb ? blocksum[i] : 0;
    int total;
    const int ex = block_exclusive_scan(v, &total);
    if (i < nb) blocksum[i] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0 && grand_total) *grand_total = carry;
}

__global__ __launch_bounds__(kScanBlock) void k_scan_add(int n, int32_t* __restrict__ out,
                                                         const int32_t* __restrict__ blocksum) {
  const int base = blockIdx.x * kScanTile + threadIdx.x * kScanPer;
  const int add = blocksum[blockIdx.x];
#pragma unroll
  for (int j = 0; j < kScanPer; ++j)
    if (base + j < n) out[base + j] += add;
}

template <int MODE>
static void exclusive_scan(int n, const int32_t* in, int32_t* out, int32_t* blocksum, int32_t* total,
                           hipStream_t s) {
  const int nb = (int)scan_blocks(n);
  hipLaunchKernelGGL(k_scan_local<MODE>, dim3(nb), dim3(kScanBlock), 0, s, n, in, out, blocksum);
  hipLaunchKernelGGL(k_scan_tops, dim3(1), dim3(kScanBlock), 0, s, nb, blocksum, total);
  hipLaunchKernelGGL(k_scan_add, dim3(nb), dim3(kScanBlock), 0, s, n, out, blocksum);
}

// ---- stable LSD radix sort of (key, value) pairs, 11-bit digits --------------------------------------
// A workgroup is one wavefront that owns kSortTile consecutive elements; it handles them 64 at a time in
// index order, so ranks inside the tile are stable without any cross-wave ordering.
constexpr int kSortTile = 1024;
constexpr int kRadixBits = 11;
constexpr int kRadix = 1 << kRadixBits;

size_t reduce_hist_entries(int N) { return (size_t)kRadix * ((N + kSortTile - 1) / kSortTile); }

__global__ __launch_bounds__(64) void k_sort_hist(int n, int shift, const int32_t* __restrict__ keys,
                                                  int32_t* __restrict__ hist, int nblocks) {
  __shared__ int cnt[kRadix];
  for (int j = threadIdx.x; j < kRadix; j += 64) cnt[j] = 0;
  __syncthreads();
  const int base = blockIdx.x * kSortTile;
  for (int o = threadIdx.x; o < kSortTile; o += 64) {
    const int i = base + o;
    if (i < n) atomicAdd(&cnt[(keys[i] >> shift) & (kRadix - 1)], 1);
  }
  __syncthreads();
  for (int j = threadIdx.x; j < kRadix; j += 64) hist[j * nblocks + blockIdx.x] = cnt[j];
}

__global__ __launch_bounds__(64) void k_sort_scatter(int n, int shift, const int32_t* __restrict__ keys,
                                                     const int32_t* __restrict__ vals,
                                                     int32_t* __restrict__ keys_out,
                                                     int32_t* __restrict__ vals_out,
                                                     const int32_t* __restrict__ hist, int nblocks,
                                                     int first_pass) {
  __shared__ int cur[kRadix];
  const int lane = threadIdx.x;
  for (int j = lane; j < kRadix; j += 64) cur[j] = hist[j * nblocks + blockIdx.x];
  __syncthreads();
  const int base = blockIdx.x * kSortTile;
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int o = 0; o < kSortTile; o += 64) {
    const int i = base + o + lane;
    const bool ok = i < n;
    const int key = ok ? keys[i] : 0;
    const int val = ok ? (first_pass ? i : vals[i]) : 0;
    const int digit = (key >> shift) & (kRadix - 1);
    // lanes holding the same digit
    unsigned long long same = __ballot(ok);
#pragma unroll
    for (int bit = 0; bit < kRadixBits; ++bit) {
      const unsigned long long m = __ballot((digit >> bit) & 1);
      same &= ((digit >> bit) & 1) ? m : ~m;
    }
    if (ok) {
      const int rank = __popcll(same & below);
      const int dst = cur[digit] + rank;
      keys_out[dst] = key;
      vals_out[dst] = val;
    }
    __syncthreads();
    if (ok && (same >> lane) >> 1 == 0)  // highest lane of its digit group advances the cursor
      cur[digit] += __popcll(same);
    __syncthreads();
  }
}

// ---- ranks, segment starts, bookkeeping outputs ------------------------------------------------------
__global__ __launch_bounds__(256) void k_fill_i32(int n, int32_t* __restrict__ p, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// out_ids, per-video offsets and the cluster count from the exclusive scan of the root flags.
__global__ __launch_bounds__(256) void k_root_outputs(Geo g, const int32_t* __restrict__ cluster_ids,
                                                      const int32_t* __restrict__ rank,
                                                      const int32_t* __restrict__ kdev, int64_t capacity,
                                                      int32_t* __restrict__ out_ids,
                                                      int64_t* __restrict__ offsets) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= g.N) return;
  if (cluster_ids[i] == i && out_ids && rank[i] < capacity) out_ids[rank[i]] = i;
  const int per_video = g.T * g.HW;
  if (i % per_video == 0) offsets[i / per_video] = rank[i];
  if (i == 0) offsets[g.B] = *kdev;
}

// seg[k] = first sorted position of output row k, seg[K] = N; orow[p] = output row of sorted position p.
__global__ __launch_bounds__(256) void k_segments(int n, const int32_t* __restrict__ skey,
                                                  const int32_t* __restrict__ rank,
                                                  const int32_t* __restrict__ kdev, int32_t* __restrict__ seg,
                                                  int32_t* __restrict__ orow) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= n) return;
  const int key = skey[p];
  const int k = rank[key];
  orow[p] = k;
  if (p == 0 || skey[p - 1] != key) seg[k] = p;
  if (p == n - 1) seg[*kdev] = n;
}

__global__ __launch_bounds__(256) void k_counts(const int32_t* __restrict__ kdev, const int32_t* __restrict__ seg,
                                                int64_t capacity, int32_t* __restrict__ counts) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k < *kdev && k < capacity) counts[k] = seg[k + 1] - seg[k];
}

// ------------------------------------------------------------------------------------------------
// The gather/average pass. The sorted member list is cut into items of kItem consecutive positions;
// an item owns the clusters whose list starts inside it. One wavefront per (item, chunk of the row):
// a lane owns VEC channels. All index look-ups of the item are done lane-parallel first, then all row
// loads are issued, then the rows are summed in list order (ascending flat index, fp32) with the
// cluster boundaries handled as wave-uniform control flow.
// Clusters with more than kBig members are left to the two kernels below, which cut them at fixed
// kBig-aligned list positions so that the summation order does not depend on scheduling.
// ------------------------------------------------------------------------------------------------
constexpr int kItem = 16;
constexpr int kBig = 64;

template <int DT> __device__ inline void acc_row(const typename Row<DT>::Raw& r, float (&acc)[Row<DT>::VEC]) {
  float t[Row<DT>::VEC];
  Row<DT>::unpack(r, t);
#pragma unroll
  for (int v = 0; v < Row<DT>::VEC; ++v) acc[v] += t[v];
}

template <int DT, int ODT>
__device__ inline void store_mean(void* merged_v, size_t elem_off, const float (&acc)[Row<DT>::VEC], float inv) {
  constexpr int VEC = Row<DT>::VEC;
  if (ODT == 0) {
    float* o = reinterpret_cast<float*>(merged_v) + elem_off;
#pragma unroll
    for (int v = 0; v < VEC; v += 4)
      *reinterpret_cast<float4*>(o + v) =
          make_float4(acc[v] * inv, acc[v + 1] * inv, acc[v + 2] * inv, acc[v + 3] * inv);
  } else {
    uint16_t* o = reinterpret_cast<uint16_t*>(merged_v) + elem_off;
    uint32_t w[VEC / 2];
#pragma unroll
    for (int v = 0; v < VEC; v += 2)
      w[v / 2] = f32_to_bf16_rne(acc[v] * inv) | (f32_to_bf16_rne(acc[v + 1] * inv) << 16);
    if (VEC == 8)
      *reinterpret_cast<uint4*>(o) = make_uint4(w[0], w[1], w[2 % (VEC / 2)], w[3 % (VEC / 2)]);
    else
      *reinterpret_cast<uint2*>(o) = make_uint2(w[0], w[1]);
  }
}

template <int DT, int ODT>
__global__ __launch_bounds__(1024) void k_reduce(Geo g, const void* __restrict__ feats_v,
                                                 const int32_t* __restrict__ order,
                                                 const int32_t* __restrict__ orow,
                                                 const int32_t* __restrict__ seg, int64_t capacity,
                                                 void* __restrict__ merged_v) {
  typedef Row<DT> R;
  constexpr int VEC = R::VEC;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
  const int p0 = blockIdx.x * kItem, p1 = min(p0 + kItem, g.N);
  const typename R::Elem* fb = reinterpret_cast<const typename R::Elem*>(feats_v);
  // lane j < kItem describes sorted position p0 + j
  int cell_v = 0, row_v = -1, beg_v = 0, end_v = 0;
  if (lane < kItem && p0 + lane < p1) {
    cell_v = order[p0 + lane];
    row_v = orow[p0 + lane];
    beg_v = seg[row_v];
    end_v = seg[row_v + 1];
  }
  for (int chunk = wave; chunk < g.nC; chunk += nw) {
    const int ch0 = chunk * g.cch + lane * VEC;
    const bool act = ch0 < g.D;
    // issue every row load of the item that this item owns
    typename R::Raw raw[kItem];
#pragma unroll
    for (int j = 0; j < kItem; ++j) {
      const int beg = __shfl(beg_v, j, 64), end = __shfl(end_v, j, 64), cell = __shfl(cell_v, j, 64);
      raw[j] = R::zero();
      const bool use = p0 + j < p1 && beg >= p0 && end - beg <= kBig;  // wave-uniform
      if (use && act) raw[j] = *reinterpret_cast<const typename R::Raw*>(fb + (size_t)cell * g.D + ch0);
    }
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
#pragma unroll
    for (int j = 0; j < kItem; ++j) {
      const int beg = __shfl(beg_v, j, 64), end = __shfl(end_v, j, 64), row = __shfl(row_v, j, 64);
      const bool use = p0 + j < p1 && beg >= p0 && end - beg <= kBig;
      if (!use) continue;
      acc_row<DT>(raw[j], acc);
      const int p = p0 + j;
      if (p + 1 == end || j == kItem - 1 || p + 1 == p1) {
        // the cluster either ends here, or runs past the item: finish it from the list
        for (int q = p + 1; q < end; ++q) {
          typename R::Raw r = R::zero();
          if (act) r = *reinterpret_cast<const typename R::Raw*>(fb + (size_t)order[q] * g.D + ch0);
          acc_row<DT>(r, acc);
        }
        if (act && row < capacity)
          store_mean<DT, ODT>(merged_v, (size_t)row * g.D + ch0, acc, 1.f / (float)(end - beg));
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
      }
    }
  }
}

// Partial sums of the big clusters over fixed windows of kBig list positions: slot 0 = the big cluster
// running into the window from the left, slot 1 = the big cluster starting inside it (at most one each).
template <int DT>
__global__ __launch_bounds__(1024) void k_reduce_big_partial(Geo g, const void* __restrict__ feats_v,
                                                             const int32_t* __restrict__ order,
                                                             const int32_t* __restrict__ orow,
                                                             const int32_t* __restrict__ seg,
                                                             float* __restrict__ bigpart) {
  typedef Row<DT> R;
  constexpr int VEC = R::VEC;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
  const int w0 = blockIdx.x * kBig, w1 = min(w0 + kBig, g.N);
  int beg = -1, end = -1, cell_v = 0;
  if (w0 + lane < w1) {
    const int row = orow[w0 + lane];
    beg = seg[row];
    end = seg[row + 1];
    cell_v = order[w0 + lane];
  }
  const bool big = end - beg > kBig;
  const int beg0 = __shfl(beg, 0, 64), end0 = __shfl(end, 0, 64);
  const bool has_left = (end0 - beg0 > kBig) && beg0 < w0;
  const unsigned long long starts = __ballot(big && beg == w0 + lane);
  if (!has_left && starts == 0) return;
  const typename R::Elem* fb = reinterpret_cast<const typename R::Elem*>(feats_v);
  for (int slot = 0; slot < 2; ++slot) {
    int a, b;
    if (slot == 0) {
      if (!has_left) continue;
      a = w0;
      b = min(end0, w1);
    } else {
      if (starts == 0) continue;
      const int l = __ffsll((long long)starts) - 1;
      a = w0 + l;
      b = min(__shfl(end, l, 64), w1);
    }
    for (int chunk = wave; chunk < g.nC; chunk += nw) {
      const int ch0 = chunk * g.cch + lane * VEC;
      const bool act = ch0 < g.D;
      float acc[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
      // rows a..b-1 of the window, eight loads in flight; the cell of list position w0 + l sits in lane l
      for (int q = a; q < b; q += 8) {
        typename R::Raw r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int cell = __shfl(cell_v, min(q + j, w1 - 1) - w0, 64);
          r[j] = R::zero();
          if (q + j < b && act) r[j] = *reinterpret_cast<const typename R::Raw*>(fb + (size_t)cell * g.D + ch0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (q + j < b) acc_row<DT>(r[j], acc);
      }
      if (!act) continue;
      float* o = bigpart + ((size_t)blockIdx.x * 2 + slot) * g.D + ch0;
#pragma unroll
      for (int v = 0; v < VEC; ++v) o[v] = acc[v];
    }
  }
}

// The window in which a big cluster starts adds up its window partials in window order and stores the mean.
template <int DT, int ODT>
__global__ __launch_bounds__(1024) void k_reduce_big_combine(Geo g, const int32_t* __restrict__ orow,
                                                             const int32_t* __restrict__ seg,
                                                             const float* __restrict__ bigpart, int64_t capacity,
                                                             void* __restrict__ merged_v) {
  constexpr int VEC = Row<DT>::VEC;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
  const int w0 = blockIdx.x * kBig, w1 = min(w0 + kBig, g.N);
  int beg = -1, end = -1, row = -1;
  if (w0 + lane < w1) {
    row = orow[w0 + lane];
    beg = seg[row];
    end = seg[row + 1];
  }
  const unsigned long long starts = __ballot(end - beg > kBig && beg == w0 + lane);
  if (starts == 0) return;
  const int l = __ffsll((long long)starts) - 1;
  const int b = __shfl(beg, l, 64), e = __shfl(end, l, 64), k = __shfl(row, l, 64);
  if (k >= capacity) return;
  const int wlast = (e - 1) / kBig;
  for (int chunk = wave; chunk < g.nC; chunk += nw) {
    const int ch0 = chunk * g.cch + lane * VEC;
    if (ch0 >= g.D) continue;
    float acc[VEC];
    const float* pp = bigpart + ((size_t)blockIdx.x * 2 + 1) * g.D + ch0;
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = pp[v];
    for (int w = blockIdx.x + 1; w <= wlast; ++w) {
      const float* q = bigpart + ((size_t)w * 2) * g.D + ch0;
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] += q[v];
    }
    store_mean<DT, ODT>(merged_v, (size_t)k * g.D + ch0, acc, 1.f / (float)(e - b));
  }
}

size_t reduce_bigpart_floats(const Geo& g) { return (size_t)((g.N + kBig - 1) / kBig) * 2 * g.D; }

// Integer plumbing of the reduce stage; leaves the sorted member list in `*order_out`.
void launch_reduce_prepare(const Geo& g, const int32_t* cluster_ids, int64_t capacity, int32_t* counts,
                           int32_t* out_ids, int64_t* offsets, const ReduceBuffers& rb,
                           const int32_t** order_out, hipStream_t s) {
  const int N = g.N;
  const dim3 b256(256), gN((N + 255) / 256);
  // ranks of the roots, K, per-video offsets, out_ids
  exclusive_scan<1>(N, cluster_ids, rb.rank, rb.blocksum, rb.kdev, s);
  hipLaunchKernelGGL(k_root_outputs, gN, b256, 0, s, g, cluster_ids, rb.rank, rb.kdev, capacity, out_ids,
                     offsets);
  // member lists: stable sort of the cells by cluster id
  int bits = 1;
  while ((1ll << bits) < (long long)N) ++bits;
  const int nblocks = (N + kSortTile - 1) / kSortTile;
  const int32_t* kin = cluster_ids;
  const int32_t* vin = nullptr;
  int32_t* kout = rb.key_a;
  int32_t* vout = rb.val_a;
  int pass = 0;
  for (int shift = 0; shift < bits; shift += kRadixBits, ++pass) {
    hipLaunchKernelGGL(k_sort_hist, dim3(nblocks), dim3(64), 0, s, N, shift, kin, rb.hist, nblocks);
    exclusive_scan<0>(kRadix * nblocks, rb.hist, rb.hist, rb.blocksum, (int32_t*)nullptr, s);
    hipLaunchKernelGGL(k_sort_scatter, dim3(nblocks), dim3(64), 0, s, N, shift, kin, vin, kout, vout, rb.hist,
                       nblocks, pass == 0 ? 1 : 0);
    kin = kout;
    vin = vout;
    if (kout == rb.key_a) { kout = rb.key_b; vout = rb.val_b; } else { kout = rb.key_a; vout = rb.val_a; }
  }
  // kout is now the free key buffer: it receives the output row of every sorted position
  hipLaunchKernelGGL(k_segments, gN, b256, 0, s, N, kin, rb.rank, rb.kdev, rb.seg, kout);
  if (counts) hipLaunchKernelGGL(k_counts, gN, b256, 0, s, rb.kdev, rb.seg, capacity, counts);
  *order_out = vin;
  rb.orow_out[0] = kout;
}

// The feature pass of the reduce stage (three kernels; the two for big clusters exit at once when there are none).
void launch_reduce_gather(const Geo& g, const void* feats, int out_dtype, int64_t capacity, void* merged,
                          const ReduceBuffers& rb, const int32_t* order, hipStream_t s) {
  const int32_t* orow = rb.orow_out[0];
  const int nitems = (g.N + kItem - 1) / kItem;
  const int nwin = (g.N + kBig - 1) / kBig;
  const int nw = g.nC < 16 ? g.nC : 16;
  dim3 grid(nitems), gridw(nwin), block(64 * nw);
#define STTM_REDUCE(DT, ODT)                                                                                     \
  do {                                                                                                           \
    hipLaunchKernelGGL((k_reduce<DT, ODT>), grid, block, 0, s, g, feats, order, orow, rb.seg, capacity, merged); \
    hipLaunchKernelGGL((k_reduce_big_partial<DT>), gridw, block, 0, s, g, feats, order, orow, rb.seg,            \
                       rb.bigpart);                                                                              \
    hipLaunchKernelGGL((k_reduce_big_combine<DT, ODT>), gridw, block, 0, s, g, orow, rb.seg, rb.bigpart,         \
                       capacity, merged);                                                                        \
  } while (0)
  if (g.dtype == 1) {
    if (out_dtype == 1) STTM_REDUCE(1, 1); else STTM_REDUCE(1, 0);
  } else {
    if (out_dtype == 1) STTM_REDUCE(0, 1); else STTM_REDUCE(0, 0);
  }
#undef STTM_REDUCE
}

}  // namespace sttm
