// Reduce stage (Sec. 3.1 / 3.3 / 3.4): one output token per cluster = mean of its member tokens, rows in
// ascending cluster id. Integer plumbing: rank of every root (prefix sum over tiles), member lists (stable
// LSD radix sort of the list elements by cluster id), then the one feature pass that gathers and averages.
//
// A list element is a cell, or -- when the caller hands over the stage-1 partition -- a whole node at level
// >= 3, represented by its top-left cell: its per-channel sum was stored by the spatial pass, so its up to
// 4^level cells are not read again; the other cells of such a node take no part in the list ("dropped", key -1).
#include "sttm_dev.h"

namespace sttm {

constexpr int kSortThreads = 256;
constexpr int kSortPer = 8;
constexpr int kSortTile = kSortThreads * kSortPer;  // 2048 elements per workgroup
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kMaxDigitBits = 11;
constexpr int kItem = 16;  // list positions per gather item
constexpr int kBig = 64;   // clusters with more list slots than this are summed item by item, then combined
constexpr int kTail = 8;
constexpr int kMaxDigits = 1 << kMaxDigitBits;
// How a scatter workgroup gets its start offsets from hist[tile][digit]: up to kDirectTiles tiles it adds up all
// rows itself; up to kGroupTiles * kMaxGroups tiles a small kernel first adds the rows in groups of kGroupTiles
// and the workgroup adds the group sums and the rows of its own group; beyond that k_sort_colscan turns the
// columns into running sums in place.
constexpr int kDirectTiles = 64;
constexpr int kGroupTiles = 32;
constexpr int kMaxGroups = 256;

struct SortPlan {
  int passes, dbits, nb;
  int mode;  // 0 = direct, 1 = grouped, 2 = column scan
};

static SortPlan sort_plan(int N) {
  SortPlan p;
  int bits = 1;
  while ((1ll << bits) < (long long)N) ++bits;  // keys 0..N-1
  p.passes = (bits + kMaxDigitBits - 1) / kMaxDigitBits;
  p.dbits = (bits + p.passes - 1) / p.passes;
  if (p.dbits < 2) p.dbits = 2;  // a histogram row is read in pieces of four digits
  p.nb = (N + kSortTile - 1) / kSortTile;
  p.mode = p.nb <= kDirectTiles ? 0 : (p.nb <= kGroupTiles * kMaxGroups ? 1 : 2);
  return p;
}

size_t reduce_tiles(int N) { return (size_t)(N + kSortTile - 1) / kSortTile; }
size_t reduce_gsum_entries() { return (size_t)kMaxGroups * kMaxDigits; }
size_t reduce_hist_entries(int N) { return (size_t)kMaxDigits * reduce_tiles(N); }

// Exclusive prefix of v over the 256 threads of the workgroup; *total = sum over all threads.
__device__ inline int block_exclusive_scan(int v, int* total) {
  __shared__ int wsum[kSortWaves];
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
  for (int w = 0; w < kSortWaves; ++w) {
    if (w < wave) base += wsum[w];
    tot += wsum[w];
  }
  __syncthreads();
  *total = tot;
  return base + inc - v;
}

// Sum of v over the workgroup, returned to every thread.
__device__ inline int block_sum(int v) {
  int total;
  (void)block_exclusive_scan(v, &total);
  return total;
}

__device__ inline int node_cells(const Geo& g, int cell_in_frame, int lvl) {
  const int y = cell_in_frame / g.W, x = cell_in_frame - y * g.W, s = 1 << lvl;
  return (min(y + s, g.H) - y) * (min(x + s, g.W) - x);
}
// True when the node with top-left cell c (in-frame index) at level lv is represented by its stored sum.
__device__ inline bool node_is_summed(const Geo& g, int c, int lv) { return lv >= 3 && node_cells(g, c, lv) >= 2; }
// The cell that stands for the second half of a summed node: the next valid cell of the node in raster order.
__device__ inline int node_second_cell(const Geo& g, int c) { return (c % g.W) + 1 < g.W ? c + 1 : c + g.W; }

// ------------------------------------------------------------------------------------------------
// k_reduce_prep: one workgroup per tile of 2048 cells. Sort keys (cluster id, or -1 for a cell covered by a
// stored node sum), tile-local exclusive ranks of the roots (cells that are their own cluster id), the
// tile's totals, and the tile's digit histogram of the first sort pass.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSortThreads) void k_reduce_prep(Geo g, const int32_t* __restrict__ cluster_ids,
                                                              const int32_t* __restrict__ node_map,
                                                              const uint8_t* __restrict__ node_level, int dbits,
                                                              int32_t* __restrict__ keys, int32_t* __restrict__ rank,
                                                              int32_t* __restrict__ tile_roots,
                                                              int32_t* __restrict__ tile_live,
                                                              int32_t* __restrict__ hist,
                                                              int32_t* __restrict__ bigcount) {
  __shared__ int cnt[kMaxDigits];
  const int DIG = 1 << dbits, b = blockIdx.x, tid = threadIdx.x;
  for (int d = tid; d < DIG; d += kSortThreads) cnt[d] = 0;
  if (b == 0 && tid == 0) *bigcount = 0;  // the list of big clusters starts empty
  __syncthreads();
  const int i0 = b * kSortTile + tid * kSortPer;
  int root[kSortPer], nroot = 0, nlive = 0;
  int cidv[kSortPer], repv[kSortPer], lvv[kSortPer];
#pragma unroll
  for (int j = 0; j < kSortPer; ++j) {  // all loads first: they do not depend on one another
    const int i = i0 + j;
    cidv[j] = repv[j] = lvv[j] = 0;
    if (i < g.N) {
      cidv[j] = cluster_ids[i];
      if (node_map) {
        repv[j] = node_map[i];
        lvv[j] = node_level[i];
      }
    }
  }
#pragma unroll
  for (int j = 0; j < kSortPer; ++j) {
    const int i = i0 + j;
    root[j] = 0;
    if (i < g.N) {
      const int cid = cidv[j];
      bool live = true;
      if (lvv[j] >= 3) {  // a node with a stored sum: only the cells standing for it stay
        const int rep = repv[j], c = rep % g.HW;
        if (node_is_summed(g, c, lvv[j]))
          live = i == rep || (g.vec == 8 && i == rep - c + node_second_cell(g, c));
      }
      keys[i] = live ? cid : -1;
      root[j] = cid == i;
      nroot += root[j];
      nlive += live;
      if (live) atomicAdd(&cnt[cid & (DIG - 1)], 1);
    }
  }
  int total;
  int ex = block_exclusive_scan(nroot, &total);
#pragma unroll
  for (int j = 0; j < kSortPer; ++j) {
    if (i0 + j < g.N) rank[i0 + j] = ex;
    ex += root[j];
  }
  const int live_total = block_sum(nlive);
  if (tid == 0) {
    tile_roots[b] = total;
    tile_live[b] = live_total;
  }
  __syncthreads();
  for (int d = tid; d < DIG; d += kSortThreads) hist[(size_t)b * DIG + d] = cnt[d];
}

// Digit histogram per tile of the (compacted) keys of a later pass; tiles beyond the list write zeros.
__global__ __launch_bounds__(kSortThreads) void k_sort_hist(const int32_t* __restrict__ kdev, int shift, int dbits,
                                                            const int32_t* __restrict__ keys,
                                                            int32_t* __restrict__ hist) {
  __shared__ int cnt[kMaxDigits];
  const int DIG = 1 << dbits, b = blockIdx.x, tid = threadIdx.x, n = kdev[1];
  for (int d = tid; d < DIG; d += kSortThreads) cnt[d] = 0;
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kSortPer; ++j) {
    const int i = b * kSortTile + j * kSortThreads + tid;
    if (i < n) atomicAdd(&cnt[(keys[i] >> shift) & (DIG - 1)], 1);
  }
  __syncthreads();
  for (int d = tid; d < DIG; d += kSortThreads) hist[(size_t)b * DIG + d] = cnt[d];
}

__global__ __launch_bounds__(256) void k_fill_i32(int n, int32_t* __restrict__ p, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Large inputs only: turns every column (digit) of hist[tile][digit] into its exclusive prefix over the
// tiles and leaves the column total in tot[digit].
__global__ __launch_bounds__(256) void k_sort_colscan(int nb, int DIG, int32_t* __restrict__ hist,
                                                      int32_t* __restrict__ tot) {
  const int d = blockIdx.x * blockDim.x + threadIdx.x;
  if (d >= DIG) return;
  int run = 0;
  for (int t = 0; t < nb; ++t) {
    const int v = hist[(size_t)t * DIG + d];
    hist[(size_t)t * DIG + d] = run;
    run += v;
  }
  tot[d] = run;
}

// Medium inputs: gsum[group][digit] = sum of the group's rows of hist[tile][digit]; one thread per digit, the
// group's rows in two batches of loads.
__global__ __launch_bounds__(256) void k_sort_groupsum(int nb, int DIG, const int32_t* __restrict__ hist,
                                                       int32_t* __restrict__ gsum) {
  const int d = blockIdx.x * blockDim.x + threadIdx.x, grp = blockIdx.y;
  if (d >= DIG) return;
  const int t0 = grp * kGroupTiles;
  int run = 0;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    int v[kGroupTiles / 2];
#pragma unroll
    for (int u = 0; u < kGroupTiles / 2; ++u) {
      const int t = t0 + h * (kGroupTiles / 2) + u;
      v[u] = t < nb ? hist[(size_t)t * DIG + d] : 0;
    }
#pragma unroll
    for (int u = 0; u < kGroupTiles / 2; ++u) run += v[u];
  }
  gsum[(size_t)grp * DIG + d] = run;
}

// Adds rows [r0, r1) of a table of 2^dbits-int rows to at[] (if to_total) and, for the rows below `limit`, to
// am[]. The table is read as 16-byte pieces, consecutive threads next to each other, sixteen loads in flight per
// thread; the four digits a thread sees do not change from load to load (two sets when a row has more pieces
// than the workgroup has threads).
__device__ inline void sort_add_rows(const int32_t* __restrict__ table, int r0, int r1, int dbits, int limit,
                                     bool to_total, int (&at)[2][4], int (&am)[2][4]) {
  const int vshift = dbits - 2;  // log2 of the 16-byte pieces per row
  const int first = r0 << vshift, last = r1 << vshift;
  const int4* h4 = reinterpret_cast<const int4*>(table);
  for (int q0 = first + (int)threadIdx.x; q0 < last; q0 += 16 * kSortThreads) {
    int4 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int q = q0 + u * kSortThreads;
      v[u] = q < last ? h4[q] : make_int4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int q = q0 + u * kSortThreads;
      const bool before = (q >> vshift) < limit;
      const int e[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (to_total) at[u & 1][i] += e[i];
        if (before) am[u & 1][i] += e[i];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// k_sort_pass: one stable scatter pass, one workgroup per tile of 2048 elements. The workgroup first turns
// the histogram into its own start offset for every digit (summing the columns over the tiles before it
// unless k_sort_colscan did so), then every wavefront ranks its 512 consecutive elements 64 at a time in
// index order (ballot matching), so the order of equal keys is kept.
//   FIRST: elements are the cells themselves (value = index), dropped cells (key < 0) stay behind, so the
//          output is compact. Also makes the root ranks global, and writes out_ids, the per-video offsets
//          and the totals (K, list length).
//   LAST:  writes the sorted element list, the output row of every list position and the first list
//          position of every row (the root is the smallest index of its cluster, hence first in its list).
// ------------------------------------------------------------------------------------------------
struct SortArgs {
  int n, shift, dbits, nb, mode;  // mode: how the start offsets are found (see kDirectTiles)
  const int32_t* gsum;
  const int32_t* keys;
  const int32_t* vals;
  int32_t* keys_out;
  int32_t* vals_out;  // LAST: the sorted element list
  const int32_t* hist;
  const int32_t* tot;
  // FIRST
  const int32_t* cluster_ids;
  int32_t* rank;
  const int32_t* tile_roots;
  const int32_t* tile_live;
  int32_t* kdev;  // [0] = K, [1] = list length
  int32_t* out_ids;
  int64_t* offsets;
  int64_t capacity;
  int per_video, B;
  // LAST
  int32_t* orow;
  int32_t* seg;
};

template <bool FIRST, bool LAST>
__global__ __launch_bounds__(kSortThreads) void k_sort_pass(SortArgs a) {
  __shared__ int s_base[kMaxDigits];
  __shared__ int cur[kSortWaves][kMaxDigits];
  const int DIG = 1 << a.dbits, b = blockIdx.x, tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int n = FIRST ? a.n : a.kdev[1];

  // ---- everything this tile reads per element is requested first, so that it arrives while the offsets
  //      are worked out
  const int e0 = b * kSortTile + wave * (kSortTile / kSortWaves);
  int key[kSortPer], val[kSortPer], aux[kSortPer];
  int rk0[kSortPer], cid[kSortPer];
  bool ok[kSortPer];
#pragma unroll
  for (int r = 0; r < kSortPer; ++r) {
    const int i = e0 + r * 64 + lane;
    key[r] = -1;
    val[r] = rk0[r] = cid[r] = 0;
    if (i < n) {
      key[r] = a.keys[i];
      val[r] = FIRST ? i : a.vals[i];
      if (FIRST) {
        rk0[r] = a.rank[i];
        cid[r] = a.cluster_ids[i];
      }
    }
    ok[r] = key[r] >= 0;
  }
  int roots_before = 0, roots_all = 0, live_all = 0;
  if (FIRST) {
    for (int t = tid; t < a.nb; t += kSortThreads) {
      const int v = a.tile_roots[t];
      roots_all += v;
      if (t < b) roots_before += v;
      if (b == 0) live_all += a.tile_live[t];
    }
  }

  // ---- start offset of every digit for this tile
  int* tot = cur[0];   // column totals and the part of them that lies in the tiles before this one
  int* mine = cur[1];  // (the cursors are not in use yet)
  if (a.mode != 2) {
    for (int d = tid; d < DIG; d += kSortThreads) tot[d] = mine[d] = 0;
    __syncthreads();
    int at[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}}, am[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
    if (a.mode == 0) {
      sort_add_rows(a.hist, 0, a.nb, a.dbits, b, true, at, am);
    } else {  // the sums of all groups, then the rows of this tile's own group up to the tile
      const int grp = b / kGroupTiles, ngrp = (a.nb + kGroupTiles - 1) / kGroupTiles;
      sort_add_rows(a.gsum, 0, ngrp, a.dbits, grp, true, at, am);
      sort_add_rows(a.hist, grp * kGroupTiles, min(a.nb, (grp + 1) * kGroupTiles), a.dbits, b, false, at, am);
    }
    const int VC = 1 << (a.dbits - 2);
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int vc = (tid + k * kSortThreads) & (VC - 1);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (at[k][i]) atomicAdd(&tot[vc * 4 + i], at[k][i]);
        if (am[k][i]) atomicAdd(&mine[vc * 4 + i], am[k][i]);
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < kSortPer; ++r) {
    aux[r] = 0;
    if (LAST && ok[r]) aux[r] = a.rank[key[r]];  // output row of the element's cluster (arrives during the scan)
  }
  {
    constexpr int kDpt = kMaxDigits / kSortThreads;
    const int dpt = DIG >= kSortThreads ? DIG / kSortThreads : 1;
    int tv[kDpt], cv[kDpt], s = 0;
#pragma unroll
    for (int j = 0; j < kDpt; ++j) {
      const int d = tid * dpt + j;
      tv[j] = cv[j] = 0;
      if (j < dpt && d < DIG) {
        tv[j] = a.mode == 2 ? a.tot[d] : tot[d];
        cv[j] = a.mode == 2 ? a.hist[(size_t)b * DIG + d] : mine[d];
      }
      s += tv[j];
    }
    int total;
    int ex = block_exclusive_scan(s, &total);  // (its barriers also fence the reads above from the clearing below)
#pragma unroll
    for (int j = 0; j < kDpt; ++j) {
      const int d = tid * dpt + j;
      if (j < dpt && d < DIG) s_base[d] = ex + cv[j];
      ex += tv[j];
    }
  }
  int root_prefix = 0;
  if (FIRST) {
    root_prefix = block_sum(roots_before);
    if (b == 0) {
      const int all = block_sum(roots_all), live = block_sum(live_all);
      if (tid == 0) {
        a.kdev[0] = all;
        a.kdev[1] = live;
        a.offsets[a.B] = all;
        if (LAST) a.seg[all] = live;
      }
    }
  }
  if (LAST && !FIRST && b == 0 && tid == 0) a.seg[a.kdev[0]] = n;
  for (int d = tid; d < DIG; d += kSortThreads)
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) cur[w][d] = 0;
  __syncthreads();

  // ---- per-wavefront digit counts of its 512 elements
#pragma unroll
  for (int r = 0; r < kSortPer; ++r)
    if (ok[r]) atomicAdd(&cur[wave][(key[r] >> a.shift) & (DIG - 1)], 1);
  if (FIRST) {
    // bookkeeping outputs of the cells themselves
#pragma unroll
    for (int r = 0; r < kSortPer; ++r) {
      const int i = e0 + r * 64 + lane;
      if (i >= n) continue;
      const int rk = rk0[r] + root_prefix;
      if (b != 0) a.rank[i] = rk;
      if (cid[r] == i && a.out_ids && rk < a.capacity) a.out_ids[rk] = i;
      if (i % a.per_video == 0) a.offsets[i / a.per_video] = rk;
    }
  }
  __syncthreads();
  for (int d = tid; d < DIG; d += kSortThreads) {
    int run = s_base[d];
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) {
      const int c = cur[w][d];
      cur[w][d] = run;
      run += c;
    }
  }
  __syncthreads();

  // ---- ranked scatter, 64 elements at a time in index order: first which lanes hold the same digit (no
  //      memory involved), then the cursors
  const unsigned long long below = (1ull << lane) - 1ull;
  int* mycur = cur[wave];
  unsigned long long same[kSortPer];
#pragma unroll
  for (int r = 0; r < kSortPer; ++r) {
    const int digit = (key[r] >> a.shift) & (DIG - 1);
    same[r] = __ballot(ok[r]);
    for (int bit = 0; bit < a.dbits; ++bit) {
      const unsigned long long m = __ballot((digit >> bit) & 1);
      same[r] &= ((digit >> bit) & 1) ? m : ~m;
    }
  }
#pragma unroll
  for (int r = 0; r < kSortPer; ++r) {  // the stores of one round travel while the next round's cursors are read
    const int digit = (key[r] >> a.shift) & (DIG - 1);
    if (ok[r]) {
      const int dst = mycur[digit] + __popcll(same[r] & below);
      if (LAST) {
        a.vals_out[dst] = val[r];
        a.orow[dst] = aux[r];
        if (key[r] == val[r]) a.seg[aux[r]] = dst;
      } else {
        a.keys_out[dst] = key[r];
        a.vals_out[dst] = val[r];
      }
    }
    wave_lds_fence();
    if (ok[r] && ((same[r] >> lane) >> 1) == 0)  // highest lane of its digit group advances the cursor
      mycur[digit] += __popcll(same[r]);
    wave_lds_fence();
  }
}

// ------------------------------------------------------------------------------------------------
// The gather/average pass. Every list slot is one 16-byte load per lane: a cell's row (VEC channels of the
// input type), or four fp32 channels of a stored node sum -- with bf16 input a lane owns eight channels, so
// such a node takes two slots (its top-left cell and the next cell of the node stand for the two halves).
// The list is cut into items of kItem consecutive slots; an item owns the clusters whose list starts
// inside it. One wavefront per (item, chunk of the row). All index look-ups of the item are done
// lane-parallel first, then all loads are issued, then the slots are added up in list order (fp32) with the
// cluster boundaries handled as wave-uniform control flow. A cluster with more than kBig slots is not
// followed past the item: every item adds up the slots of such a cluster that lie inside it and leaves the
// partial sum in the workspace (at most two per item: the cluster running in from the left and the one
// starting inside), the item in which the cluster starts puts it on a list, and k_reduce_big_combine adds
// the partial sums up in item order -- so the summation order does not depend on scheduling.
// ------------------------------------------------------------------------------------------------

// Where a list slot's data lives.
struct Slot {
  int kind;    // 0 = cell row, 1 / 2 = first / second four channels of a lane's share of a node sum
  int idx;     // flat cell index, or row of the node-sum table
  int weight;  // member cells it stands for
};

template <int DT>
__device__ inline Slot describe(const Geo& g, const int32_t* __restrict__ node_map,
                                const uint8_t* __restrict__ lvl, int cell) {
  Slot e;
  e.kind = 0;
  e.idx = cell;
  e.weight = 1;
  if (lvl) {
    const int lv = lvl[cell];
    if (lv >= 3) {
      const int rep = node_map[cell];
      const int f = rep / g.HW, c = rep - f * g.HW;
      if (node_is_summed(g, c, lv)) {
        const int y = c / g.W, x = c - y * g.W;
        e.idx = f * (g.NN - g.lvl_base[3]) + node_index(g, lv, y >> lv, x >> lv) - g.lvl_base[3];
        e.kind = cell == rep ? 1 : 2;
        e.weight = cell == rep ? node_cells(g, c, lv) : 0;
      }
    }
  }
  return e;
}

template <int DT>
__device__ inline typename Row<DT>::Raw load_slot(const void* feats, const float* nsum, int D, int ch0, int kind,
                                                  int idx) {
  typedef Row<DT> R;
  if (kind == 0)  // a feature row: this is its last use
    return load_once(reinterpret_cast<const typename R::Raw*>(reinterpret_cast<const typename R::Elem*>(feats) +
                                                              (size_t)idx * D + ch0));
  return *reinterpret_cast<const typename R::Raw*>(nsum + (size_t)idx * D + ch0 + (kind - 1) * 4);
}

template <int DT>
__device__ inline void acc_slot(const float4& r, int, float (&acc)[4]) {  // fp32 rows and node sums share a layout
  acc[0] += r.x; acc[1] += r.y; acc[2] += r.z; acc[3] += r.w;
}
template <int DT>
__device__ inline void acc_slot(const uint4& r, int kind, float (&acc)[8]) {
  if (kind == 0) {
    Row<DT>::add_row(r, acc);
  } else {
    const float f0 = __uint_as_float(r.x), f1 = __uint_as_float(r.y);
    const float f2 = __uint_as_float(r.z), f3 = __uint_as_float(r.w);
    if (kind == 1) {
      acc[0] += f0; acc[1] += f1; acc[2] += f2; acc[3] += f3;
    } else {
      acc[4] += f0; acc[5] += f1; acc[6] += f2; acc[7] += f3;
    }
  }
}

template <int DT, int ODT>
__device__ inline void store_mean(void* merged_v, size_t elem_off, const float (&acc)[Row<DT>::VEC], float inv) {
  constexpr int VEC = Row<DT>::VEC;
  if (ODT == 0) {
    float* o = reinterpret_cast<float*>(merged_v) + elem_off;
#pragma unroll
    for (int v = 0; v < VEC; v += 4)
      store_once(reinterpret_cast<float4*>(o + v),
                 make_float4(acc[v] * inv, acc[v + 1] * inv, acc[v + 2] * inv, acc[v + 3] * inv));
  } else {
    uint16_t* o = reinterpret_cast<uint16_t*>(merged_v) + elem_off;
    uint32_t w[VEC / 2];
#pragma unroll
    for (int v = 0; v < VEC; v += 2)
      w[v / 2] = ODT == 1 ? pack2_bf16(acc[v] * inv, acc[v + 1] * inv) : pack2_f16(acc[v] * inv, acc[v + 1] * inv);
    if (VEC == 8)
      store_once(reinterpret_cast<uint4*>(o), make_uint4(w[0], w[1], w[2 % (VEC / 2)], w[3 % (VEC / 2)]));
    else
      *reinterpret_cast<uint2*>(o) = make_uint2(w[0], w[1]);
  }
}

struct GatherArgs {
  const void* feats;
  const float* nsum;
  const int32_t* node_map;  // the stage-1 partition, or both NULL when every slot is a cell
  const uint8_t* lvl;
  const int32_t* order;
  const int32_t* orow;
  const int32_t* seg;
  const int32_t* kdev;
  int64_t capacity;
  void* merged;
  int32_t* counts;
  float* bigpart;     // [items][2][D] partial sums of big clusters
  int32_t* bigw;      // [items][2] member cells behind them
  int4* biglist;      // one entry per big cluster: output row, first list position, end of its list
  int32_t* bigcount;  // length of that list
  const int32_t* zpos;  // output row of every cluster rank when the rows follow the Z-shaped scan, else NULL
};

// Wavefronts that share an item: one per chunk of the row, at most 16 (beyond that a wavefront takes several chunks).
__host__ __device__ inline int gather_waves(const Geo& g) { return g.nC < 16 ? g.nC : 16; }

template <int VEC>
__device__ inline void store_partial(float* o, const float (&acc)[VEC]) {
#pragma unroll
  for (int v = 0; v < VEC; v += 4) *reinterpret_cast<float4*>(o + v) = make_float4(acc[v], acc[v + 1], acc[v + 2], acc[v + 3]);
}

template <int DT, int ODT>
__global__ __launch_bounds__(64) void k_reduce(Geo g, GatherArgs a) {
  typedef Row<DT> R;
  constexpr int VEC = R::VEC;
  // one-wavefront workgroups; consecutive ones take the chunks of one item
  const int nw = gather_waves(g), wave = blockIdx.x % nw, item = blockIdx.x / nw, lane = threadIdx.x;
  // Lane j < kItem describes list position p0 + j, the next kTail lanes the positions after the item (the start of
  // a cluster that runs past it). The list entries are requested together with the list's length: entries at or
  // beyond the end are stale and are not used.
  const int p0 = item * kItem, pl = p0 + lane;
  int cell_l = 0, rank_l = 0;
  if (lane < kItem + kTail && pl < g.N) {
    cell_l = a.order[pl];
    rank_l = a.orow[pl];  // clusters are listed in ascending id; the output row may differ
  }
  const int M = a.kdev[1];
  const int p1 = min(p0 + kItem, M);
  if (p0 >= M) return;
  Slot sv = {0, 0, 0};
  int row_v = -1, beg_v = 0, end_v = 0;
  if (lane < kItem + kTail && pl < M) {
    sv = describe<DT>(g, a.node_map, a.lvl, cell_l);
    if (lane < kItem) {
      beg_v = a.seg[rank_l];
      end_v = a.seg[rank_l + 1];
      row_v = a.zpos ? a.zpos[rank_l] : rank_l;
    }
  }
  Slot tnext;  // lanes 0..kTail-1: the positions p0 + kItem ... described above
  tnext.kind = __shfl(sv.kind, kItem + (lane & (kTail - 1)), 64);
  tnext.idx = __shfl(sv.idx, kItem + (lane & (kTail - 1)), 64);
  tnext.weight = __shfl(sv.weight, kItem + (lane & (kTail - 1)), 64);
  for (int chunk = wave; chunk < g.nC; chunk += nw) {
    const int ch0 = chunk * g.cch + lane * VEC;
    const bool act = ch0 < g.D;
    // issue every load of the positions this item adds up: clusters starting here, and big ones
    typename R::Raw raw[kItem];
#pragma unroll
    for (int j = 0; j < kItem; ++j) {
      const int beg = __shfl(beg_v, j, 64), end = __shfl(end_v, j, 64);
      const int kind = __shfl(sv.kind, j, 64), idx = __shfl(sv.idx, j, 64);
      raw[j] = R::zero();
      const bool use = p0 + j < p1 && (beg >= p0 || end - beg > kBig);  // wave-uniform
      if (use && act) raw[j] = load_slot<DT>(a.feats, a.nsum, g.D, ch0, kind, idx);
    }
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    int members = 0, open_row = -1, open_end = 0;  // the cluster still open after the item's last position
#pragma unroll
    for (int j = 0; j < kItem; ++j) {
      const int beg = __shfl(beg_v, j, 64), end = __shfl(end_v, j, 64), row = __shfl(row_v, j, 64);
      const int kind = __shfl(sv.kind, j, 64), wgt = __shfl(sv.weight, j, 64);
      const bool big = end - beg > kBig;
      const bool use = p0 + j < p1 && (beg >= p0 || big);
      const int p = p0 + j;
      // a cluster of one cell whose row is written in the type it came in: the mean is the row itself
      const bool one = (DT == ODT) && use && !big && beg == p && end == p + 1 && kind == 0;
      if (one) {
        if (row < a.capacity) {
          if (act) store_once(reinterpret_cast<typename R::Raw*>(
                                  reinterpret_cast<typename R::Elem*>(a.merged) + (size_t)row * g.D + ch0), raw[j]);
          if (chunk == 0 && lane == 0 && a.counts) a.counts[row] = 1;
        }
      } else if (use) {
        acc_slot<DT>(raw[j], kind, acc);
        members += wgt;
        const bool closes = p + 1 == end, last = p + 1 == p1;
        if (big) {
          if (closes || last) {  // this item's share of a big cluster
            const int slot = beg < p0 ? 0 : 1;
            if (act) store_partial<VEC>(a.bigpart + ((size_t)item * 2 + slot) * g.D + ch0, acc);
            if (chunk == 0 && lane == 0) {
              a.bigw[item * 2 + slot] = members;
              if (slot == 1) a.biglist[atomicAdd(a.bigcount, 1)] = make_int4(row, beg, end, 0);
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
            members = 0;
          }
        } else if (closes) {
          if (row < a.capacity) {
            if (act) store_mean<DT, ODT>(a.merged, (size_t)row * g.D + ch0, acc, 1.f / (float)members);
            if (chunk == 0 && lane == 0 && a.counts) a.counts[row] = members;
          }
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
          members = 0;
        } else if (last) {
          open_row = row;
          open_end = end;
        }
      }
    }
    if (open_row >= 0) {
      // the last cluster runs past the item: finish it from the list, kTail loads in flight
      for (int q = p1; q < open_end; q += kTail) {
        Slot ts = {0, 0, 0};
        if (q == p1) ts = tnext;  // (an open cluster means the item is full: p1 == p0 + kItem)
        else if (lane < kTail && q + lane < open_end) ts = describe<DT>(g, a.node_map, a.lvl, a.order[q + lane]);
        typename R::Raw tr[kTail];
#pragma unroll
        for (int u = 0; u < kTail; ++u) {
          const int kd = __shfl(ts.kind, u, 64), ix = __shfl(ts.idx, u, 64);
          tr[u] = R::zero();
          if (q + u < open_end && act) tr[u] = load_slot<DT>(a.feats, a.nsum, g.D, ch0, kd, ix);
        }
#pragma unroll
        for (int u = 0; u < kTail; ++u) {
          const int kd = __shfl(ts.kind, u, 64), wg = __shfl(ts.weight, u, 64);
          if (q + u < open_end) {
            acc_slot<DT>(tr[u], kd, acc);
            members += wg;
          }
        }
      }
      if (open_row < a.capacity) {
        if (act) store_mean<DT, ODT>(a.merged, (size_t)open_row * g.D + ch0, acc, 1.f / (float)members);
        if (chunk == 0 && lane == 0 && a.counts) a.counts[open_row] = members;
      }
    }
  }
}

// A fixed number of workgroups per chunk walks the list of big clusters. A cluster's partial sums are added up
// in item order (the starting item's own, then the left-hand shares of the items after it): the run of items is
// cut into kBigSeg contiguous segments, one wavefront each, eight loads in flight, and the segment sums are
// added in segment order through LDS -- an order that depends on the list alone.
constexpr int kBigGrid = 256;
constexpr int kBigBatch = 8;
constexpr int kBigSeg = 8;

template <int DT, int ODT>
__global__ __launch_bounds__(64 * kBigSeg) void k_reduce_big_combine(Geo g, GatherArgs a) {
  constexpr int VEC = Row<DT>::VEC;
  __shared__ float segsum[kBigSeg - 1][64][VEC];
  __shared__ int segmem[kBigSeg];
  const int seg = threadIdx.x >> 6, lane = threadIdx.x & 63, chunk = blockIdx.y;
  const int ch0 = chunk * g.cch + lane * VEC;
  const bool act = ch0 < g.D;
  const int nbig = *a.bigcount;
  for (int e = blockIdx.x; e < nbig; e += gridDim.x) {  // uniform over the workgroup
    const int4 en = a.biglist[e];
    const int k = en.x, it0 = en.y / kItem, it1 = (en.z - 1) / kItem;
    // the partial sums of the cluster: number 0 is the starting item's (slot 1), number j > 0 item it0 + j's (slot 0)
    const int np = it1 - it0 + 1, per = (np + kBigSeg - 1) / kBigSeg;
    const int j0 = min(np, seg * per), j1 = min(np, j0 + per);
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    int members = 0;
    for (int j = j0; j < j1; j += kBigBatch) {
      float4 r[kBigBatch][VEC / 4];
#pragma unroll
      for (int u = 0; u < kBigBatch; ++u) {
        const int jj = min(j + u, j1 - 1);
        const float4* q =
            reinterpret_cast<const float4*>(a.bigpart + ((size_t)(it0 + jj) * 2 + (jj == 0 ? 1 : 0)) * g.D + (act ? ch0 : 0));
#pragma unroll
        for (int v = 0; v < VEC / 4; ++v) r[u][v] = q[v];
      }
#pragma unroll
      for (int u = 0; u < kBigBatch; ++u) {
        if (j + u >= j1) continue;
#pragma unroll
        for (int v = 0; v < VEC / 4; ++v) {
          acc[4 * v] += r[u][v].x; acc[4 * v + 1] += r[u][v].y;
          acc[4 * v + 2] += r[u][v].z; acc[4 * v + 3] += r[u][v].w;
        }
      }
    }
    for (int j = j0 + lane; j < j1; j += 64) members += a.bigw[(it0 + j) * 2 + (j == 0 ? 1 : 0)];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) members += __shfl_xor(members, o, 64);
    if (seg > 0) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) segsum[seg - 1][lane][v] = acc[v];
    }
    if (lane == 0) segmem[seg] = members;
    __syncthreads();
    if (seg == 0 && k < a.capacity) {
      int total = 0;
#pragma unroll
      for (int u = 0; u < kBigSeg; ++u) total += segmem[u];
#pragma unroll
      for (int u = 1; u < kBigSeg; ++u)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] += segsum[u - 1][lane][v];
      if (chunk == 0 && lane == 0 && a.counts) a.counts[k] = total;
      if (act) store_mean<DT, ODT>(a.merged, (size_t)k * g.D + ch0, acc, 1.f / (float)total);
    }
    __syncthreads();
  }
}

size_t reduce_items(const Geo& g) { return (size_t)(g.N + kItem - 1) / kItem; }
size_t reduce_bigpart_floats(const Geo& g) { return reduce_items(g) * 2 * g.D; }
size_t reduce_bigw_entries(const Geo& g) { return reduce_items(g) * 2; }
size_t reduce_biglist_entries(const Geo& g) { return (size_t)g.N / (kBig + 1) + 1; }  // a big cluster has > kBig slots

// ------------------------------------------------------------------------------------------------
// Z-shaped scan (Sec. 3.4): inside a frame the rows follow the Morton rank of the root's top-left cell
// instead of its raster index. The clusters stay listed by ascending id (rank); this kernel, one workgroup per
// frame, gives every rank of the frame its output row: the frame's rows are the same range either way, only
// permuted. Needs the global ranks (after the first sort pass). Also writes out_ids in the new order.
// ------------------------------------------------------------------------------------------------
__device__ inline int morton_rank(int y, int x) {
  int z = 0;
#pragma unroll
  for (int b = 0; b < kMaxLevels; ++b) z |= (((x >> b) & 1) << (2 * b)) | (((y >> b) & 1) << (2 * b + 1));
  return z;
}

__global__ __launch_bounds__(256) void k_zorder(Geo g, const int32_t* __restrict__ cluster_ids,
                                                const int32_t* __restrict__ rank, int64_t capacity,
                                                int32_t* __restrict__ zpos, int32_t* __restrict__ out_ids) {
  __shared__ int flag[1024];  // root cells of the frame at their Morton slot, then their exclusive count
  const int f = blockIdx.x, tid = threadIdx.x, PP = g.P * g.P;
  for (int z = tid; z < 1024; z += 256) flag[z] = 0;
  __syncthreads();
  for (int c = tid; c < g.HW; c += 256) {
    const int i = f * g.HW + c;
    if (cluster_ids[i] == i) flag[morton_rank(c / g.W, c % g.W)] = 1;
  }
  __syncthreads();
  // exclusive scan over the (up to 1024) Morton slots: four consecutive slots per thread
  int v[4], sum = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    v[j] = tid * 4 + j < PP ? flag[tid * 4 + j] : 0;
    sum += v[j];
  }
  int total;
  int ex = block_exclusive_scan(sum, &total);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (tid * 4 + j < PP) flag[tid * 4 + j] = ex;
    ex += v[j];
  }
  __syncthreads();
  const int r0 = rank[f * g.HW];  // roots before this frame
  for (int c = tid; c < g.HW; c += 256) {
    const int i = f * g.HW + c;
    if (cluster_ids[i] != i) continue;
    const int row = r0 + flag[morton_rank(c / g.W, c % g.W)];
    zpos[rank[i]] = row;
    if (out_ids && row < capacity) out_ids[row] = i;
  }
}

// ------------------------------------------------------------------------------------------------
// Position indices of the output rows (Sec. 3.4). k_positions_cells adds every cell's original index (within
// its video) to its row's integer sum; k_positions_rows turns the sums into means and writes the root's
// own index, the row's index in its video's output, and the root's (t, y0, x0, level).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_positions_clear(int n, unsigned long long* __restrict__ possum,
                                                         unsigned* __restrict__ poscnt) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    possum[i] = 0ull;
    poscnt[i] = 0u;
  }
}

// With the stage-1 partition at hand a whole node is added at once, by its top-left cell: the sum of the indices
// of its valid cells has a closed form, and a cluster made of a few large nodes costs a few atomics instead of
// hundreds on one address.
__global__ __launch_bounds__(256) void k_positions_cells(Geo g, const int32_t* __restrict__ cluster_ids,
                                                         const int32_t* __restrict__ node_map,
                                                         const uint8_t* __restrict__ node_level,
                                                         const int32_t* __restrict__ rank,
                                                         unsigned long long* __restrict__ possum,
                                                         unsigned* __restrict__ poscnt) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= g.N) return;
  const int loc = i % (g.T * g.HW);
  unsigned long long sum = (unsigned long long)loc;
  unsigned cnt = 1u;
  if (node_map) {
    if (node_map[i] != i) return;
    const int c = loc % g.HW, y0 = c / g.W, x0 = c - y0 * g.W, s = 1 << node_level[i];
    const int ny = min(y0 + s, g.H) - y0, nx = min(x0 + s, g.W) - x0;
    // sum over y0 <= y < y0+ny, x0 <= x < x0+nx of (loc + (y - y0) * W + (x - x0))
    cnt = (unsigned)(ny * nx);
    sum = (unsigned long long)cnt * loc + (unsigned long long)nx * g.W * (ny * (ny - 1) / 2) +
          (unsigned long long)ny * (nx * (nx - 1) / 2);
  }
  const int r = rank[cluster_ids[i]];
  atomicAdd(&possum[r], sum);
  atomicAdd(&poscnt[r], cnt);
}

__global__ __launch_bounds__(256) void k_positions_rows(Geo g, const int32_t* __restrict__ kdev,
                                                        const int32_t* __restrict__ order,
                                                        const int32_t* __restrict__ seg,
                                                        const int32_t* __restrict__ zpos,
                                                        const uint8_t* __restrict__ node_level,
                                                        const int64_t* __restrict__ offsets,
                                                        const unsigned long long* __restrict__ possum,
                                                        const unsigned* __restrict__ poscnt, int64_t capacity,
                                                        int32_t* __restrict__ survived,
                                                        int32_t* __restrict__ reassigned,
                                                        float* __restrict__ merged_pos,
                                                        int32_t* __restrict__ root_tyxl) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;  // cluster rank (ascending id)
  if (r >= kdev[0]) return;
  const int root = order[seg[r]];  // the root is the first element of its cluster's list
  const int row = zpos ? zpos[r] : r;
  if (row >= capacity) return;
  const int per_video = g.T * g.HW, b = root / per_video, loc = root - b * per_video;
  if (survived) survived[row] = loc;
  if (reassigned) reassigned[row] = row - (int)offsets[b];
  if (merged_pos) merged_pos[row] = (float)((double)possum[r] / (double)poscnt[r]);
  if (root_tyxl) {
    const int t = loc / g.HW, c = loc - t * g.HW;
    root_tyxl[4 * row + 0] = t;
    root_tyxl[4 * row + 1] = c / g.W;
    root_tyxl[4 * row + 2] = c % g.W;
    root_tyxl[4 * row + 3] = node_level ? (int)node_level[root] : -1;
  }
}

void launch_positions(const Geo& g, const int32_t* cluster_ids, const int32_t* node_map, const uint8_t* node_level,
                      const int64_t* offsets,
                      int64_t capacity, const ReduceBuffers& rb, bool zscan, unsigned long long* possum,
                      unsigned* poscnt, int32_t* survived, int32_t* reassigned, float* merged_pos,
                      int32_t* root_tyxl, hipStream_t s) {
  const dim3 grid((g.N + 255) / 256), block(256);
  if (merged_pos) {
    hipLaunchKernelGGL(k_positions_clear, grid, block, 0, s, g.N, possum, poscnt);
    hipLaunchKernelGGL(k_positions_cells, grid, block, 0, s, g, cluster_ids, node_level ? node_map : nullptr,
                       node_level, rb.rank, possum, poscnt);
  }
  hipLaunchKernelGGL(k_positions_rows, grid, block, 0, s, g, rb.kdev, rb.order, rb.seg, zscan ? rb.zpos : nullptr,
                     node_level, offsets, possum, poscnt, capacity, survived, reassigned, merged_pos, root_tyxl);
}

// Integer plumbing of the reduce stage: sorted element list, row of every list position, row starts.
void launch_reduce_prepare(const Geo& g, const int32_t* cluster_ids, const int32_t* node_map,
                           const uint8_t* node_level, int64_t capacity, int32_t* out_ids, int64_t* offsets,
                           const ReduceBuffers& rb, bool zscan, hipStream_t s) {
  const int N = g.N;
  const SortPlan pl = sort_plan(N);
  const int DIG = 1 << pl.dbits;
  const dim3 grid(pl.nb), block(kSortThreads);
  hipLaunchKernelGGL(k_reduce_prep, grid, block, 0, s, g, cluster_ids, node_map, node_level, pl.dbits, rb.key_a,
                     rb.rank, rb.tile_roots, rb.tile_live, rb.hist, rb.kdev + 2);
  const int32_t* kin = rb.key_a;
  const int32_t* vin = nullptr;
  int32_t* kout = rb.key_b;
  int32_t* vout = rb.val_b;
  for (int pass = 0; pass < pl.passes; ++pass) {
    const bool first = pass == 0, last = pass == pl.passes - 1;
    if (!first)
      hipLaunchKernelGGL(k_sort_hist, grid, block, 0, s, rb.kdev, pass * pl.dbits, pl.dbits, kin, rb.hist);
    if (pl.mode == 2)
      hipLaunchKernelGGL(k_sort_colscan, dim3((DIG + 255) / 256), dim3(256), 0, s, pl.nb, DIG, rb.hist, rb.tot);
    else if (pl.mode == 1)
      hipLaunchKernelGGL(k_sort_groupsum, dim3((DIG + 255) / 256, (pl.nb + kGroupTiles - 1) / kGroupTiles), dim3(256), 0,
                         s, pl.nb, DIG, rb.hist, rb.gsum);
    SortArgs a;
    a.n = N; a.shift = pass * pl.dbits; a.dbits = pl.dbits; a.nb = pl.nb; a.mode = pl.mode; a.gsum = rb.gsum;
    a.keys = kin; a.vals = vin; a.keys_out = kout; a.vals_out = last ? rb.order : vout;
    a.hist = rb.hist; a.tot = rb.tot;
    a.cluster_ids = cluster_ids; a.rank = rb.rank; a.tile_roots = rb.tile_roots; a.tile_live = rb.tile_live;
    a.kdev = rb.kdev; a.out_ids = zscan ? nullptr : out_ids; a.offsets = offsets; a.capacity = capacity;
    a.per_video = g.T * g.HW; a.B = g.B;
    a.orow = rb.orow; a.seg = rb.seg;
    if (first && last) hipLaunchKernelGGL((k_sort_pass<true, true>), grid, block, 0, s, a);
    else if (first) hipLaunchKernelGGL((k_sort_pass<true, false>), grid, block, 0, s, a);
    else if (last) hipLaunchKernelGGL((k_sort_pass<false, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((k_sort_pass<false, false>), grid, block, 0, s, a);
    kin = kout;
    vin = vout;
    if (kout == rb.key_b) { kout = rb.key_a; vout = rb.val_a; } else { kout = rb.key_b; vout = rb.val_b; }
  }
  if (zscan)
    hipLaunchKernelGGL(k_zorder, dim3(g.F), dim3(256), 0, s, g, cluster_ids, rb.rank, capacity, rb.zpos, out_ids);
}

static GatherArgs gather_args(const void* feats, const float* nsum, const int32_t* node_map,
                              const uint8_t* node_level, int64_t capacity, void* merged, int32_t* counts,
                              const ReduceBuffers& rb, bool zscan) {
  GatherArgs a;
  a.feats = feats; a.nsum = nsum; a.node_map = node_map; a.lvl = node_level; a.order = rb.order; a.orow = rb.orow;
  a.seg = rb.seg; a.kdev = rb.kdev; a.capacity = capacity; a.merged = merged; a.counts = counts;
  a.bigpart = rb.bigpart; a.bigw = rb.bigw;
  a.biglist = reinterpret_cast<int4*>(rb.biglist); a.bigcount = rb.kdev + 2;
  a.zpos = zscan ? rb.zpos : nullptr;
  return a;
}

// Input / output element types a gather kernel is built for: fp32 in with any output type; a 16-bit input with
// the same type or fp32 out (reduce_io_supported() says which pairs exist).
#define STTM_DISPATCH_IO(KERNEL, IN, OUT, GRID, BLOCK, STREAM, ...)                                      \
  do {                                                                                                   \
    const int io_ = (IN) * 3 + (OUT);                                                                    \
    if (io_ == 0) hipLaunchKernelGGL((KERNEL<0, 0>), GRID, BLOCK, 0, STREAM, __VA_ARGS__);               \
    else if (io_ == 1) hipLaunchKernelGGL((KERNEL<0, 1>), GRID, BLOCK, 0, STREAM, __VA_ARGS__);          \
    else if (io_ == 2) hipLaunchKernelGGL((KERNEL<0, 2>), GRID, BLOCK, 0, STREAM, __VA_ARGS__);          \
    else if (io_ == 3) hipLaunchKernelGGL((KERNEL<1, 0>), GRID, BLOCK, 0, STREAM, __VA_ARGS__);          \
    else if (io_ == 4) hipLaunchKernelGGL((KERNEL<1, 1>), GRID, BLOCK, 0, STREAM, __VA_ARGS__);          \
    else if (io_ == 6) hipLaunchKernelGGL((KERNEL<2, 0>), GRID, BLOCK, 0, STREAM, __VA_ARGS__);          \
    else if (io_ == 8) hipLaunchKernelGGL((KERNEL<2, 2>), GRID, BLOCK, 0, STREAM, __VA_ARGS__);          \
  } while (0)

bool reduce_io_supported(int in_dtype, int out_dtype) {
  if (in_dtype < 0 || in_dtype > 2 || out_dtype < 0 || out_dtype > 2) return false;
  return in_dtype == 0 || out_dtype == 0 || out_dtype == in_dtype;
}

// The feature pass of the reduce stage: the gather over the whole list (clusters of up to kBig slots) ...
void launch_reduce_gather(const Geo& g, const void* feats, const float* nsum, const int32_t* node_map,
                          const uint8_t* node_level, int out_dtype, int64_t capacity, void* merged, int32_t* counts,
                          const ReduceBuffers& rb, bool zscan, hipStream_t s) {
  const int nitems = (g.N + kItem - 1) / kItem;
  dim3 grid((unsigned)(nitems * gather_waves(g))), block(64);  // <= N + 15 workgroups
  const GatherArgs a = gather_args(feats, nsum, node_map, node_level, capacity, merged, counts, rb, zscan);
  STTM_DISPATCH_IO(k_reduce, g.dtype, out_dtype, grid, block, s, g, a);
}

// ... and the means of the clusters with more than kBig slots from the partial sums the gather left behind.
void launch_reduce_big(const Geo& g, const void* feats, const float* nsum, const int32_t* node_map,
                       const uint8_t* node_level, int out_dtype, int64_t capacity, void* merged, int32_t* counts,
                       const ReduceBuffers& rb, bool zscan, hipStream_t s) {
  const int nmax = (int)reduce_biglist_entries(g);
  dim3 grid(nmax < kBigGrid ? nmax : kBigGrid, g.nC), block(64 * kBigSeg);
  const GatherArgs a = gather_args(feats, nsum, node_map, node_level, capacity, merged, counts, rb, zscan);
  STTM_DISPATCH_IO(k_reduce_big_combine, g.dtype, out_dtype, grid, block, s, g, a);
}

}  // namespace sttm
