// Temporal stage (Sec. 3.3): similarities between every kept node of frame t and the kept nodes of
// frame t-1 it overlaps, directed edges with top-left priority, and the common root of every chain.
#include "sttm_dev.h"

namespace sttm {

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
// k_temporal_dots: grid (chunk, frame pair); the one pass over the features of the temporal stage.
// The two frames' partitions are both quadtree cuts, so any two overlapping nodes are nested; a pair is
// named by the top-left cell q of its finer node, and its "join" block is the coarser node. Work is
// listed per workgroup by join level J:
//  * J <= 1 ("fast"): aligned 2x2 regions in which both frames' nodes are single cells or the 2x2 block.
//    A wavefront loads the 4+4 cells of two regions at once (16 rows in flight) and emits up to four dot
//    products per region. With `skip_cells` the regions of single cells in both frames are left out: the spatial
//    pass has already formed those dot products (k_temporal_resolve reads them from its table).
//  * J == 2 ("mid"): a wavefront sums the 4x4 block in the frame where it is one node, then dots every cell
//    of the other frame's block with that sum; a finer node's dot product is the sum over its cells.
//  * J >= 3 ("big"): the coarse sum is not recomputed: the spatial pass left the per-channel sums of all
//    nodes at levels >= 3 in `nsum`; the workgroup stages the rows it needs in LDS. Pairs whose finer
//    node is a single cell are handled sixteen at a time (their list entries carry the cell, the join level and
//    the frame the cell belongs to), the others one by one (finer nodes at levels >= 3 also come from `nsum`).
// Per-lane partial dot products are reduced across the wavefront through LDS ([scalar][lane] rows).
// Frame pairs are visited last-to-first: the spatial pass before it reads frames first-to-last, so the
// tail of the video may still sit in the memory-side cache.
// Output: pd_part[f][chunk][q].
// ------------------------------------------------------------------------------------------------
constexpr int kFastRows = 16;

template <int DT>
__global__ __launch_bounds__(256) void k_temporal_dots(Geo g, const void* __restrict__ feats_v,
                                                       const uint8_t* __restrict__ node_level,
                                                       const float* __restrict__ nsum,
                                                       int skip_cells, float* __restrict__ pd_part,
                                                       SelState* __restrict__ sel) {
  typedef Row<DT> R;
  constexpr int VEC = R::VEC;
  STTM_DYNAMIC_LDS(float, bigS);  // [big join blocks][cch]
  __shared__ int8_t slot_of[24];  // node at a level >= 3 (counted from the first level-3 node) -> its row of bigS
  __shared__ uint8_t lvl_t[1024], lvl_p[1024];
  __shared__ int16_t fast[256], mid[64], bighead[16], pairs0[1024], pairsX[512];
  __shared__ int nfast, nmid, nbig, n0, nX;
  __shared__ float tbuf[4][kFastRows * 68];
  // Workgroups are handed to the eight accelerator dies (each with an L2 of its own) round-robin by their
  // linear index. A frame is read by two pairs: the mapping gives every die a contiguous range of pairs and
  // walks it pair by pair, all chunks of a pair together, so the two readers of a frame run on the same die
  // at about the same time and the second one finds the rows in that L2.
  const int npairs = g.B * (g.T - 1), per_die = (npairs + 7) / 8;
  const int die = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int chunk = slot % g.nC, pl = slot / g.nC;
  if (pl >= per_die || die * per_die + pl >= npairs) return;
  const int pair = npairs - 1 - (die * per_die + pl);  // frame pairs of all videos: (b, t) with t >= 1
  const int b = pair / (g.T - 1), t = pair - b * (g.T - 1) + 1;
  const int f = b * g.T + t;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int H = g.H, W = g.W, HW = g.HW;
  const int NB = g.NN - g.lvl_base[3];
  if (chunk == 0 && t == 1) sel_clear(sel + b);  // the temporal budget search of this video starts afresh
  if (threadIdx.x == 0) { nfast = nmid = nbig = n0 = nX = 0; }
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    lvl_t[c] = node_level[(size_t)f * HW + c];
    lvl_p[c] = node_level[(size_t)(f - 1) * HW + c];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    const int a = lvl_t[c], bb = lvl_p[c];
    const int J = max(a, bb), lf = min(a, bb);
    const int y = c / W, x = c - y * W;
    const bool join_head = !(y & ((1 << J) - 1)) && !(x & ((1 << J) - 1));
    if (J <= 1) {
      // (a region of single cells in both frames has nothing to do when the spatial pass left those dot products)
      if (!(y & 1) && !(x & 1) && (J == 1 || !skip_cells)) fast[atomicAdd(&nfast, 1)] = (int16_t)c;
    } else if (J == 2) {
      if (join_head) mid[atomicAdd(&nmid, 1)] = (int16_t)c;
    } else {
      if (join_head) bighead[atomicAdd(&nbig, 1)] = (int16_t)c;
      if (!(y & ((1 << lf) - 1)) && !(x & ((1 << lf) - 1))) {  // top-left cell of the finer node
        // packed: x (5 bits), y (5), join level (3), whether the cell is frame t's (1)
        if (lf == 0) pairs0[atomicAdd(&n0, 1)] = (int16_t)(x | (y << 5) | (J << 10) | ((a < bb ? 1 : 0) << 13));
        else pairsX[atomicAdd(&nX, 1)] = (int16_t)c;
      }
    }
  }
  __syncthreads();
  const int ch0 = chunk * g.cch + lane * VEC;
  const bool act = ch0 < g.D;
  const typename R::Elem* ft =
      reinterpret_cast<const typename R::Elem*>(feats_v) + (size_t)f * HW * g.D + (act ? ch0 : 0);
  const typename R::Elem* fp = ft - (size_t)HW * g.D;
  float* out = pd_part + (size_t)(f * g.nC + chunk) * HW;
  float* tb = tbuf[wave];

  // ---- stage the coarse sums of the big join blocks
  const int nb = min(nbig, 16);
  for (int s = 0; s < nb; ++s) {
    const int c = bighead[s];
    const int a = lvl_t[c], bb = lvl_p[c];
    const int J = max(a, bb), y = c / W, x = c - y * W;
    const int fc = a >= bb ? f : f - 1;  // frame in which the join block is one node
    const int nid = node_index(g, J, y >> J, x >> J) - g.lvl_base[3];
    const float* row = nsum + ((size_t)fc * NB + nid) * g.D;
    if (threadIdx.x == 0) slot_of[nid] = (int8_t)s;  // where the pairs under this block find its sum
    for (int cc = threadIdx.x; cc < g.cch; cc += blockDim.x) {
      const int ch = chunk * g.cch + cc;
      bigS[s * g.cch + cc] = ch < g.D ? row[ch] : 0.f;
    }
  }
  if (nb) __syncthreads();

  // ---- fast regions: four per batch and wavefront, two at a time
  const int nf = min(nfast, 256);
  for (int base = wave * 4; base < nf; base += 16) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      typename R::Raw rt[2][4], rp[2][4];
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) {
        const int ri = base + half * 2 + rr;
        const int c0 = ri < nf ? fast[ri] : -1;
        const int y0 = c0 / W, x0 = c0 - y0 * W;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int y = y0 + (k >> 1), x = x0 + (k & 1);
          rt[rr][k] = R::zero();
          rp[rr][k] = R::zero();
          if (c0 >= 0 && y < H && x < W && act) {
            rt[rr][k] = *reinterpret_cast<const typename R::Raw*>(ft + (size_t)(y * W + x) * g.D);
            rp[rr][k] = *reinterpret_cast<const typename R::Raw*>(fp + (size_t)(y * W + x) * g.D);
          }
        }
      }
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) {
        const int ri = base + half * 2 + rr;
        const int c0 = ri < nf ? fast[ri] : 0;
        const bool t_block = lvl_t[c0] == 1, p_block = lvl_p[c0] == 1;  // wave-uniform
        if (!t_block && !p_block) {  // four cells against four cells: no sums needed
#pragma unroll
          for (int k = 0; k < 4; ++k) tb[((half * 2 + rr) * 4 + k) * 68 + lane] = R::dot(rt[rr][k], rp[rr][k]);
          continue;
        }
        float xt[4][VEC], xp[4][VEC];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          R::unpack(rt[rr][k], xt[k]);
          R::unpack(rp[rr][k], xp[k]);
        }
        if (t_block) {
#pragma unroll
          for (int v = 0; v < VEC; ++v) {
            const float sum = (xt[0][v] + xt[1][v]) + (xt[2][v] + xt[3][v]);
            xt[0][v] = xt[1][v] = xt[2][v] = xt[3][v] = sum;
          }
        }
        if (p_block) {
#pragma unroll
          for (int v = 0; v < VEC; ++v) {
            const float sum = (xp[0][v] + xp[1][v]) + (xp[2][v] + xp[3][v]);
            xp[0][v] = xp[1][v] = xp[2][v] = xp[3][v] = sum;
          }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          float d = 0.f;
#pragma unroll
          for (int v = 0; v < VEC; ++v) d = fmaf(xt[k][v], xp[k][v], d);
          tb[((half * 2 + rr) * 4 + k) * 68 + lane] = d;
        }
      }
    }
    wave_lds_fence();
    if (lane < kFastRows) {
      const float4* row = reinterpret_cast<const float4*>(tb + lane * 68);
      float acc = 0.f;
#pragma unroll
      for (int jj = 0; jj < 16; ++jj) {
        const float4 q = row[jj];
        acc += (q.x + q.y) + (q.z + q.w);
      }
      const int ri = base + (lane >> 2), k = lane & 3;
      if (ri < nf) {
        const int c0 = fast[ri];
        const int y = c0 / W + (k >> 1), x = c0 % W + (k & 1);
        const bool both_block = lvl_t[c0] == 1 && lvl_p[c0] == 1;
        if (y < H && x < W && (k == 0 || !both_block)) out[y * W + x] = acc;
      }
    }
    wave_lds_fence();
  }

  // ---- big pairs whose finer node is one cell: sixteen per batch and wavefront, in stages without branches: the list
  //      entries (a position beyond the list's end repeats the batch's first entry and is dropped at the end), the
  //      sixteen row loads, the places of the coarse sums, then the dot products -- so that the look-ups of different
  //      pairs overlap instead of forming one chain per pair.
  const int np0 = min(n0, 1024);
  for (int base = wave * 16; base < np0; base += 64) {
    int ent[16];
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) ent[jj] = pairs0[min(base + jj, np0 - 1)];
    typename R::Raw r[16];
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
      const int e = ent[jj];
      const typename R::Elem* fine = (e >> 13) ? ft : fp;
      r[jj] = *reinterpret_cast<const typename R::Raw*>(fine + (size_t)(((e >> 5) & 31) * W + (e & 31)) * g.D);
    }
    int srow[16];
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
      const int e = ent[jj], J = (e >> 10) & 7;
      srow[jj] = slot_of[node_index(g, J, ((e >> 5) & 31) >> J, (e & 31) >> J) - g.lvl_base[3]];
    }
    float dv[16];
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
      float xv[VEC];
      R::unpack(r[jj], xv);
      const float* sm = bigS + srow[jj] * g.cch + lane * VEC;
      float d = 0.f;
#pragma unroll
      for (int v = 0; v < VEC; ++v) d = fmaf(xv[v], sm[v], d);
      dv[jj] = (act && base + jj < np0) ? d : 0.f;
    }
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) tb[jj * 68 + lane] = dv[jj];
    wave_lds_fence();
    if (lane < 16) {
      const float4* row = reinterpret_cast<const float4*>(tb + lane * 68);
      float acc = 0.f;
#pragma unroll
      for (int jj = 0; jj < 16; ++jj) {
        const float4 q = row[jj];
        acc += (q.x + q.y) + (q.z + q.w);
      }
      if (base + lane < np0) {
        const int e = pairs0[base + lane];
        out[((e >> 5) & 31) * W + (e & 31)] = acc;
      }
    }
    wave_lds_fence();
  }

  // ---- big pairs with a finer node above the cell level, one at a time
  const int npx = min(nX, 512);
  for (int pi = wave; pi < npx; pi += 4) {
    const int q = pairsX[pi];
    const int a = lvl_t[q], bb = lvl_p[q];
    const int J = max(a, bb), lf = min(a, bb);
    const int y = q / W, x = q - y * W;
    const int nid = node_index(g, J, y >> J, x >> J) - g.lvl_base[3];
    float SB[VEC];
    if (lf >= 3) {
      // when the levels are equal the join block is frame t's node (staged), the finer one is frame t-1's
      const int ff = a < bb ? f : f - 1;
      const float* row = nsum + ((size_t)ff * NB + node_index(g, lf, y >> lf, x >> lf) - g.lvl_base[3]) * g.D;
#pragma unroll
      for (int v = 0; v < VEC; ++v) SB[v] = act ? row[ch0 + v] : 0.f;
    } else {
      block_sum<DT>(a < bb ? ft : fp, g.D, H, W, y, x, 1 << lf, act, SB);
    }
    const float* sm = bigS + slot_of[nid] * g.cch + lane * VEC;
    float d = 0.f;
#pragma unroll
    for (int v = 0; v < VEC; ++v) d = fmaf(SB[v], sm[v], d);
    d = wave_sum(d);
    if (lane == 0) out[q] = d;
  }

  // ---- mid join blocks (4x4): the block's sum in the frame where it is one node, then every cell of the other
  //      frame dotted with it; the dot product of a finer node is the sum over its cells (eight rows in flight)
  const int nm = min(nmid, 64);
  for (int ti = wave; ti < nm; ti += 4) {
    const int c = mid[ti];
    const int a = lvl_t[c], bb = lvl_p[c];
    const bool coarse_is_t = a >= bb;
    const int y0 = c / W, x0 = c - y0 * W;
    const typename R::Elem* coarse = coarse_is_t ? ft : fp;
    const typename R::Elem* fine = coarse_is_t ? fp : ft;
    const uint8_t* fine_lvl = coarse_is_t ? lvl_p : lvl_t;
    float SA[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) SA[v] = 0.f;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      typename R::Raw r[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int y = y0 + half * 2 + (j >> 2), x = x0 + (j & 3);
        r[j] = R::zero();
        if (y < H && x < W && act) r[j] = *reinterpret_cast<const typename R::Raw*>(coarse + (size_t)(y * W + x) * g.D);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float t[VEC];
        R::unpack(r[j], t);
#pragma unroll
        for (int v = 0; v < VEC; ++v) SA[v] += t[v];
      }
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      typename R::Raw r[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int y = y0 + half * 2 + (j >> 2), x = x0 + (j & 3);
        r[j] = R::zero();
        if (y < H && x < W && act) r[j] = *reinterpret_cast<const typename R::Raw*>(fine + (size_t)(y * W + x) * g.D);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float t[VEC];
        R::unpack(r[j], t);
        float d = 0.f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) d = fmaf(t[v], SA[v], d);
        tb[(half * 8 + j) * 68 + lane] = d;
      }
    }
    wave_lds_fence();
    float cd = 0.f;  // lane i < 16: the dot product of cell (i / 4, i % 4) of the block with the coarse sum
    if (lane < 16) {
      const float4* row = reinterpret_cast<const float4*>(tb + lane * 68);
#pragma unroll
      for (int jj = 0; jj < 16; ++jj) {
        const float4 q = row[jj];
        cd += (q.x + q.y) + (q.z + q.w);
      }
    }
    wave_lds_fence();
    const float s4 = (cd + __shfl_down(cd, 1, 64)) + (__shfl_down(cd, 4, 64) + __shfl_down(cd, 5, 64));  // 2x2 at lane
    float s16 = s4;  // lanes 0, 2, 8, 10 hold the four 2x2 sums
    s16 = (s16 + __shfl_down(s16, 2, 64)) + (__shfl_down(s16, 8, 64) + __shfl_down(s16, 10, 64));
    if (lane < 16) {
      const int dy = lane >> 2, dx = lane & 3, y = y0 + dy, x = x0 + dx;
      if (y < H && x < W) {
        const int cb = y * W + x, lf = min((int)fine_lvl[cb], 2);
        if (lf == 0) out[cb] = cd;
        else if (lf == 1 && !(dy & 1) && !(dx & 1)) out[cb] = s4;
        else if (lf == 2 && lane == 0) out[cb] = s16;
      }
    }
  }
}

__global__ __launch_bounds__(256) void k_select_clear_all(SelState* st) { sel_clear(st + blockIdx.x); }

void launch_temporal_dots(const Geo& g, const void* feats, const uint8_t* node_level, const float* nsum,
                          bool skip_cells, float* pd_part, SelState* sel, hipStream_t s) {
  if (g.T < 2) {  // no frame pairs: only the search states have to be reset
    hipLaunchKernelGGL(k_select_clear_all, dim3(g.B), dim3(256), 0, s, sel);
    return;
  }
  const int per_die = (g.B * (g.T - 1) + 7) / 8;
  dim3 grid(8 * per_die * g.nC), block(256);
  const int U = g.P >= 8 ? g.P >> 3 : 1;  // at most U x U disjoint join blocks at levels >= 3
  const size_t lds = g.L >= 3 ? (size_t)U * U * g.cch * sizeof(float) : 0;
  if (g.dtype == 1)
    hipLaunchKernelGGL(k_temporal_dots<1>, grid, block, lds, s, g, feats, node_level, nsum, (int)skip_cells, pd_part,
                       sel);
  else if (g.dtype == 2)
    hipLaunchKernelGGL(k_temporal_dots<2>, grid, block, lds, s, g, feats, node_level, nsum, (int)skip_cells, pd_part,
                       sel);
  else
    hipLaunchKernelGGL(k_temporal_dots<0>, grid, block, lds, s, g, feats, node_level, nsum, (int)skip_cells, pd_part,
                       sel);
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
// match = 1 (only the destination under n's top-left cell counts): that pair always lives at n's own top-left
// cell -- n is the finer node, or the destination there is and shares the corner -- so e_n is that one entry.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_temporal_resolve(Geo g, int match, const int32_t* __restrict__ node_map,
                                                          const uint8_t* __restrict__ node_level,
                                                          const float* __restrict__ pd_part,
                                                          const float* __restrict__ cell_part,
                                                          const float* __restrict__ nrm2,
                                                          float* __restrict__ sig, float* __restrict__ e,
                                                          uint32_t* __restrict__ sel_key,
                                                          SelState* __restrict__ sel) {
  __shared__ PairFrame pf;
  __shared__ unsigned ekey[1024];
  __shared__ unsigned h0[kSelBins];
  const int f = blockIdx.x, HW = g.HW, W = g.W;
  if (f % g.T == 0) {
    for (int c = threadIdx.x; c < HW; c += blockDim.x) sel_key[(size_t)f * HW + c] = 0;
    return;
  }
  load_pair_frame(g, f, node_map, node_level, pf);
  for (int c = threadIdx.x; c < HW; c += blockDim.x) ekey[c] = 0;
  for (int j = threadIdx.x; j < kSelBins; j += blockDim.x) h0[j] = 0;
  __syncthreads();
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    const int a = pf.lvl_t[c], b = pf.lvl_p[c];
    const int n = pf.rep_t[c], d = pf.rep_p[c];
    if ((a <= b ? n : d) != c) continue;  // not the top-left cell of the finer node
    // the two norms and the per-chunk partial dot products, eight chunks in flight, added in chunk order
    const float nn = nrm2[(size_t)f * g.NN + node_idx_of(g, a, n / W, n % W)];
    const float nd = nrm2[(size_t)(f - 1) * g.NN + node_idx_of(g, b, d / W, d % W)];
    float dot = 0.f;
    const float* pp = pd_part + (size_t)f * g.nC * HW + c;
    size_t cstride = HW;  // from one chunk's partial to the next
    if (cell_part && a == 0 && b == 0) {
      // two single cells: the spatial pass of frame t-1 left the dot product with the same cell of frame t
      const int y = c / W, x = c - y * W, NU = unit_cols(g) * unit_rows(g);
      cstride = (size_t)NU * kUnitScalars;
      pp = cell_part + ((size_t)(f - 1) * g.nC * NU + (y >> 3) * unit_cols(g) + (x >> 3)) * kUnitScalars +
           unit_cell_dot_slot(y, x);
    }
    for (int k0 = 0; k0 < g.nC; k0 += 8) {
      float pv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) pv[u] = k0 + u < g.nC ? pp[(size_t)(k0 + u) * cstride] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) dot += pv[u];
    }
    const float v = cosine_from(dot, nn, nd);
    sig[(size_t)f * HW + c] = v;
    if (v == v && (match != 1 || c == n)) atomicMax(&ekey[n], float_key(v));
  }
  __syncthreads();
  for (int c0 = 0; c0 < HW; c0 += blockDim.x) {  // uniform trip count: the histogram update is wave-wide
    const int c = c0 + threadIdx.x;
    unsigned key = 0;
    if (c < HW) {
      const size_t i = (size_t)f * HW + c;
      if (pf.rep_t[c] == c) {
        const unsigned k = ekey[c];                 // 0 only if every similarity was NaN
        e[i] = k ? key_float(k) : -2.f;
        key = k ? k : float_key(-2.f);
      }
      sel_key[i] = key;
    }
    wave_hist_add(h0, key != 0, key >> 21, 1u);
  }
  __syncthreads();
  sel_flush_level0(sel + f / g.T, h0);
}

void launch_temporal_resolve(const Geo& g, int match, const int32_t* node_map, const uint8_t* node_level,
                             const float* pd_part, const float* cell_part, const float* nrm2, float* sig, float* e,
                             uint32_t* sel_key, SelState* sel, hipStream_t s) {
  hipLaunchKernelGGL(k_temporal_resolve, dim3(g.F), dim3(256), 0, s, g, match, node_map, node_level, pd_part, cell_part,
                     nrm2, sig, e, sel_key, sel);
}

// ------------------------------------------------------------------------------------------------
// k_temporal_parent: directed edge of every kept node (Sec. 3.3). Among the destinations whose similarity
// exceeds tau_T: the one towards the top-left (smallest raster index; integer min in LDS) -- or, by `match`,
// only the one under the node's top-left cell, or the most similar one (64-bit integer max in LDS over
// (similarity image, reversed raster index), so ties go towards the top-left). Also seeds the
// pointer-jumping array.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void k_temporal_parent(Geo g, int match, const int32_t* __restrict__ node_map,
                                                         const uint8_t* __restrict__ node_level,
                                                         const float* __restrict__ sig,
                                                         float* __restrict__ tau,
                                                         const SelState* __restrict__ pending,
                                                         int32_t* __restrict__ parent, int32_t* __restrict__ ptr) {
  __shared__ PairFrame pf;
  __shared__ int par[1024];
  __shared__ unsigned long long best[1024];
  const int f = blockIdx.x, HW = g.HW;
  float th;
  if (pending) {  // the budget search left its last digit to this kernel
    th = sel_last_digit(pending + f / g.T);
    if (f % g.T == 0 && threadIdx.x == 0) tau[f / g.T] = th;
  } else {
    th = tau[f / g.T];
  }
  if (f % g.T == 0) {
    for (int c = threadIdx.x; c < HW; c += blockDim.x) {
      parent[(size_t)f * HW + c] = -1;
      ptr[(size_t)f * HW + c] = f * HW + c;
    }
    return;
  }
  load_pair_frame(g, f, node_map, node_level, pf);
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    par[c] = 0x7fffffff;
    best[c] = 0ull;
  }
  __syncthreads();
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    const int a = pf.lvl_t[c], b = pf.lvl_p[c];
    const int n = pf.rep_t[c], d = pf.rep_p[c];
    if ((a <= b ? n : d) != c) continue;
    const float v = sig[(size_t)f * HW + c];
    if (!(v > th)) continue;
    if (match == 2)
      atomicMax(&best[n], ((unsigned long long)float_key(v) << 32) | (unsigned)(0x7fffffff - d));
    else if (match == 0 || c == n)
      atomicMin(&par[n], d);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < HW; c += blockDim.x) {
    const int i = f * HW + c;
    int p = -1;
    if (pf.rep_t[c] == c) {
      if (match == 2) {
        if (best[c] != 0ull) p = (f - 1) * HW + (0x7fffffff - (int)(best[c] & 0xffffffffull));
      } else if (par[c] != 0x7fffffff) {
        p = (f - 1) * HW + par[c];
      }
    }
    parent[i] = p;
    ptr[i] = p >= 0 ? p : i;
  }
}

void launch_temporal_parent(const Geo& g, int match, const int32_t* node_map, const uint8_t* node_level,
                            const float* sig, float* tau, const SelState* pending, int32_t* parent, int32_t* ptr,
                            hipStream_t s) {
  hipLaunchKernelGGL(k_temporal_parent, dim3(g.F), dim3(kSelThreads), 0, s, g, match, node_map, node_level, sig, tau,
                     pending, parent, ptr);
}

// ------------------------------------------------------------------------------------------------
// Common root of every chain by pointer jumping (root finding of Sec. 3.3): every edge points one
// frame back, so a chain has at most T-1 edges; each launch multiplies the reach by kHops.
// ------------------------------------------------------------------------------------------------
// One launch follows up to kHops edges of the previous array, i.e. multiplies the reach by kHops; a walk stops at a
// root (an entry that points to itself), so short chains cost a load or two.
constexpr int kHops = 23;
__global__ __launch_bounds__(256) void k_root_jump(int n, const int32_t* __restrict__ src,
                                                   int32_t* __restrict__ dst) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int p = i;
  for (int h = 0; h < kHops; ++h) {
    const int q = src[p];
    if (q == p) break;
    p = q;
  }
  dst[i] = p;
}

// Last round, taken from every cell's node: cluster id = root of the node covering the cell.
__global__ __launch_bounds__(256) void k_root_jump_cells(int n, int hops, const int32_t* __restrict__ src,
                                                         const int32_t* __restrict__ node_map,
                                                         int32_t* __restrict__ cluster_ids) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int p = node_map[i];
  for (int h = 0; h < hops; ++h) {
    const int q = src[p];
    if (q == p) break;
    p = q;
  }
  cluster_ids[i] = p;
}

void launch_roots(const Geo& g, int32_t* ptr_a, int32_t* ptr_b, const int32_t* node_map, int32_t* cluster_ids,
                  hipStream_t s) {
  int rounds = 0;
  for (long long reach = 1; reach < g.T; reach *= kHops) ++rounds;
  dim3 grid((g.N + 255) / 256), block(256);
  int32_t* src = ptr_a;
  int32_t* dst = ptr_b;
  for (int r = 0; r + 1 < rounds; ++r) {
    hipLaunchKernelGGL(k_root_jump, grid, block, 0, s, g.N, src, dst);
    int32_t* tmp = src; src = dst; dst = tmp;
  }
  hipLaunchKernelGGL(k_root_jump_cells, grid, block, 0, s, g.N, rounds > 0 ? kHops : 0, src, node_map,
                     cluster_ids);
}

}  // namespace sttm
