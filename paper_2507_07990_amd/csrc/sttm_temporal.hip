// Temporal stage (Sec. 3.3): similarities between every kept node of frame t and the kept nodes of
// frame t-1 it overlaps, directed edges with top-left priority, and the common root of every chain.
#include "sttm_dev.h"

namespace sttm {

// Sum of the valid cells of a block of at most 4x4 cells (h x w of them valid, h, w >= 1) with top-left cell
// (y0, x0), for this lane's channels: all row loads are issued before the first one is used.
template <int DT>
__device__ inline void block_sum16(const typename Row<DT>::Elem* fb, int D, int W, int y0, int x0, int h, int w,
                                   bool act, float (&S)[Row<DT>::VEC]) {
  typedef Row<DT> R;
  constexpr int VEC = R::VEC;
  typename R::Raw r[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int dy = i >> 2, dx = i & 3;
    r[i] = R::zero();
    if (dy < h && dx < w && act) r[i] = *reinterpret_cast<const typename R::Raw*>(fb + (size_t)((y0 + dy) * W + x0 + dx) * D);
  }
#pragma unroll
  for (int v = 0; v < VEC; ++v) S[v] = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    float t[VEC];
    R::unpack(r[i], t);
#pragma unroll
    for (int v = 0; v < VEC; ++v) S[v] += t[v];
  }
}

// ------------------------------------------------------------------------------------------------
// The feature pass of the temporal stage, in two kernels.
// The two frames' partitions are both quadtree cuts, so any two overlapping nodes are nested; a pair is named by
// the top-left cell q of its finer node, and its "join" block is the coarser node.
//
// k_temporal_plan, one workgroup per frame t >= 1, looks at the node levels of frames t and t-1 only and cuts the
// pair's work into items of about equal size, by join level J:
//  * J <= 1 ("fast"): aligned 2x2 regions in which both frames' nodes are single cells or the 2x2 block; four
//    regions per item.
//  * J == 2 ("mid"): one 4x4 block per item.
//    With `skip_same` the regions (1: of single cells; 2: also 2x2 and 4x4 blocks) that are the same node
//    in both frames are left out: the spatial pass has already formed those dot products (k_temporal_resolve
//    reads them from its table).
//  * J >= 3 ("big"): the coarse sum is not recomputed: the spatial pass left the per-channel sums of all nodes
//    at levels >= 3 in `nsum`. Pairs whose finer node is a single cell go sixteen to an item (all under the same
//    join block), every other finer node is an item of its own.
// The items go into kTQueues queues, frame f into queue f mod kTQueues (a workgroup reserves its stretch with one
// atomic on the queue's counter; with one counter for all, the five hundred atomics of a long video queued up
// behind one another). The order of the stretches varies from run to run, what is computed for an item does not.
//
// k_temporal_dots, a fixed grid of four-wavefront workgroups, a fixed share of them per queue: wavefront w of a
// queue's share takes the (item, chunk) tasks w, w + W, w + 2W, ... of that queue (a trip count known on entry),
// loads the rows the item names, and reduces its lanes' partial dot products through LDS ([scalar][lane] rows).
// Because every task is small and they are all alike, the pass no longer depends on how unevenly the work is
// spread over the frame pairs (scene cuts concentrate it in a few of them).
// Output: pd_part[f][chunk][q].
// ------------------------------------------------------------------------------------------------
struct TItem {
  int32_t f;     // frame t of the pair
  int16_t type;  // 0 fast, 1 mid, 2 cells under a big block, 3 one finer node under a big block
  int16_t n;     // fast: regions (1..4); cells: cells (1..16)
  int16_t a;     // mid: top-left cell of the block; big: join block's node index counted from the first level-3 node
  int16_t b;     // mid, big: 1 when the join block is frame t's node (else frame t-1's)
  // fast: region's top-left cell | (frame t holds the 2x2 block) << 10 | (frame t-1 does) << 11
  // mid:  level (0..2) of the other frame's node at each of the block's 16 cells
  // cells: the cells; node: top-left cell of the finer node, its level
  int16_t e[18];
};
static_assert(sizeof(TItem) == 48, "three 16-byte pieces");

__host__ __device__ inline int temporal_items_per_pair(const Geo& g) { return g.P * g.P / 4 + g.P * g.P / 64 + 4; }
constexpr int kFastRows = 16;
constexpr int kBigNodes = 24;  // nodes at levels >= 3 of a 32x32 grid: 16 + 4 + 1
constexpr int kTQueues = 64;
constexpr int kTShare = 16;  // workgroups per queue at most
constexpr int kTCountStride = 32;  // ints between two queues' counters: a 128-byte line each

__host__ __device__ inline int temporal_queue_items(const Geo& g) {
  return ((g.F + kTQueues - 1) / kTQueues) * temporal_items_per_pair(g);
}


__global__ __launch_bounds__(256) void k_temporal_plan(Geo g, const uint8_t* __restrict__ node_level, int skip_same,
                                                       TItem* __restrict__ items, int* __restrict__ count,
                                                       SelState* __restrict__ sel) {
  __shared__ uint8_t lvl_t[1024], lvl_p[1024];
  __shared__ int16_t fast[256], mid[64], pairs0[1024], pairsX[256];
  __shared__ int nfast, nmid, nX, s_base;
  __shared__ int cnt0[kBigNodes], fill0[kBigNodes], off0[kBigNodes + 1], ioff0[kBigNodes + 1];
  __shared__ uint8_t coarse_t[kBigNodes];
  const int f = blockIdx.x, t = f % g.T, b = f / g.T;
  const int H = g.H, W = g.W, HW = g.HW, tid = threadIdx.x;
  if (t == 0) {  // no pair ends here; the temporal budget search of this video starts afresh
    sel_clear(sel + b);
    return;
  }
  if (tid == 0) { nfast = nmid = nX = 0; }
  if (tid < kBigNodes) cnt0[tid] = fill0[tid] = 0;
  for (int c = tid; c < HW; c += blockDim.x) {
    lvl_t[c] = node_level[(size_t)f * HW + c];
    lvl_p[c] = node_level[(size_t)(f - 1) * HW + c];
  }
  __syncthreads();
  for (int c = tid; c < HW; c += blockDim.x) {
    const int a = lvl_t[c], bb = lvl_p[c];
    const int J = max(a, bb), lf = min(a, bb);
    const int y = c / W, x = c - y * W;
    const bool join_head = !(y & ((1 << J) - 1)) && !(x & ((1 << J) - 1));
    // (where both frames keep the same node at a level <= 2 there is nothing to do when the spatial pass left
    // those dot products)
    const bool same_done = a == bb && (skip_same >= 2 || (skip_same == 1 && a == 0));
    if (J <= 1) {
      if (!(y & 1) && !(x & 1) && !same_done) fast[atomicAdd(&nfast, 1)] = (int16_t)c;
    } else if (J == 2) {
      if (join_head && !same_done) mid[atomicAdd(&nmid, 1)] = (int16_t)c;
    } else {
      const int nid = node_index(g, J, y >> J, x >> J) - g.lvl_base[3];
      if (join_head) coarse_t[nid] = a >= bb ? 1 : 0;
      if (!(y & ((1 << lf) - 1)) && !(x & ((1 << lf) - 1))) {  // top-left cell of the finer node
        if (lf == 0) atomicAdd(&cnt0[nid], 1);
        else pairsX[atomicAdd(&nX, 1)] = (int16_t)c;
      }
    }
  }
  __syncthreads();
  if (tid <= kBigNodes) {  // where each join block's cells start in pairs0, and where its items start among the cell items
    int o = 0, io = 0;
    for (int s = 0; s < tid; ++s) {
      o += cnt0[s];
      io += (cnt0[s] + 15) >> 4;
    }
    off0[tid] = o;
    ioff0[tid] = io;
    if (tid == kBigNodes) {
      const int total = ((nfast + 3) >> 2) + nmid + io + nX;
      s_base = total ? atomicAdd(count + (f % kTQueues) * kTCountStride, total) : 0;
    }
  }
  __syncthreads();
  for (int c = tid; c < HW; c += blockDim.x) {
    const int a = lvl_t[c], bb = lvl_p[c];
    if (max(a, bb) >= 3 && min(a, bb) == 0) {
      const int J = max(a, bb), y = c / W, x = c - y * W;
      const int nid = node_index(g, J, y >> J, x >> J) - g.lvl_base[3];
      pairs0[off0[nid] + atomicAdd(&fill0[nid], 1)] = (int16_t)c;
    }
  }
  __syncthreads();
  // The items are written piecemeal, one thread per header and one per entry (an item assembled in registers and
  // stored in one piece needs its entry array indexed at run time, which cost more than everything else here).
  const int nfi = (nfast + 3) >> 2, nmi = nmid, n0i = ioff0[kBigNodes], nxi = nX;
  const int ntot = nfi + nmi + n0i + nxi;
  TItem* out = items + (size_t)(f % kTQueues) * temporal_queue_items(g) + s_base;
  for (int idx = tid; idx < ntot * 19; idx += blockDim.x) {
    const int i = idx / 19, j = idx - i * 19 - 1;  // j = -1: the header
    int type, n = 0, a = 0, bflag = 0, ev = 0;
    if (i < nfi) {
      type = 0;
      n = min(4, nfast - 4 * i);
      if (j >= 0 && j < n) {
        const int c0 = fast[4 * i + j];
        ev = c0 | ((lvl_t[c0] == 1 ? 1 : 0) << 10) | ((lvl_p[c0] == 1 ? 1 : 0) << 11);
      }
    } else if (i < nfi + nmi) {
      const int c = mid[i - nfi];
      const bool coarse_is_t = lvl_t[c] >= lvl_p[c];
      type = 1;
      a = c;
      bflag = coarse_is_t ? 1 : 0;
      if (j >= 0 && j < 16) {
        const int y = c / W + (j >> 2), x = c % W + (j & 3);
        if (y < H && x < W) ev = min((int)(coarse_is_t ? lvl_p : lvl_t)[y * W + x], 2);
      }
    } else if (i < nfi + nmi + n0i) {
      const int k = i - nfi - nmi;
      int sl = 0;
      while (ioff0[sl + 1] <= k) ++sl;  // the join block this item belongs to (at most kBigNodes steps)
      const int first = off0[sl] + 16 * (k - ioff0[sl]);
      type = 2;
      n = min(16, off0[sl + 1] - first);
      a = sl;
      bflag = coarse_t[sl];
      if (j >= 0 && j < n) ev = pairs0[first + j];
    } else {
      const int q = pairsX[i - nfi - nmi - n0i];
      const int la = lvl_t[q], lb = lvl_p[q], J = max(la, lb), y = q / W, x = q - y * W;
      type = 3;
      a = node_index(g, J, y >> J, x >> J) - g.lvl_base[3];
      bflag = la >= lb ? 1 : 0;
      ev = j == 0 ? q : min(la, lb);
    }
    if (j < 0) {
      out[i].f = f;
      out[i].type = (int16_t)type;
      out[i].n = (int16_t)n;
      out[i].a = (int16_t)a;
      out[i].b = (int16_t)bflag;
    } else if (j < 18) {
      out[i].e[j] = (int16_t)ev;
    }
  }
}

// Sums the 16 rows [row][lane] of a wavefront's LDS staging area: lane r < 16 returns the sum of row r.
__device__ inline float rows16_sum(const float* tb, int lane) {
  float acc = 0.f;
  if (lane < 16) {
    const float4* row = reinterpret_cast<const float4*>(tb + lane * 68);
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
      const float4 q = row[jj];
      acc += (q.x + q.y) + (q.z + q.w);
    }
  }
  return acc;
}

template <int DT>
__global__ __launch_bounds__(256) void k_temporal_dots(Geo g, const void* __restrict__ feats_v,
                                                       const float* __restrict__ nsum,
                                                       const TItem* __restrict__ items,
                                                       const int* __restrict__ count, float* __restrict__ pd_part) {
  typedef Row<DT> R;
  constexpr int VEC = R::VEC;
  __shared__ float tbuf[4][kFastRows * 68];
  // (the wavefront's number is the same in all its lanes: said explicitly, so that everything derived from it --
  // the task, the item and the row addresses -- is kept in scalar registers)
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;
  const int H = g.H, W = g.W, HW = g.HW;
  const int NB = g.NN - g.lvl_base[3];
  float* tb = tbuf[wave];
  // Workgroups go to the eight dies round-robin by their index: the workgroups of die d serve the queues 8d .. 8d+7,
  // i.e. eight consecutive frames of every 64, so that the two frame pairs that need a frame's rows mostly meet in
  // one L2.
  const int slot = blockIdx.x % kTQueues, share = blockIdx.x / kTQueues;
  static_assert(kTQueues == 64, "queue <-> die mapping below");
  const int queue = ((slot & 7) << 3) | (slot >> 3);
  items += (size_t)queue * temporal_queue_items(g);
  const int ntasks = count[queue * kTCountStride] * g.nC, stride = (int)(gridDim.x / kTQueues) * 4;
  for (int task = share * 4 + wave; task < ntasks; task += stride) {
    const int ii = task / g.nC, chunk = task - ii * g.nC;
    const TItem it = items[ii];  // the same for all lanes
    const int f = it.f;
    const int ch0 = chunk * g.cch + lane * VEC;
    const bool act = ch0 < g.D;
    const typename R::Elem* ft =
        reinterpret_cast<const typename R::Elem*>(feats_v) + (size_t)f * HW * g.D + (act ? ch0 : 0);
    const typename R::Elem* fp = ft - (size_t)HW * g.D;
    float* out = pd_part + (size_t)(f * g.nC + chunk) * HW;
    if (it.type == 0) {
      // ---- up to four 2x2 regions, two at a time (16 rows in flight)
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        typename R::Raw rt[2][4], rp[2][4];
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
          const int ri = half * 2 + rr;
          const int c0 = ri < it.n ? (it.e[ri] & 1023) : -1;
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
          const int ri = half * 2 + rr;
          const int e = ri < it.n ? it.e[ri] : 0;
          const bool t_block = (e >> 10) & 1, p_block = (e >> 11) & 1;  // wave-uniform
          if (!t_block && !p_block) {  // four cells against four cells: no sums needed
#pragma unroll
            for (int k = 0; k < 4; ++k) tb[(ri * 4 + k) * 68 + lane] = R::dot(rt[rr][k], rp[rr][k]);
            continue;
          }
          // a frame that holds the 2x2 block takes part with the sum of its four cells
          float st[VEC], sp[VEC];
#pragma unroll
          for (int v = 0; v < VEC; ++v) st[v] = sp[v] = 0.f;
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            float xv[VEC];
            if (t_block) {
              R::unpack(rt[rr][k], xv);
#pragma unroll
              for (int v = 0; v < VEC; ++v) st[v] += xv[v];
            }
            if (p_block) {
              R::unpack(rp[rr][k], xv);
#pragma unroll
              for (int v = 0; v < VEC; ++v) sp[v] += xv[v];
            }
          }
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            float xa[VEC], xb[VEC];
            if (t_block) {
#pragma unroll
              for (int v = 0; v < VEC; ++v) xa[v] = st[v];
            } else {
              R::unpack(rt[rr][k], xa);
            }
            if (p_block) {
#pragma unroll
              for (int v = 0; v < VEC; ++v) xb[v] = sp[v];
            } else {
              R::unpack(rp[rr][k], xb);
            }
            float d = 0.f;
#pragma unroll
            for (int v = 0; v < VEC; ++v) d = fmaf(xa[v], xb[v], d);
            tb[(ri * 4 + k) * 68 + lane] = d;
          }
        }
        STTM_SCHED_FENCE();  // (the second half's rows are not asked for before the first half is done with its registers)
      }
      wave_lds_fence();
      const float acc = rows16_sum(tb, lane);
      if (lane < kFastRows) {
        const int ri = lane >> 2, k = lane & 3;
        if (ri < it.n) {
          const int e = items[ii].e[ri], c0 = e & 1023;
          const int y = c0 / W + (k >> 1), x = c0 % W + (k & 1);
          const bool both_block = ((e >> 10) & 3) == 3;
          if (y < H && x < W && (k == 0 || !both_block)) out[y * W + x] = acc;
        }
      }
      wave_lds_fence();
    } else if (it.type == 1) {
      // ---- a 4x4 join block: its sum in the frame where it is one node, then every cell of the other frame dotted
      //      with it; the dot product of a finer node is the sum over its cells
      const int c = it.a;
      const bool coarse_is_t = it.b != 0;
      const int y0 = c / W, x0 = c - y0 * W;
      const typename R::Elem* coarse = coarse_is_t ? ft : fp;
      const typename R::Elem* fine = coarse_is_t ? fp : ft;
      float SA[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) SA[v] = 0.f;
      {
        typename R::Raw rc[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int y = y0 + (j >> 2), x = x0 + (j & 3);
          rc[j] = R::zero();
          if (y < H && x < W && act) rc[j] = *reinterpret_cast<const typename R::Raw*>(coarse + (size_t)(y * W + x) * g.D);
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          float tv[VEC];
          R::unpack(rc[j], tv);
#pragma unroll
          for (int v = 0; v < VEC; ++v) SA[v] += tv[v];
        }
      }
      STTM_SCHED_FENCE();  // the second sixteen rows are asked for only now: 32 in flight cost a wavefront per SIMD
      {
        typename R::Raw rf[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int y = y0 + (j >> 2), x = x0 + (j & 3);
          rf[j] = R::zero();
          if (y < H && x < W && act) rf[j] = *reinterpret_cast<const typename R::Raw*>(fine + (size_t)(y * W + x) * g.D);
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          float tv[VEC];
          R::unpack(rf[j], tv);
          float d = 0.f;
#pragma unroll
          for (int v = 0; v < VEC; ++v) d = fmaf(tv[v], SA[v], d);
          tb[j * 68 + lane] = d;
        }
      }
      wave_lds_fence();
      const float cd = rows16_sum(tb, lane);  // lane i < 16: cell (i / 4, i % 4) of the block against the coarse sum
      wave_lds_fence();
      const float s4 = (cd + __shfl_down(cd, 1, 64)) + (__shfl_down(cd, 4, 64) + __shfl_down(cd, 5, 64));  // 2x2 at lane
      float s16 = s4;  // lanes 0, 2, 8, 10 hold the four 2x2 sums
      s16 = (s16 + __shfl_down(s16, 2, 64)) + (__shfl_down(s16, 8, 64) + __shfl_down(s16, 10, 64));
      if (lane < 16) {
        const int dy = lane >> 2, dx = lane & 3, y = y0 + dy, x = x0 + dx;
        if (y < H && x < W) {
          const int cb = y * W + x, lf = items[ii].e[lane];
          if (lf == 0) out[cb] = cd;
          else if (lf == 1 && !(dy & 1) && !(dx & 1)) out[cb] = s4;
          else if (lf == 2 && lane == 0) out[cb] = s16;
        }
      }
    } else {
      // ---- under a join block at a level >= 3: its stored sum against single cells (sixteen at a time) or against
      //      one finer node
      const bool coarse_is_t = it.b != 0;
      const int fc = coarse_is_t ? f : f - 1;  // frame in which the join block is one node
      const typename R::Elem* fine = coarse_is_t ? fp : ft;
      const float* srow = nsum + ((size_t)fc * NB + it.a) * g.D + (act ? ch0 : 0);
      float S[VEC];
#pragma unroll
      for (int v = 0; v < VEC; v += 4) {
        const float4 q = *reinterpret_cast<const float4*>(srow + v);
        S[v] = q.x; S[v + 1] = q.y; S[v + 2] = q.z; S[v + 3] = q.w;
      }
      if (it.type == 2) {
        typename R::Raw r[16];
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
          const int cq = jj < it.n ? it.e[jj] : it.e[0];  // (a position beyond the item's end repeats a cell and is dropped)
          r[jj] = *reinterpret_cast<const typename R::Raw*>(fine + (size_t)cq * g.D);
        }
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
          float xv[VEC];
          R::unpack(r[jj], xv);
          float d = 0.f;
#pragma unroll
          for (int v = 0; v < VEC; ++v) d = fmaf(xv[v], S[v], d);
          tb[jj * 68 + lane] = act ? d : 0.f;
        }
        wave_lds_fence();
        const float acc = rows16_sum(tb, lane);
        if (lane < it.n) out[items[ii].e[lane]] = acc;
        wave_lds_fence();
      } else {
        const int q = it.e[0], lf = it.e[1];
        const int y = q / W, x = q - y * W;
        float SB[VEC];
        if (lf >= 3) {
          const int ff = coarse_is_t ? f - 1 : f;
          const float* row = nsum + ((size_t)ff * NB + node_index(g, lf, y >> lf, x >> lf) - g.lvl_base[3]) * g.D;
#pragma unroll
          for (int v = 0; v < VEC; ++v) SB[v] = act ? row[ch0 + v] : 0.f;
        } else {
          const int s = 1 << lf;
          block_sum16<DT>(fine, g.D, W, y, x, min(s, H - y), min(s, W - x), act, SB);
        }
        float d = 0.f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) d = fmaf(SB[v], S[v], d);
        if (!act) d = 0.f;
        d = wave_sum(d);
        if (lane == 0) out[q] = d;
      }
    }
  }
}

size_t temporal_items_bytes(const Geo& g) { return (size_t)kTQueues * temporal_queue_items(g) * sizeof(TItem); }
size_t temporal_count_bytes() { return (size_t)kTQueues * kTCountStride * sizeof(int); }

void launch_temporal_dots(const Geo& g, const void* feats, const uint8_t* node_level, const float* nsum,
                          int skip_same, float* pd_part, SelState* sel, void* items, int* item_count,
                          hipStream_t s) {
  TItem* q = reinterpret_cast<TItem*>(items);
  hipLaunchKernelGGL(k_temporal_plan, dim3(g.F), dim3(256), 0, s, g, node_level, skip_same, q, item_count, sel);
  // enough wavefronts for about four tasks each if every pair came with all the items it can have, the same
  // number of workgroups for every queue
  const long long worst = (long long)temporal_queue_items(g) * g.nC;
  long long share = (worst + 15) / 16;
  if (share < 1) share = 1;
  if (share > kTShare) share = kTShare;
  const dim3 grid((unsigned)(share * kTQueues)), block(256);
  if (g.dtype == 1)
    hipLaunchKernelGGL(k_temporal_dots<1>, grid, block, 0, s, g, feats, nsum, q, item_count, pd_part);
  else if (g.dtype == 2)
    hipLaunchKernelGGL(k_temporal_dots<2>, grid, block, 0, s, g, feats, nsum, q, item_count, pd_part);
  else
    hipLaunchKernelGGL(k_temporal_dots<0>, grid, block, 0, s, g, feats, nsum, q, item_count, pd_part);
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
__global__ __launch_bounds__(256) void k_temporal_resolve(Geo g, int match, int same_level,
                                                          const int32_t* __restrict__ node_map,
                                                          const uint8_t* __restrict__ node_level,
                                                          const float* __restrict__ pd_part,
                                                          const float* __restrict__ cell_part,
                                                          const float* __restrict__ nrm2,
                                                          float* __restrict__ sig, float* __restrict__ e,
                                                          uint32_t* __restrict__ sel_key,
                                                          SelState* __restrict__ sel, int* __restrict__ item_count) {
  __shared__ PairFrame pf;
  __shared__ unsigned ekey[1024];
  __shared__ unsigned h0[kSelBins];
  const int f = blockIdx.x, HW = g.HW, W = g.W;
  if (f == 0 && threadIdx.x < kTQueues) item_count[threadIdx.x * kTCountStride] = 0;  // the feature pass is over: its queues are empty for the next one
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
    if (cell_part && a == b && a <= same_level) {
      // the same node (a cell, a 2x2 or a 4x4 block) in both frames: the spatial pass of frame t-1 left the dot
      // product of its sum with the same node's sum in frame t
      const int y = c / W, x = c - y * W, NU = unit_cols(g) * unit_rows(g);
      cstride = (size_t)NU * kUnitScalars;
      pp = cell_part + ((size_t)(f - 1) * g.nC * NU + (y >> 3) * unit_cols(g) + (x >> 3)) * kUnitScalars +
           (a == 0 ? unit_cell_dot_slot(y, x) : unit_node_dot_slot(a, y, x));
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

void launch_temporal_resolve(const Geo& g, int match, int same_level, const int32_t* node_map,
                             const uint8_t* node_level,
                             const float* pd_part, const float* cell_part, const float* nrm2, float* sig, float* e,
                             uint32_t* sel_key, SelState* sel, int* item_count, hipStream_t s) {
  hipLaunchKernelGGL(k_temporal_resolve, dim3(g.F), dim3(256), 0, s, g, match, same_level, node_map, node_level, pd_part,
                     cell_part,
                     nrm2, sig, e, sel_key, sel, item_count);
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
