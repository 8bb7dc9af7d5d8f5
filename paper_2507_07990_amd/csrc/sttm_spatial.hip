// Spatial stage (Sec. 3.2): pyramid sums, squared norms, parent-child cosine similarities, the
// coarse-to-fine decision, and the budget-driven threshold for it.
#include "sttm_dev.h"

namespace sttm {

constexpr int kTileRows = 36;    // 16 n0 + 16 d0 + 4 d1
// Rows of the staging area per tile, in batches of eight: four batches of the 2x2 blocks' statistics, one of the
// blocks' dot products with the tile (4) and with the next frame (4), two of the cell-to-cell dot products, one for
// the tile with the next frame.
constexpr int kStageRows = 64;
constexpr int kStageStride = 8;  // floats per staging row: one per group of eight lanes

// Issues the row loads of the tile whose top-left cell is (ty, tx); th x tw of its 4x4 cells are valid
// (th, tw >= 1). Every one of the 16 loads is issued, without a condition: a cell beyond the edge, or a lane
// beyond the last channel, reads a valid cell of the tile again (a cache hit) and tile_mask() discards it. The
// number of loads in flight is then known at compile time, and the wavefront can wait for this tile's rows
// while the next tile's are still on their way.
template <int DT>
__device__ __forceinline__ void tile_load(typename Row<DT>::Raw (&raw)[16], const typename Row<DT>::Elem* fbase,
                                          int W, int D, int ty, int tx, int th, int tw) {
  typedef Row<DT> R;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int q1 = i >> 2, k = i & 3;
    const int dy = min((q1 >> 1) * 2 + (k >> 1), th - 1), dx = min((q1 & 1) * 2 + (k & 1), tw - 1);
    raw[i] = *reinterpret_cast<const typename R::Raw*>(fbase + (size_t)((ty + dy) * W + tx + dx) * D);
  }
}

// Zeroes what tile_load fetched for cells beyond the edge and for lanes beyond the last channel.
template <int DT>
__device__ __forceinline__ void tile_mask(typename Row<DT>::Raw (&raw)[16], int th, int tw, bool act) {
  typedef Row<DT> R;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int q1 = i >> 2, k = i & 3;
    const int dy = (q1 >> 1) * 2 + (k >> 1), dx = (q1 & 1) * 2 + (k & 1);
    if (!(dy < th && dx < tw && act)) raw[i] = R::zero();
  }
}

// Eight scalars of the wavefront at once (v[i] = this lane's share of scalar i): returns, in lane l, the sum of
// scalar (l & 7) over the eight lanes of l's group (l >> 3). Three exchanges, each halving the scalars a lane
// carries: with the neighbour (lane ^ 1), across the quad (^ 2), across the two quads (^ 4).
__device__ __forceinline__ float group_sums8(const float (&v)[8], int lane) {
  const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
  float a[4], c[2];
#ifndef STTM_HOST_EMULATION
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float keep = b0 ? v[2 * i + 1] : v[2 * i], give = b0 ? v[2 * i] : v[2 * i + 1];
    a[i] = keep + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(give), 0xB1, 0xF, 0xF, true));  // quad_perm [1,0,3,2]
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float keep = b1 ? a[2 * i + 1] : a[2 * i], give = b1 ? a[2 * i] : a[2 * i + 1];
    c[i] = keep + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(give), 0x4E, 0xF, 0xF, true));  // quad_perm [2,3,0,1]
  }
  const float keep = b2 ? c[1] : c[0], give = b2 ? c[0] : c[1];
  int r = __builtin_amdgcn_update_dpp(0, __float_as_int(give), 0x104, 0xF, 0x5, true);  // lanes 0-3, 8-11 of a row: from lane + 4
  r = __builtin_amdgcn_update_dpp(r, __float_as_int(give), 0x114, 0xF, 0xA, true);      // lanes 4-7, 12-15: from lane - 4
  return keep + __int_as_float(r);
#else
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float keep = b0 ? v[2 * i + 1] : v[2 * i], give = b0 ? v[2 * i] : v[2 * i + 1];
    a[i] = keep + __shfl_xor(give, 1, 64);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float keep = b1 ? a[2 * i + 1] : a[2 * i], give = b1 ? a[2 * i] : a[2 * i + 1];
    c[i] = keep + __shfl_xor(give, 2, 64);
  }
  const float keep = b2 ? c[1] : c[0], give = b2 ? c[0] : c[1];
  return keep + __shfl_xor(give, 4, 64);
#endif
}

// Eight scalars go into the staging area as rows 8 * batch .. 8 * batch + 7, each row the eight partial sums of one
// scalar over the groups of eight lanes: one store per lane, all to different words. (Every lane calls it.)
__device__ __forceinline__ void stage8(float* tbs, int batch, int lane, const float (&v)[8]) {
  tbs[(batch * 8 + (lane & 7)) * kStageStride + (lane >> 3)] = group_sums8(v, lane);
}

// Adds row `row` of the staging area up (a fixed order).
__device__ __forceinline__ float staged_row_sum(const float* tbs, int row) {
  const float4* p = reinterpret_cast<const float4*>(tbs + row * kStageStride);
  const float4 a = p[0], b = p[1];
  return ((a.x + a.y) + (a.z + a.w)) + ((b.x + b.y) + (b.z + b.w));
}

// Sums and per-lane scalars of one tile: returns the tile's per-channel sum in S2 and stages the tile's scalars --
// batch q1 (rows 8 q1 .. 8 q1 + 7): squared norms of the four cells of 2x2 block q1, then each cell . the block's
// sum; p1[q1]: block sum . tile sum, left to the caller to stage (zero for cells and blocks beyond the edge).
// The rows must be zero for cells beyond the edge and for lanes beyond the last channel (tile_mask).
template <int DT>
__device__ __forceinline__ void tile_stats(const typename Row<DT>::Raw (&raw)[16], float* tbs, int lane, int th, int tw,
                                           float (&p1)[4], float (&S2)[Row<DT>::VEC],
                                           float (&S1)[4][Row<DT>::VEC]) {
  typedef Row<DT> R;
  constexpr int VEC = R::VEC;
#pragma unroll
  for (int v = 0; v < VEC; ++v) S2[v] = 0.f;
#pragma unroll
  for (int q1 = 0; q1 < 4; ++q1) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) S1[q1][v] = 0.f;
    if ((q1 >> 1) * 2 >= th || (q1 & 1) * 2 >= tw) continue;  // block beyond the edge (wave-uniform)
    // the block's sum, channel by channel; a cell's dot product with it is the sum of the cell's dot products with
    // the block's four cells, which come straight from the packed rows (no element is widened for them)
#pragma unroll
    for (int k = 0; k < 4; ++k) R::add_row(raw[q1 * 4 + k], S1[q1]);
    float nd[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) nd[k] = R::dot(raw[q1 * 4 + k], raw[q1 * 4 + k]);  // (zero rows give zero)
    {
      const float p01 = R::dot(raw[q1 * 4 + 0], raw[q1 * 4 + 1]), p02 = R::dot(raw[q1 * 4 + 0], raw[q1 * 4 + 2]);
      const float p03 = R::dot(raw[q1 * 4 + 0], raw[q1 * 4 + 3]), p12 = R::dot(raw[q1 * 4 + 1], raw[q1 * 4 + 2]);
      const float p13 = R::dot(raw[q1 * 4 + 1], raw[q1 * 4 + 3]), p23 = R::dot(raw[q1 * 4 + 2], raw[q1 * 4 + 3]);
      nd[4] = (nd[0] + p01) + (p02 + p03);
      nd[5] = (nd[1] + p01) + (p12 + p13);
      nd[6] = (nd[2] + p02) + (p12 + p23);
      nd[7] = (nd[3] + p03) + (p13 + p23);
    }
    stage8(tbs, q1, lane, nd);
#pragma unroll
    for (int v = 0; v < VEC; ++v) S2[v] += S1[q1][v];
  }
#pragma unroll
  for (int q1 = 0; q1 < 4; ++q1) {
    float d1 = 0.f;
#pragma unroll
    for (int v = 0; v < VEC; ++v) d1 = fmaf(S1[q1][v], S2[v], d1);
    p1[q1] = d1;
  }
}

// Asks for 16 bytes per lane straight into LDS: lane l's piece lands at byte address lds_row + 16 l of the
// workgroup's LDS (`lds_row` is the same in all lanes). No registers are involved; it completes in order with the
// wavefront's other loads. Written as an instruction of its own (the register that carries the LDS address is
// saved and put back) so that the compiler, which would wait for every load in flight at the next use of any loaded
// register once it has seen such a request, goes on counting the ordinary loads exactly; the wavefront waits for
// these rows itself (wait_loads_but) before it reads them.
template <class Elem>
__device__ __forceinline__ void load_row_to_lds(void* lds_base, int row_bytes, const Elem* src_lane, int lane) {
#ifndef STTM_HOST_EMULATION
  const unsigned dst = (unsigned)(size_t)(__attribute__((address_space(3))) void*)lds_base + (unsigned)row_bytes;
  unsigned keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(keep)
               : "v"(src_lane), "s"(dst)
               : "memory");
#else
  memcpy(static_cast<char*>(lds_base) + row_bytes + 16 * lane, src_lane, 16);
#endif
}

// Waits until at most `newer` (0 or 16) of the wavefront's loads are still on their way (they complete in issue
// order), and until its earlier LDS traffic is through.
__device__ __forceinline__ void wait_loads_but(int newer) {
#ifndef STTM_HOST_EMULATION
  if (newer >= 16) asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#endif
}

// ------------------------------------------------------------------------------------------------
// k_pyramid_stats: the one pass over the features of the spatial stage.
//
// One workgroup per (chunk, unit, frame) -- a 3-D grid, or a 1-D grid decoded die by die when the frame-to-frame dot
// products are wanted (template parameter CC, see below); a workgroup is ONE wavefront that owns a "unit" = an 8x8
// cell block (level 3) of one frame for one chunk of the token rows. Units at the ragged edge of the grid are
// smaller, but every workgroup is a single wavefront, so the hardware dispatcher evens the load out. A lane owns VEC
// consecutive channels, so all pyramid sums are private to the lane and only scalars are reduced across lanes:
// three exchanges between lanes leave eight partial sums per scalar, which go through a small LDS area
// ([scalar][8]) to the lane that adds them up.
// The unit is walked quadrant by quadrant: 4 tiles (4x4, level 2) of 4 level-1 blocks of 4 cells. The row
// loads of the next tile are issued before the current one is worked on; cells and blocks beyond the
// grid's edge cost no arithmetic (the tests are wave-uniform) and no memory traffic (their loads hit a row
// the tile has just fetched).
// Scalars: the squared norm of every cell, and for every node below the root the dot product of its sum
// with its parent's sum. (The squared norm of a parent is the sum of its children's dot products with it,
// which the finalize kernel adds up.)
// With CC the wavefront also needs each tile of the next frame, for x_c(t) . x_c(t+1) of the tile's cells (the dot
// products the temporal stage needs where both frames keep single cells): its 16 rows are asked for straight into
// LDS as soon as the tile's own rows have arrived -- no registers are held for them -- travel while the tile's
// statistics are worked out, and are read back for the dot products.
// Output: part[f][chunk][unit][kUnitScalars] = the workgroup's scalars, partial over this chunk's channels, written
//         as one block: per tile 16 squared norms, 16 cell and 4 level-1 dot products (child sum . parent sum), then
//         the 4 level-2 dot products, then per tile the 16 cell-to-cell dot products and the 4 + 1 of its blocks and
//         itself (zeros without CC); the levels from 3 up are the finalize kernel's when the pyramid is taller than
//         a unit;
//         nsum[f][node - first level-3 node][D] = the per-channel sums of the level-3 nodes (fp32), which
//         the later stages read instead of re-adding up to 64 token rows.
// (Two wavefronts per SIMD asked for: the CC = 2 instances would otherwise take a few registers more than half the
// file and run alone on their SIMD.)
// ------------------------------------------------------------------------------------------------
template <int DT, int CC>  // CC: 0 = statistics only, 1 = + cell-to-cell dot products, 2 = + the same for levels 1 and 2
__global__ __launch_bounds__(64, 2) void k_pyramid_stats(Geo g, const void* __restrict__ feats_v,
                                                         float* __restrict__ part, float* __restrict__ nsum,
                                                         SelState* __restrict__ sel) {
  typedef Row<DT> R;
  constexpr int VEC = R::VEC;
  __shared__ __attribute__((aligned(16))) float tbs[kStageRows * kStageStride];
  __shared__ __attribute__((aligned(16))) float st[kUnitScalars];
  __shared__ typename R::Raw pbuf[CC ? 16 * 64 : 1];  // the partner tile (the same tile of frame t + 1), as loaded
  const int NU = unit_cols(g) * unit_rows(g), lane = threadIdx.x;
  int chunk, u, f;
  if (CC) {
    // With the frame-to-frame dot products a tile is asked for by two workgroups: its own frame's and the one of the
    // frame before. Workgroups go to the eight dies round-robin by their index; each die gets a contiguous range of
    // frames and walks it in order, so the two requests come from the same die within a few microseconds of each
    // other and the second one is served by that die's L2.
    const int per_die = (g.F + 7) / 8, die = blockIdx.x & 7;
    int slot = blockIdx.x >> 3;
    chunk = slot % g.nC;
    slot /= g.nC;
    u = slot % NU;
    const int fl = slot / NU;
    f = die * per_die + fl;
    if (fl >= per_die || f >= g.F) return;
  } else {
    chunk = blockIdx.x;
    u = blockIdx.y;
    f = blockIdx.z;
  }
  const int ch0 = chunk * g.cch + lane * VEC;
  const bool act = ch0 < g.D;
  const int H = g.H, W = g.W, L = g.L;
  const typename R::Elem* fbase =
      reinterpret_cast<const typename R::Elem*>(feats_v) + (size_t)f * g.HW * g.D + (act ? ch0 : 0);
  const int UX = (W + 7) >> 3;  // units per row that hold valid cells
  const int y3 = (u / UX) * 8, x3 = (u % UX) * 8;
  const int vh = min(8, H - y3), vw = min(8, W - x3);  // valid rows / columns of the unit

  const bool has_next = CC && f % g.T != g.T - 1;
  const typename R::Elem* nbase = has_next ? fbase + (size_t)g.HW * g.D : fbase;
  typename R::Raw bufA[16], bufB[16];
  tile_load<DT>(bufA, fbase, W, g.D, y3, x3, min(vh, 4), min(vw, 4));
  if (chunk == 0 && u == 0 && f % g.T == 0) sel_clear(sel + f / g.T);  // this video's budget search starts afresh
  float S3[VEC], S2[4][VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) S3[v] = 0.f;
#pragma unroll
  for (int q2 = 0; q2 < 4; ++q2) {
    const int th = max(0, min(4, vh - (q2 >> 1) * 4)), tw = max(0, min(4, vw - (q2 & 1) * 4));
    const bool some = th > 0 && tw > 0;
    // the tile's own rows are waited for here (nothing newer is in flight at this point); a full tile of a full
    // chunk needs no masking
    const bool ragged = th < 4 || tw < 4 || (chunk + 1) * g.cch > g.D;
    if (some && ragged) tile_mask<DT>((q2 & 1) ? bufB : bufA, th, tw, act);
    if (CC && has_next && some) {
      // the partner tile, with the same clamping as the tile's own loads: sixteen requests, whatever the edge
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int q1 = i >> 2, k = i & 3;
        const int dy = min((q1 >> 1) * 2 + (k >> 1), th - 1), dx = min((q1 & 1) * 2 + (k & 1), tw - 1);
        load_row_to_lds(pbuf, i * 1024,
                        nbase + (size_t)((y3 + (q2 >> 1) * 4 + dy) * W + x3 + (q2 & 1) * 4 + dx) * g.D, lane);
      }
    }
    if (q2 < 3) {
      // the next tile's rows fly while this one is worked on; a tile wholly beyond the edge reads the
      // first tile again instead (nothing is done with it), so that the loads stay unconditional
      const int n = q2 + 1;
      const int nh = max(0, min(4, vh - (n >> 1) * 4)), nw = max(0, min(4, vw - (n & 1) * 4));
      const bool none = nh == 0 || nw == 0;
      tile_load<DT>((q2 & 1) ? bufA : bufB, fbase, W, g.D, none ? y3 : y3 + (n >> 1) * 4,
                    none ? x3 : x3 + (n & 1) * 4, none ? 1 : nh, none ? 1 : nw);
    }
    if (some) {
      float S1[4][VEC];  // the tile's 2x2 block sums
      float b4[8];  // the blocks' dot products with the tile, then (CC = 2) with the same blocks of the next frame
#pragma unroll
      for (int i = 0; i < 8; ++i) b4[i] = 0.f;
      {
        float p1[4];
        tile_stats<DT>((q2 & 1) ? bufB : bufA, tbs, lane, th, tw, p1, S2[q2], S1);
#pragma unroll
        for (int i = 0; i < 4; ++i) b4[i] = p1[i];
      }
      if (CC && has_next) {
        // x_c(t) . x_c(t+1) for the tile's cells: where both frames keep single cells the temporal stage needs
        // nothing else (Sec. 3.3 compares node features; a cell's feature is its own row).
        wait_loads_but(q2 < 3 ? 16 : 0);  // the partner rows are there; the next tile's may still be on their way
        float SN2[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) SN2[v] = 0.f;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          float cd[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) cd[i] = 0.f;
#pragma unroll
          for (int qq = 0; qq < 2; ++qq) {
            const int q1 = h * 2 + qq;
            if ((q1 >> 1) * 2 >= th || (q1 & 1) * 2 >= tw) continue;
            typename R::Raw pr[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              pr[k] = pbuf[(q1 * 4 + k) * 64 + lane];
              if (ragged) {  // (a clamped request repeated another cell; a lane beyond the last channel read channel 0)
                const bool in = (q1 >> 1) * 2 + (k >> 1) < th && (q1 & 1) * 2 + (k & 1) < tw && act;
                if (!in) pr[k] = R::zero();
              }
              cd[qq * 4 + k] = R::dot(((q2 & 1) ? bufB : bufA)[q1 * 4 + k], pr[k]);
            }
            if (CC >= 2) {
              // The same for the tile's 2x2 blocks and for the tile itself: S_n(t) . S_n(t+1), what the temporal
              // stage needs where both frames keep the same node n at level 1 or 2: the block's sum (kept from the
              // tile's statistics) with the sum of the partner block's four rows, the tile's sum with the sum of
              // the partner blocks.
              float SN1[VEC], d1 = 0.f;
#pragma unroll
              for (int v = 0; v < VEC; ++v) SN1[v] = 0.f;
#pragma unroll
              for (int k = 0; k < 4; ++k) R::add_row(pr[k], SN1);
#pragma unroll
              for (int v = 0; v < VEC; ++v) {
                d1 = fmaf(S1[q1][v], SN1[v], d1);
                SN2[v] += SN1[v];
              }
              b4[4 + q1] = d1;
            }
          }
          stage8(tbs, 5 + h, lane, cd);
        }
        if (CC >= 2) {
          float t8[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) t8[i] = 0.f;
#pragma unroll
          for (int v = 0; v < VEC; ++v) t8[0] = fmaf(S2[q2][v], SN2[v], t8[0]);
          stage8(tbs, 7, lane, t8);
        }
      }
      stage8(tbs, 4, lane, b4);
      // row r of the staging area is added up by lane r and goes to its place in the unit's block (zero where the
      // row stands for nothing: beyond the edge, above the root level, no next frame)
      wave_lds_fence();
      if (lane < 57) {
        const int r = lane;
        bool live;
        int dst;
        if (r < 32 || (r >= 40 && r < 56)) {  // a cell's row: norm, dot with its block, or with the next frame
          const int q1 = r < 32 ? r >> 3 : (r - 40) >> 2, k = r & 3;
          live = (q1 >> 1) * 2 + (k >> 1) < th && (q1 & 1) * 2 + (k & 1) < tw;
          if (r < 32 && (r & 4)) live = live && 0 < L;
          if (r >= 40) live = live && has_next;
          dst = r < 32 ? q2 * kTileRows + ((r & 4) ? 16 : 0) + q1 * 4 + k : kUnitCellDots + q2 * 16 + (r - 40);
        } else if (r < 40) {  // a 2x2 block's row: dot with the tile, or with the next frame
          const int q1 = r & 3;
          live = (q1 >> 1) * 2 < th && (q1 & 1) * 2 < tw;
          live = live && (r < 36 ? 1 < L : (CC >= 2 && has_next));
          dst = r < 36 ? q2 * kTileRows + 32 + q1 : kUnitNodeDots + q2 * 8 + q1;
        } else {  // the tile with the next frame's
          live = CC >= 2 && has_next;
          dst = kUnitNodeDots + q2 * 8 + 4;
        }
        st[dst] = live ? staged_row_sum(tbs, r) : 0.f;
      }
      wave_lds_fence();
    } else {
#pragma unroll
      for (int v = 0; v < VEC; ++v) S2[q2][v] = 0.f;
      if (lane < kTileRows) st[q2 * kTileRows + lane] = 0.f;
      if (lane < 16) st[kUnitCellDots + q2 * 16 + lane] = 0.f;
      if (lane < 5) st[kUnitNodeDots + q2 * 8 + lane] = 0.f;
    }
    if (lane >= 5 && lane < 8) st[kUnitNodeDots + q2 * 8 + lane] = 0.f;
#pragma unroll
    for (int v = 0; v < VEC; ++v) S3[v] += S2[q2][v];
  }
  // level-2 dot products of the four tiles with the unit's sum
  if (lane < kUnitCellDots - 4 * kTileRows) st[4 * kTileRows + lane] = 0.f;
  if (L >= 3) {
    float d2[8];
#pragma unroll
    for (int q2 = 0; q2 < 8; ++q2) d2[q2] = 0.f;
#pragma unroll
    for (int q2 = 0; q2 < 4; ++q2) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) d2[q2] = fmaf(S2[q2][v], S3[v], d2[q2]);
    }
    stage8(tbs, 0, lane, d2);
    wave_lds_fence();
    if (lane < 4) {
      const int q2 = lane;
      if ((q2 >> 1) * 4 < vh && (q2 & 1) * 4 < vw) st[4 * kTileRows + q2] = staged_row_sum(tbs, lane);
    }
    wave_lds_fence();
    if (act) {
      float* o = nsum + ((size_t)f * (g.NN - g.lvl_base[3]) + (y3 >> 3) * (g.P >> 3) + (x3 >> 3)) * g.D + ch0;
#pragma unroll
      for (int v = 0; v < VEC; v += 4)
        *reinterpret_cast<float4*>(o + v) = make_float4(S3[v], S3[v + 1], S3[v + 2], S3[v + 3]);
    }
  }
  // the workgroup's scalars leave in one piece: whole, aligned 128-byte lines that no other workgroup touches
  wave_lds_fence();
  if (lane < kUnitScalars / 4)
    reinterpret_cast<float4*>(part + ((size_t)(f * g.nC + chunk) * NU + u) * kUnitScalars)[lane] =
        reinterpret_cast<const float4*>(st)[lane];
}

// ------------------------------------------------------------------------------------------------
// pyramid_upper_node: one node of a level >= 4 of one frame from the stored sums of its children, for one
// chunk, by one wavefront; a lane owns four channels (the chunk is covered in VEC/4 sweeps). Stores the node's
// sum next to the level-3 sums and the partial dot product of every child with it in the same per-chunk
// tables as above. Runs at the head of the finalize kernel, level by level.
// ------------------------------------------------------------------------------------------------
__device__ inline void pyramid_upper_node(const Geo& g, float* partu, float* nsum, int chunk, int f, int lane, int lvl,
                                          int nd) {
  const int NB = g.NN - g.lvl_base[3];
  float* pd = partu + (size_t)(f * g.nC + chunk) * NB;  // indexed by node - first level-3 node
  float* rows = nsum + (size_t)f * NB * g.D;
  const int G = g.P >> lvl;
  const int by = nd / G, bx = nd - by * G;
  if (!node_exists(g, lvl, by, bx)) return;  // wave-uniform
  float tot[4] = {0.f, 0.f, 0.f, 0.f};
  for (int c = lane * 4; c < g.cch; c += 256) {
    const int ch = chunk * g.cch + c;
    if (ch >= g.D) continue;
    float4 a[4];
    float4 S = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int cy = 2 * by + (k >> 1), cx = 2 * bx + (k & 1);
      a[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (node_exists(g, lvl - 1, cy, cx))
        a[k] = *reinterpret_cast<const float4*>(rows + (size_t)(node_index(g, lvl - 1, cy, cx) - g.lvl_base[3]) * g.D + ch);
    }
    S.x = (a[0].x + a[1].x) + (a[2].x + a[3].x);
    S.y = (a[0].y + a[1].y) + (a[2].y + a[3].y);
    S.z = (a[0].z + a[1].z) + (a[2].z + a[3].z);
    S.w = (a[0].w + a[1].w) + (a[2].w + a[3].w);
    *reinterpret_cast<float4*>(rows + (size_t)(node_index(g, lvl, by, bx) - g.lvl_base[3]) * g.D + ch) = S;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      tot[k] = fmaf(a[k].x, S.x, fmaf(a[k].y, S.y, fmaf(a[k].z, S.z, fmaf(a[k].w, S.w, tot[k]))));
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) tot[j] = wave_sum(tot[j]);
  if (lane == 0) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int cy = 2 * by + (k >> 1), cx = 2 * bx + (k & 1);
      if (node_exists(g, lvl - 1, cy, cx)) pd[node_index(g, lvl - 1, cy, cx) - g.lvl_base[3]] = tot[k];
    }
  }
}

template <int CC>
static void launch_pyramid_cc(const Geo& g, const void* feats, float* part, float* nsum, SelState* sel, hipStream_t s) {
  const int NU = unit_cols(g) * unit_rows(g);
  const dim3 grid((unsigned)(8 * ((g.F + 7) / 8) * NU * g.nC)), block(64);
  if (g.dtype == 1)
    hipLaunchKernelGGL((k_pyramid_stats<1, CC>), grid, block, 0, s, g, feats, part, nsum, sel);
  else if (g.dtype == 2)
    hipLaunchKernelGGL((k_pyramid_stats<2, CC>), grid, block, 0, s, g, feats, part, nsum, sel);
  else
    hipLaunchKernelGGL((k_pyramid_stats<0, CC>), grid, block, 0, s, g, feats, part, nsum, sel);
}

void launch_pyramid_stats(const Geo& g, const void* feats, int cell_dots, float* part, float* nsum, SelState* sel,
                          hipStream_t s) {
  if (cell_dots >= 2) {
    launch_pyramid_cc<2>(g, feats, part, nsum, sel, s);
  } else if (cell_dots == 1) {
    launch_pyramid_cc<1>(g, feats, part, nsum, sel, s);
  } else {
    const dim3 grid(g.nC, unit_cols(g) * unit_rows(g), g.F), block(64);
    if (g.dtype == 1)
      hipLaunchKernelGGL((k_pyramid_stats<1, 0>), grid, block, 0, s, g, feats, part, nsum, sel);
    else if (g.dtype == 2)
      hipLaunchKernelGGL((k_pyramid_stats<2, 0>), grid, block, 0, s, g, feats, part, nsum, sel);
    else
      hipLaunchKernelGGL((k_pyramid_stats<0, 0>), grid, block, 0, s, g, feats, part, nsum, sel);
  }
}

// ------------------------------------------------------------------------------------------------
// k_spatial_finalize: one workgroup per frame. First the levels above the 8x8 units (see pyramid_upper_node),
// then it sums the per-chunk partials in chunk order, turns
// them into sigma(parent, child) (Sec. 3.2: cosine between a level's nodes and their children),
// m_n = min over existing children, and the split score s_n = max of m along the path from the root.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void k_spatial_finalize(Geo g, const float* __restrict__ part, float* partu,
                                                          float* __restrict__ nsum,
                                                          float* __restrict__ nrm2, float* __restrict__ sim,
                                                          float* __restrict__ m, uint32_t* __restrict__ sel_key,
                                                          uint8_t* __restrict__ sel_w,
                                                          SelState* __restrict__ sel) {
  STTM_DYNAMIC_LDS(float, sm);
  __shared__ unsigned h0[kSelBins];
  for (int j = threadIdx.x; j < kSelBins; j += blockDim.x) h0[j] = 0;
  float* s_n = sm;
  float* s_sim = sm + g.NN;
  float* s_m = sm + 2 * g.NN;
  const int f = blockIdx.x;
  const size_t fo = (size_t)f * g.NN;
  for (int lvl = 4; lvl <= g.L; ++lvl) {  // the levels above the 8x8 units: one wavefront per (node, chunk)
    const int wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6, side = g.P >> lvl;
    for (int w = wave; w < side * side * g.nC; w += nwaves)
      pyramid_upper_node(g, partu, nsum, w % g.nC, f, threadIdx.x & 63, lvl, w / g.nC);
    __syncthreads();  // sums and dot products written above are read by other wavefronts of this workgroup
  }
  for (int idx = threadIdx.x; idx < g.NN; idx += blockDim.x) {
    int lvl, by, bx;
    node_decode(g, idx, lvl, by, bx);
    float n = 0.f, d = 0.f;
    if (node_exists(g, lvl, by, bx)) {
      // where the first pass (levels 0..2) or the step above (levels >= 3) left this node's partials
      const float* p;
      size_t cstride;  // from one chunk's value to the next
      int dn = 0;      // offset of the squared norm relative to the dot product (cells only)
      if (lvl <= 2) {
        const int y = by << lvl, x = bx << lvl;
        const int NU = unit_cols(g) * unit_rows(g);
        const int q2 = ((y >> 2) & 1) * 2 + ((x >> 2) & 1), q1 = ((y >> 1) & 1) * 2 + ((x >> 1) & 1);
        const int slot = lvl == 2 ? 4 * kTileRows + q2
                                  : q2 * kTileRows + (lvl == 1 ? 32 + q1 : 16 + q1 * 4 + (y & 1) * 2 + (x & 1));
        p = part + ((size_t)f * g.nC * NU + (y >> 3) * unit_cols(g) + (x >> 3)) * kUnitScalars + slot;
        cstride = (size_t)NU * kUnitScalars;
        dn = -16;
      } else {
        const int NB = g.NN - g.lvl_base[3];
        p = partu + (size_t)f * g.nC * NB + (idx - g.lvl_base[3]);
        cstride = NB;
      }
      const bool want_n = lvl == 0, want_d = lvl < g.L;
      for (int c0 = 0; c0 < g.nC; c0 += 8) {  // eight chunks' partials in flight, added in chunk order
        float pn[8], pd[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const bool in = c0 + u < g.nC;
          pn[u] = in && want_n ? p[(size_t)(c0 + u) * cstride + dn] : 0.f;
          pd[u] = in && want_d ? p[(size_t)(c0 + u) * cstride] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          n += pn[u];
          d += pd[u];
        }
      }
    }
    s_n[idx] = n;
    s_sim[idx] = d;  // dot for now
  }
  __syncthreads();
  // squared norm of a node above the cells = sum over its children of (child sum) . (node sum)
  for (int idx = threadIdx.x; idx < g.NN; idx += blockDim.x) {
    int lvl, by, bx;
    node_decode(g, idx, lvl, by, bx);
    float n = s_n[idx];
    if (lvl >= 1) {
      n = 0.f;
      if (node_exists(g, lvl, by, bx))
        for (int k = 0; k < 4; ++k) {
          const int cy = 2 * by + (k >> 1), cx = 2 * bx + (k & 1);
          if (node_exists(g, lvl - 1, cy, cx)) n += s_sim[node_index(g, lvl - 1, cy, cx)];
        }
      s_n[idx] = n;
    }
    nrm2[fo + idx] = n;
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < g.NN; idx += blockDim.x) {
    int lvl, by, bx;
    node_decode(g, idx, lvl, by, bx);
    float v = 0.f;
    if (lvl < g.L && node_exists(g, lvl, by, bx))
      v = cosine_from(s_sim[idx], s_n[idx], s_n[node_index(g, lvl + 1, by >> 1, bx >> 1)]);
    sim[fo + idx] = v;
    s_m[idx] = v;  // reuse as sim storage until the next phase reads it
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < g.NN; idx += blockDim.x) {
    int lvl, by, bx;
    node_decode(g, idx, lvl, by, bx);
    float mv = 2.f;
    if (lvl >= 1 && node_exists(g, lvl, by, bx)) {
      bool nan = false;
      for (int k = 0; k < 4; ++k) {
        const int cy = 2 * by + (k >> 1), cx = 2 * bx + (k & 1);
        if (!node_exists(g, lvl - 1, cy, cx)) continue;
        const float v = s_m[node_index(g, lvl - 1, cy, cx)];
        if (v != v) nan = true;
        mv = fminf(mv, v);
      }
      if (nan) mv = __uint_as_float(0x7fc00000u);
    }
    s_sim[idx] = mv;  // m in LDS
    m[fo + idx] = mv;
  }
  __syncthreads();
  for (int i0 = 0; i0 < g.NN; i0 += blockDim.x) {  // uniform trip count: the histogram update is wave-wide
    const int idx = i0 + threadIdx.x;
    uint32_t key = 0;
    unsigned wgt = 0;
    if (idx < g.NN) {
      int lvl, by, bx;
      node_decode(g, idx, lvl, by, bx);
      float s = -2.f;
      if (lvl >= 1 && node_exists(g, lvl, by, bx)) {
        int l = lvl, y = by, x = bx;
        while (true) {
          const float v = s_sim[node_index(g, l, y, x)];
          s = fmaxf(s, (v != v) ? -2.f : v);  // NaN always splits
          if (l == g.L) break;
          ++l; y >>= 1; x >>= 1;
        }
      }
      // compact (value, weight) element of the budget search: upper-level nodes with >= 2 children
      if (lvl >= 1) {
        int kids = 0;
        if (node_exists(g, lvl, by, bx))
          for (int k = 0; k < 4; ++k) kids += node_exists(g, lvl - 1, 2 * by + (k >> 1), 2 * bx + (k & 1));
        const size_t o = (size_t)f * (g.NN - g.lvl_base[1]) + (idx - g.lvl_base[1]);
        if (kids >= 2) { key = float_key(s); wgt = (unsigned)(kids - 1); }
        sel_key[o] = key;
        sel_w[o] = (uint8_t)wgt;
      }
    }
    wave_hist_add(h0, wgt != 0, key >> 21, wgt);
  }
  __syncthreads();
  sel_flush_level0(sel + f / g.T, h0);
}

void launch_spatial_finalize(const Geo& g, const float* part, float* partu, float* nsum, float* nrm2, float* sim,
                             float* m, uint32_t* sel_key, uint8_t* sel_w, SelState* sel, hipStream_t s) {
  const int threads = g.NN <= 256 ? 256 : 512;  // one node per thread where it fits; more workgroups per CU beyond
  hipLaunchKernelGGL(k_spatial_finalize, dim3(g.F), dim3(threads), 3 * g.NN * sizeof(float), s, g, part, partu, nsum, nrm2,
                     sim,
                     m, sel_key, sel_w, sel);
}

// ------------------------------------------------------------------------------------------------
// k_spatial_decide: coarse-to-fine search (Sec. 3.2). Grid (cells of a video / 256, videos); one thread per cell
// walks down from its root: the first node on the path whose smallest child similarity exceeds tau_S is kept.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void k_spatial_decide(Geo g, const float* __restrict__ m,
                                                                float* __restrict__ tau,
                                                                const SelState* __restrict__ pending,
                                                                int32_t* __restrict__ node_map,
                                                                uint8_t* __restrict__ node_level) {
  const int b = blockIdx.y, per_video = g.T * g.HW;
  float t;
  if (pending) {  // the budget search left its last digit to this kernel
    t = sel_last_digit(pending + b);
    if (blockIdx.x == 0 && threadIdx.x == 0) tau[b] = t;
  } else {
    t = tau[b];
  }
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= per_video) return;
  const int i = b * per_video + j;
  const int f = i / g.HW, c = i - f * g.HW;
  const int y = c / g.W, x = c - y * g.W;
  const float* mf = m + (size_t)f * g.NN;
  int lvl = g.L;
  for (; lvl >= 1; --lvl)
    if (mf[node_index(g, lvl, y >> lvl, x >> lvl)] > t) break;
  const int y0 = (y >> lvl) << lvl, x0 = (x >> lvl) << lvl;
  node_map[i] = f * g.HW + y0 * g.W + x0;
  if (node_level) node_level[i] = (uint8_t)lvl;
}

void launch_spatial_decide(const Geo& g, const float* m, float* tau, const SelState* pending, int32_t* node_map,
                           uint8_t* node_level, hipStream_t s) {
  const int per_video = g.T * g.HW;
  hipLaunchKernelGGL(k_spatial_decide, dim3((per_video + kSelThreads - 1) / kSelThreads, g.B), dim3(kSelThreads), 0, s,
                     g, m, tau, pending, node_map, node_level);
}

// Recovers node levels from a node map (callers may pass node_level == NULL to the temporal stage).
__global__ __launch_bounds__(256) void k_node_levels(Geo g, const int32_t* __restrict__ node_map,
                                                     uint8_t* __restrict__ node_level) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= g.N) return;
  const int f = i / g.HW, c = i - f * g.HW;
  const int y = c / g.W, x = c - y * g.W;
  const int r = node_map[i] - f * g.HW;
  const int y0 = r / g.W, x0 = r - y0 * g.W;
  // smallest level whose block at (y0, x0) contains (y, x) and is aligned; the partition's block is
  // the largest aligned block rooted at (y0,x0) in which every valid cell maps to it -- found by growing.
  int lvl = 0;
  while (lvl < g.L) {
    const int s2 = 2 << lvl;
    if ((y0 & (s2 - 1)) || (x0 & (s2 - 1))) break;
    // the candidate block [y0, y0+s2) x [x0, x0+s2): its bottom-right valid corner must map to r as well
    const int yy = min(y0 + s2 - 1, g.H - 1), xx = min(x0 + s2 - 1, g.W - 1);
    if (node_map[f * g.HW + yy * g.W + xx] - f * g.HW != r) break;
    ++lvl;
  }
  (void)y; (void)x;
  node_level[i] = (uint8_t)lvl;
}

void launch_node_levels(const Geo& g, const int32_t* node_map, uint8_t* node_level, hipStream_t s) {
  hipLaunchKernelGGL(k_node_levels, dim3((g.N + 255) / 256), dim3(256), 0, s, g, node_map, node_level);
}

// ------------------------------------------------------------------------------------------------
// Budget-driven thresholds. Token count as a function of the threshold is the step function
// K(tau) = base + sum_j w_j [v_j <= tau]. An MSB-first radix select (11 + 11 + 10 bits) over the
// order-preserving integer image of v finds the smallest value whose cumulative weight exceeds
// target - base, then the largest value below it; tau is the midpoint of the two.
// The level-0 histogram is filled by the statistics pass of the stage; two launches follow, grid
// (slices, videos): every workgroup finds the next digit from the (complete) histogram of the level before
// and bins its slice under the prefix (the second also collects the largest key below the prefix); a last
// small launch resolves the last digit and writes tau. Each launch leaves what it found in the state, so the
// next one resolves one digit only.
// Input: keys[video][per_video] (0 = not an element), weights (NULL = 1 for every element).
// ------------------------------------------------------------------------------------------------
constexpr int kSelPer = 8;   // elements per thread and pass

__device__ inline int sel_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ inline int sel_width(int pass) { return pass == 2 ? 10 : 11; }

// base of the step function: spatial = constant (roots * T), temporal = kept nodes of the video's first frame
__device__ inline int sel_base(const Geo& g, int b, int base_const, const int32_t* node_map) {
  if (!node_map) return base_const;
  __shared__ int s_base;
  if (threadIdx.x == 0) s_base = 0;
  __syncthreads();
  int c = 0;
  for (int j = threadIdx.x; j < g.HW; j += blockDim.x) {
    const int i = b * g.T * g.HW + j;
    c += (node_map[i] == i);
  }
  if (c) atomicAdd(&s_base, c);
  __syncthreads();
  const int r = s_base;
  __syncthreads();
  return r;
}

// Clears what a search leaves behind (levels 1-2, the lower neighbour); level 0 stays.
__global__ __launch_bounds__(256) void k_select_reset(SelState* st) {
  SelState* s = st + blockIdx.x;
  for (int j = threadIdx.x; j < kSelBins; j += blockDim.x) s->hist[0][j] = s->hist[1][j] = 0;
  if (threadIdx.x == 0) s->lo_out = 0;
}

// One digit of the search per launch, grid (slices, videos). Every workgroup finds the digit of level
// PASS - 1 from that level's (complete) histogram -- the first launch also works out the budget, the second
// starts from what the first one left in the state -- and bins its slice of the keys under the prefix found
// so far; the workgroup of slice 0 leaves the prefix for the next launch.
template <int PASS>  // 1 or 2
__global__ __launch_bounds__(kSelThreads) void k_select_pass(Geo g, const uint32_t* __restrict__ keys,
                                                             const uint8_t* __restrict__ weights, int per_video,
                                                             const int* __restrict__ target, int base_const,
                                                             const int32_t* __restrict__ node_map,
                                                             SelState* __restrict__ states) {
  __shared__ unsigned hist[kSelBins];
  const int b = blockIdx.y, tid = threadIdx.x;
  SelState* st = states + b;
  // the slice's keys do not depend on the search: their loads fly while the digit is being found
  const uint32_t* kv = keys + (size_t)b * per_video;
  const uint8_t* wv = weights ? weights + (size_t)b * per_video : nullptr;
  const int j0 = blockIdx.x * (kSelThreads * kSelPer);
  uint32_t key[kSelPer];
  unsigned w[kSelPer];
#pragma unroll
  for (int u = 0; u < kSelPer; ++u) {
    const int j = j0 + u * kSelThreads + tid;
    key[u] = j < per_video ? kv[j] : 0u;
    w[u] = 1u;
    if (wv) w[u] = j < per_video ? wv[j] : 0u;
  }
  for (int j = tid; j < kSelBins; j += kSelThreads) hist[j] = 0;
  SelFound fd;
  if (PASS == 1) {
    const int base = sel_base(g, b, base_const, node_map);
    const long long budget = (long long)target[b] - base;
    fd.budget = budget < 0 ? 0ull : (unsigned long long)budget;
    fd.acc = 0;
    fd.prefix = 0;
    fd.rc = budget < 0 ? 2 : 0;
  } else {
    fd = st->found[0];
  }
  if (fd.rc == 0) {  // uniform over the workgroup
    unsigned d;
    unsigned long long a2;
    const bool hit = PASS == 1 ? sel_pick<kSelCopies>(st->hist0[0], fd.acc, fd.budget, &d, &a2, nullptr)
                               : sel_pick<1>(st->hist[0], fd.acc, fd.budget, &d, &a2, nullptr);
    if (hit) {
      fd.prefix = (fd.prefix << sel_width(PASS - 1)) | d;
      fd.acc = a2;
    } else {
      fd.rc = 1;
    }
  }
  if (blockIdx.x == 0 && tid == 0) st->found[PASS - 1] = fd;
  __syncthreads();  // the LDS histogram is clear
  if (fd.rc == 0) {
    const unsigned prefix = fd.prefix;
    const int shift = sel_shift(PASS), width = sel_width(PASS);
    unsigned lo = 0;  // key 0 is below every real value
#pragma unroll
    for (int u = 0; u < kSelPer; ++u) {
      if (w[u] == 0) key[u] = 0;
      const unsigned top = key[u] >> (shift + width);
      const bool valid = key[u] != 0 && top == prefix;
      wave_hist_add(hist, valid, (key[u] >> shift) & ((1u << width) - 1u), w[u]);
      if (PASS == 2 && key[u] != 0 && top < prefix && key[u] > lo) lo = key[u];
    }
    if (PASS == 2) {
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) lo = max(lo, (unsigned)__shfl_xor((int)lo, o, 64));
      if ((tid & 63) == 0 && lo) atomicMax(&st->lo_out, lo);
    }
    __syncthreads();
    for (int j = tid; j < kSelBins; j += kSelThreads)
      if (hist[j]) atomicAdd(&st->hist[PASS - 1][j], hist[j]);
  }
}

// Last digit as a launch of its own (when the caller wants the threshold back).
__global__ __launch_bounds__(kSelThreads) void k_select_tau(const SelState* __restrict__ states,
                                                            float* __restrict__ tau) {
  const float t = sel_last_digit(states + blockIdx.x);
  if (threadIdx.x == 0) tau[blockIdx.x] = t;
}

static void launch_select(const Geo& g, const uint32_t* keys, const uint8_t* weights, int per_video,
                          const int* target, int base_const, const int32_t* node_map, SelState* st, bool dirty,
                          float* tau, hipStream_t s) {
  const int slices = per_video > 0 ? (per_video + kSelThreads * kSelPer - 1) / (kSelThreads * kSelPer) : 1;
  const dim3 grid(slices, g.B), block(kSelThreads);
  if (dirty) hipLaunchKernelGGL(k_select_reset, dim3(g.B), dim3(256), 0, s, st);
  hipLaunchKernelGGL(k_select_pass<1>, grid, block, 0, s, g, keys, weights, per_video, target, base_const,
                     node_map, st);
  hipLaunchKernelGGL(k_select_pass<2>, grid, block, 0, s, g, keys, weights, per_video, target, base_const,
                     node_map, st);
  if (tau) hipLaunchKernelGGL(k_select_tau, dim3(g.B), block, 0, s, st, tau);
}

void launch_select_spatial(const Geo& g, const uint32_t* keys, const uint8_t* weights, const int* target,
                           SelState* state, bool dirty, float* tau, hipStream_t s) {
  int roots = 0;
  for (int ry = 0; ry < g.R; ++ry)
    for (int rx = 0; rx < g.R; ++rx) roots += node_exists(g, g.L, ry, rx);
  const int per_video = g.T * (g.NN - g.lvl_base[1]);
  launch_select(g, keys, weights, per_video, target, roots * g.T, nullptr, state, dirty, tau, s);
}

void launch_select_temporal(const Geo& g, const int32_t* node_map, const uint32_t* keys, const int* target,
                            SelState* state, bool dirty, float* tau, hipStream_t s) {
  launch_select(g, keys, nullptr, g.T * g.HW, target, 0, node_map, state, dirty, tau, s);
}

}  // namespace sttm
