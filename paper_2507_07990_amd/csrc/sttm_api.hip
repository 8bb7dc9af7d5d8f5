// C ABI of libsttm: argument checking, workspace layout, stage ordering. See include/sttm.h.
#include "sttm_dev.h"
#include "../../include/sttm.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace sttm;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  size_t part, partu, nsum, nrm2, sim, m, sel_key_s, sel_w_s, sel_key_t, tau_s, tau_t, target_s, target_t, sel_s, sel_t, lvl,
      titems, tcount, pd_part, sig, e, parent, ptr_a, ptr_b;
  size_t rank, key_a, val_a, key_b, val_b, order, orow, hist, tot, gsum, tile_roots, tile_live, seg, kdev,
      bigpart, bigw, biglist, zpos, possum, poscnt;
  size_t total;
};

bool make_geo(int B, int T, int H, int W, int D, int dtype, int root_grid, Geo* g) {
  if (B < 1 || T < 1 || H < 1 || W < 1 || D < 8 || H > 32 || W > 32 || (D % 8) != 0) return false;
  if (dtype != STTM_F32 && dtype != STTM_BF16 && dtype != STTM_F16) return false;
  long long n = (long long)B * T * H * W;
  if (n >= (1ll << 31) - 1) return false;
  if ((long long)B * T > 65535) return false;  // frames index a grid dimension
  int P = 1;
  while (P < (H > W ? H : W)) P *= 2;
  if (root_grid < 1 || (root_grid & (root_grid - 1)) || root_grid > P) return false;
  int L = 0;
  while ((root_grid << L) < P) ++L;
  g->B = B; g->T = T; g->H = H; g->W = W; g->D = D;
  g->P = P; g->L = L; g->R = root_grid; g->HW = H * W; g->F = B * T;
  int base = 0;
  for (int l = 0; l <= kMaxLevels; ++l) {
    g->lvl_base[l] = base;
    if (l <= L) base += (P >> l) * (P >> l);
  }
  g->NN = base;
  g->dtype = dtype;
  g->vec = dtype == STTM_F32 ? 4 : 8;
  g->cch = 64 * g->vec;
  g->nC = (D + g->cch - 1) / g->cch;
  g->N = (int)n;
  return true;
}

// The tables of the reduce stage (ranks, sort buffers, member lists, partial sums of large clusters), laid out
// from byte `off` on; returns the first byte after them.
size_t layout_reduce(const Geo& g, size_t off, Layout* lp) {
  Layout& l = *lp;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  const size_t N = g.N;
  l.rank = take(N * sizeof(int32_t));
  l.key_a = take(N * sizeof(int32_t));
  l.val_a = take(N * sizeof(int32_t));
  l.key_b = take(N * sizeof(int32_t));
  l.val_b = take(N * sizeof(int32_t));
  l.order = take(N * sizeof(int32_t));
  l.orow = take(N * sizeof(int32_t));
  l.hist = take(reduce_hist_entries(g.N) * sizeof(int32_t));
  l.tot = take(2048 * sizeof(int32_t));
  l.gsum = take(reduce_gsum_entries() * sizeof(int32_t));
  l.tile_roots = take(reduce_tiles(g.N) * sizeof(int32_t));
  l.tile_live = take(reduce_tiles(g.N) * sizeof(int32_t));
  l.seg = take((N + 1) * sizeof(int32_t));
  l.kdev = take(4 * sizeof(int32_t));
  l.bigpart = take(reduce_bigpart_floats(g) * sizeof(float));
  l.bigw = take(reduce_bigw_entries(g) * sizeof(int32_t));
  l.biglist = take(reduce_biglist_entries(g) * 4 * sizeof(int32_t));
  l.zpos = take(N * sizeof(int32_t));
  return off;
}

Layout make_layout(const Geo& g) {
  Layout l;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  const size_t F = g.F, NN = g.NN, N = g.N;
  l.part = take(F * g.nC * unit_cols(g) * unit_rows(g) * kUnitScalars * sizeof(float));
  l.partu = take(F * g.nC * nsum_nodes(g) * sizeof(float));
  l.nsum = take(F * nsum_nodes(g) * g.D * sizeof(float));
  l.nrm2 = take(F * NN * sizeof(float));
  l.sim = take(F * NN * sizeof(float));
  l.m = take(F * NN * sizeof(float));
  l.sel_key_s = take(F * (NN - g.lvl_base[1]) * sizeof(uint32_t) + 4);
  l.sel_w_s = take(F * (NN - g.lvl_base[1]) + 4);
  l.sel_key_t = take(N * sizeof(uint32_t));
  l.tau_s = take(g.B * sizeof(float));
  l.tau_t = take(g.B * sizeof(float));
  l.target_s = take(g.B * sizeof(int));
  l.target_t = take(g.B * sizeof(int));
  l.sel_s = take(select_state_bytes(g.B));
  l.sel_t = take(select_state_bytes(g.B));
  l.lvl = take(N);
  l.titems = take(temporal_items_bytes(g));
  l.tcount = take(temporal_count_bytes());
  l.pd_part = take(F * g.nC * g.HW * sizeof(float));
  l.sig = take(N * sizeof(float));
  l.e = take(N * sizeof(float));
  l.parent = take(N * sizeof(int32_t));
  l.ptr_a = take(N * sizeof(int32_t));
  l.ptr_b = take(N * sizeof(int32_t));
  off = layout_reduce(g, off, &l);
  l.possum = take(N * sizeof(unsigned long long));
  l.poscnt = take(N * sizeof(unsigned));
  l.total = off;
  return l;
}

}  // namespace

// Scratch memory of sttm_reduce_noalloc: a fixed array in the library's device image, so that the call needs no
// allocation and no caller-provided workspace. Every device the library is loaded on holds its own copy; the
// array's name is only a handle on the host, its device address is looked up once per device (see sttm_create).
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on every device seen so far

// Device address of the static scratch array on `device` (which must be the current device), or NULL on failure.
void* static_scratch_on(int device, hipError_t* err) {
  *err = hipSuccess;
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    g_scratch_ptr[device] = p;
  }
  return g_scratch_ptr[device];
}
}  // namespace

struct sttm_ctx {
  int device = 0;
  char* static_scratch = nullptr;  // this device's copy of the static scratch array
  hipStream_t stream = nullptr;
  char* ws = nullptr;
  size_t ws_bytes = 0;
  bool bound = false;
  Geo g{};
  Layout lay{};
  bool have_spatial = false, have_tau_s = false, have_temporal = false, have_tau_t = false;
  bool tau_s_pending = false, tau_t_pending = false;  // the budget search left its last digit to the consumer kernel
  int match_mode = STTM_MATCH_FIRST_PASSING, order = STTM_ORDER_RASTER;
  int cell_dots = 1;       // setting: the spatial pass also emits frame-to-frame dot products (0 no, 1 cells, 2 + 2x2 / 4x4 blocks)
  int have_cell_dots = 0;  // what the statistics in the workspace were computed with
  const int32_t* cluster_ids_reduced = nullptr;  // cluster ids of the last reduce call (NULL: none since the shape was bound)
  bool reduced_zscan = false;
  const void* feats_spatial = nullptr;
  const int32_t* node_map_temporal = nullptr;  // caller's node map of the last temporal statistics pass
  std::vector<float> h_tau_s, h_tau_t;         // host staging that outlives the asynchronous uploads
  std::vector<int> h_target_s, h_target_t;
  bool target_s_on_device = false, target_t_on_device = false;  // the device copy equals the host staging
  bool sel_s_dirty = false, sel_t_dirty = false;                // searched since the statistics pass
  std::string err;
  // optional per-kernel timing of the three feature passes (HIP events on the context's stream)
  int profiling = 0;  // 0 = off, n = every n-th launch of each feature kernel is bracketed by events
  size_t prof_seen[STTM_KERNEL_COUNT] = {0, 0, 0};
  struct EvPair { hipEvent_t a, b; };
  std::vector<EvPair> ev[STTM_KERNEL_COUNT];
  size_t ev_used[STTM_KERNEL_COUNT] = {0, 0, 0};
};

namespace {

// The reduce stage's tables inside a buffer laid out by layout_reduce().
ReduceBuffers reduce_buffers(char* base, const Layout& l) {
  ReduceBuffers rb;
  auto i32 = [&](size_t off) { return reinterpret_cast<int32_t*>(base + off); };
  rb.rank = i32(l.rank);
  rb.key_a = i32(l.key_a);
  rb.val_a = i32(l.val_a);
  rb.key_b = i32(l.key_b);
  rb.val_b = i32(l.val_b);
  rb.order = i32(l.order);
  rb.orow = i32(l.orow);
  rb.hist = i32(l.hist);
  rb.tot = i32(l.tot);
  rb.gsum = i32(l.gsum);
  rb.tile_roots = i32(l.tile_roots);
  rb.tile_live = i32(l.tile_live);
  rb.seg = i32(l.seg);
  rb.kdev = i32(l.kdev);
  rb.bigpart = reinterpret_cast<float*>(base + l.bigpart);
  rb.bigw = i32(l.bigw);
  rb.biglist = i32(l.biglist);
  rb.zpos = i32(l.zpos);
  return rb;
}

int fail(sttm_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  return code;
}

int hip_check(sttm_ctx* c, hipError_t e, const char* what) {
  if (e == hipSuccess) return STTM_OK;
  return fail(c, STTM_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define STTM_HIP(c, call)                                   \
  do {                                                      \
    int rc_ = hip_check((c), (call), #call);                \
    if (rc_ != STTM_OK) return rc_;                         \
  } while (0)

template <class T> T* at(sttm_ctx* c, size_t off) { return reinterpret_cast<T*>(c->ws + off); }

int bind_shape(sttm_ctx* c, int dtype, int B, int T, int H, int W, int D, int root_grid) {
  if (dtype != STTM_F32 && dtype != STTM_BF16 && dtype != STTM_F16)
    return fail(c, STTM_ERR_DTYPE, "dtype must be STTM_F32, STTM_BF16 or STTM_F16");
  Geo g;
  std::memset(&g, 0, sizeof g);
  if (!make_geo(B, T, H, W, D, dtype, root_grid, &g))
    return fail(c, STTM_ERR_SHAPE,
                "need B,T >= 1, B*T <= 65535, 1 <= H,W <= 32, D % 8 == 0, B*T*H*W < 2^31, root_grid a power of two <= P");
  Layout l = make_layout(g);
  if (!c->ws) return fail(c, STTM_ERR_WORKSPACE, "no workspace set (sttm_set_workspace)");
  if (c->ws_bytes < l.total) {
    char buf[160];
    snprintf(buf, sizeof buf, "workspace too small: have %zu bytes, need %zu", c->ws_bytes, l.total);
    return fail(c, STTM_ERR_WORKSPACE, buf);
  }
  const bool same = c->bound && std::memcmp(&c->g, &g, sizeof g) == 0;
  c->g = g;
  c->lay = l;
  c->bound = true;
  c->have_spatial = c->have_tau_s = c->have_temporal = c->have_tau_t = false;
  c->tau_s_pending = c->tau_t_pending = false;
  c->cluster_ids_reduced = nullptr;
  if (!same) {
    c->target_s_on_device = c->target_t_on_device = false;  // the layout moved: upload targets again
    // the work queue of the temporal pass starts empty (afterwards every pass leaves it empty behind itself)
    STTM_HIP(c, hipMemsetAsync(at<int>(c, c->lay.tcount), 0, temporal_count_bytes(), c->stream));
  }
  return STTM_OK;
}

bool same_shape(const Geo& g, int dtype, int B, int T, int H, int W, int D, int root_grid) {
  return g.dtype == dtype && g.B == B && g.T == T && g.H == H && g.W == W && g.D == D && g.R == root_grid;
}

int upload_tau(sttm_ctx* c, const float* host, float* dev, std::vector<float>* staging) {
  for (int b = 0; b < c->g.B; ++b)
    if (host[b] != host[b]) return fail(c, STTM_ERR_ARG, "threshold is NaN");
  staging->assign(host, host + c->g.B);
  STTM_HIP(c, hipMemcpyAsync(dev, staging->data(), c->g.B * sizeof(float), hipMemcpyHostToDevice, c->stream));
  return STTM_OK;
}

// Brackets one feature kernel with two events when profiling is on.
struct Timed {
  sttm_ctx* c;
  int kid;
  sttm_ctx::EvPair* p = nullptr;
  Timed(sttm_ctx* c_, int kid_) : c(c_), kid(kid_) {
    if (!c->profiling || (c->prof_seen[kid]++ % (size_t)c->profiling) != 0) return;
    if (c->ev_used[kid] == c->ev[kid].size()) {
      sttm_ctx::EvPair n;
      if (hipEventCreate(&n.a) != hipSuccess || hipEventCreate(&n.b) != hipSuccess) return;
      c->ev[kid].push_back(n);
    }
    p = &c->ev[kid][c->ev_used[kid]++];
    (void)hipEventRecord(p->a, c->stream);
  }
  ~Timed() {
    if (p) (void)hipEventRecord(p->b, c->stream);
  }
};

int after_launch(sttm_ctx* c) { return hip_check(c, hipGetLastError(), "kernel launch"); }

int run_spatial_stats(sttm_ctx* c, const void* feats) {
  {
    Timed t(c, STTM_KERNEL_PYRAMID_STATS);
    launch_pyramid_stats(c->g, feats, c->g.T > 1 ? c->cell_dots : 0, at<float>(c, c->lay.part),
                         at<float>(c, c->lay.nsum), at<SelState>(c, c->lay.sel_s), c->stream);
  }
  launch_spatial_finalize(c->g, at<float>(c, c->lay.part), at<float>(c, c->lay.partu), at<float>(c, c->lay.nsum),
                          at<float>(c, c->lay.nrm2),
                          at<float>(c, c->lay.sim),
                          at<float>(c, c->lay.m), at<uint32_t>(c, c->lay.sel_key_s), at<uint8_t>(c, c->lay.sel_w_s),
                          at<SelState>(c, c->lay.sel_s), c->stream);
  int rc = after_launch(c);
  if (rc == STTM_OK) {
    c->sel_s_dirty = false;
    c->have_spatial = true;
    c->have_temporal = false;
    c->feats_spatial = feats;
    c->have_cell_dots = c->g.T > 1 ? c->cell_dots : 0;
  }
  return rc;
}

int run_temporal_stats(sttm_ctx* c, const void* feats, const int32_t* node_map, const uint8_t* node_level) {
  {
    Timed t(c, STTM_KERNEL_TEMPORAL_DOTS);
    launch_temporal_dots(c->g, feats, node_level, at<float>(c, c->lay.nsum), c->have_cell_dots,
                         at<float>(c, c->lay.pd_part), at<SelState>(c, c->lay.sel_t), at<char>(c, c->lay.titems),
                         at<int>(c, c->lay.tcount), c->stream);
  }
  launch_temporal_resolve(c->g, c->match_mode, c->have_cell_dots == 2 ? 2 : 0, node_map, node_level,
                          at<float>(c, c->lay.pd_part),
                          c->have_cell_dots ? at<float>(c, c->lay.part) : nullptr, at<float>(c, c->lay.nrm2),
                          at<float>(c, c->lay.sig), at<float>(c, c->lay.e), at<uint32_t>(c, c->lay.sel_key_t),
                          at<SelState>(c, c->lay.sel_t), at<int>(c, c->lay.tcount), c->stream);
  int rc = after_launch(c);
  // the search state of the temporal budget starts afresh with these statistics: a threshold chosen from the
  // statistics before them (or a last digit still pending) no longer applies
  c->have_tau_t = c->tau_t_pending = false;
  if (rc == STTM_OK) {
    c->sel_t_dirty = false;
    c->have_temporal = true;
    c->node_map_temporal = node_map;
  }
  return rc;
}

int check_feats(sttm_ctx* c, const void* feats) {
  if (!feats) return fail(c, STTM_ERR_NULL, "feats is NULL");
  if (reinterpret_cast<uintptr_t>(feats) & 15) return fail(c, STTM_ERR_ARG, "feats must be 16-byte aligned");
  return STTM_OK;
}

}  // namespace

extern "C" {

int sttm_create(sttm_ctx** out, int device, void* hip_stream) {
  if (!out) return STTM_ERR_NULL;
  *out = nullptr;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return STTM_ERR_HIP;
  sttm_ctx* c = new (std::nothrow) sttm_ctx();
  if (!c) return STTM_ERR_HIP;
  c->device = device;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  c->err.reserve(256);  // so that short messages need no allocation later
  hipError_t e = hipSetDevice(device);
  if (e == hipSuccess) c->static_scratch = static_cast<char*>(static_scratch_on(device, &e));
  if (e != hipSuccess || !c->static_scratch) {
    delete c;
    return STTM_ERR_HIP;
  }
  *out = c;
  return STTM_OK;
}

int sttm_destroy(sttm_ctx* ctx) {
  if (ctx)
    for (auto& v : ctx->ev)
      for (auto& p : v) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  delete ctx;
  return STTM_OK;
}

const char* sttm_last_error(const sttm_ctx* ctx) {
  if (!ctx) return "null context";
  return ctx->err.c_str();
}

int sttm_nodes_per_frame(int H, int W, int root_grid) {
  Geo g;
  if (!make_geo(1, 1, H, W, 8, STTM_F32, root_grid, &g)) return 0;
  return g.NN;
}

int sttm_node_index(int H, int W, int root_grid, int level, int by, int bx) {
  Geo g;
  if (!make_geo(1, 1, H, W, 8, STTM_F32, root_grid, &g)) return -1;
  if (level < 0 || level > g.L) return -1;
  const int side = g.P >> level;
  if (by < 0 || bx < 0 || by >= side || bx >= side) return -1;
  return node_index(g, level, by, bx);
}

size_t sttm_workspace_bytes(int B, int T, int H, int W, int D, int dtype, int root_grid) {
  Geo g;
  if (!make_geo(B, T, H, W, D, dtype, root_grid, &g)) return 0;
  return make_layout(g).total;
}

int sttm_set_workspace(sttm_ctx* ctx, void* workspace_dev, size_t bytes) {
  if (!ctx) return STTM_ERR_NULL;
  if (!workspace_dev && bytes) return fail(ctx, STTM_ERR_NULL, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(workspace_dev) & (kAlign - 1))
    return fail(ctx, STTM_ERR_ARG, "workspace must be 256-byte aligned");
  ctx->ws = static_cast<char*>(workspace_dev);
  ctx->ws_bytes = bytes;
  ctx->bound = false;
  ctx->have_spatial = ctx->have_tau_s = ctx->have_temporal = ctx->have_tau_t = false;
  ctx->cluster_ids_reduced = nullptr;
  return STTM_OK;
}

int sttm_invalidate(sttm_ctx* ctx) {
  if (!ctx) return STTM_ERR_NULL;
  ctx->have_spatial = ctx->have_tau_s = ctx->have_temporal = ctx->have_tau_t = false;
  ctx->tau_s_pending = ctx->tau_t_pending = false;
  ctx->have_cell_dots = 0;
  ctx->feats_spatial = nullptr;
  ctx->node_map_temporal = nullptr;
  ctx->cluster_ids_reduced = nullptr;
  return STTM_OK;
}

int sttm_set_match_mode(sttm_ctx* ctx, int mode) {
  if (!ctx) return STTM_ERR_NULL;
  if (mode != STTM_MATCH_FIRST_PASSING && mode != STTM_MATCH_TOPLEFT_ONLY && mode != STTM_MATCH_MOST_SIMILAR)
    return fail(ctx, STTM_ERR_ARG, "unknown match mode");
  if (mode != ctx->match_mode) ctx->have_temporal = ctx->have_tau_t = false;  // e_n depends on the rule
  ctx->match_mode = mode;
  return STTM_OK;
}

int sttm_set_cell_dots(sttm_ctx* ctx, int on) {
  if (!ctx) return STTM_ERR_NULL;
  if (on < 0 || on > 2) return fail(ctx, STTM_ERR_ARG, "cell dots: 0, 1 or 2");
  ctx->cell_dots = on;  // takes effect with the next spatial statistics pass
  return STTM_OK;
}

int sttm_set_output_order(sttm_ctx* ctx, int order) {
  if (!ctx) return STTM_ERR_NULL;
  if (order != STTM_ORDER_RASTER && order != STTM_ORDER_ZSCAN) return fail(ctx, STTM_ERR_ARG, "unknown output order");
  ctx->order = order;
  return STTM_OK;
}

int sttm_spatial_stats(sttm_ctx* ctx, const void* feats_dev, int dtype, int B, int T, int H, int W, int D,
                       int root_grid) {
  if (!ctx) return STTM_ERR_NULL;
  int rc = check_feats(ctx, feats_dev);
  if (rc) return rc;
  STTM_HIP(ctx, hipSetDevice(ctx->device));
  rc = bind_shape(ctx, dtype, B, T, H, W, D, root_grid);
  if (rc) return rc;
  return run_spatial_stats(ctx, feats_dev);
}

int sttm_spatial_quadtree(sttm_ctx* ctx, const void* feats_dev, int dtype, int B, int T, int H, int W, int D,
                          int root_grid, const float* tau_s_host, int32_t* node_map_dev,
                          uint8_t* node_level_dev) {
  if (!ctx) return STTM_ERR_NULL;
  if (!node_map_dev) return fail(ctx, STTM_ERR_NULL, "node_map is NULL");
  STTM_HIP(ctx, hipSetDevice(ctx->device));
  int rc;
  if (tau_s_host) {
    rc = check_feats(ctx, feats_dev);
    if (rc) return rc;
    rc = bind_shape(ctx, dtype, B, T, H, W, D, root_grid);
    if (rc) return rc;
    rc = upload_tau(ctx, tau_s_host, at<float>(ctx, ctx->lay.tau_s), &ctx->h_tau_s);
    if (rc) return rc;
    ctx->have_tau_s = true;
    ctx->tau_s_pending = false;
    rc = run_spatial_stats(ctx, feats_dev);
    if (rc) return rc;
  } else {
    if (!ctx->bound || !ctx->have_spatial)
      return fail(ctx, STTM_ERR_STATE, "no spatial statistics in the workspace (call sttm_spatial_stats first)");
    if (!same_shape(ctx->g, dtype, B, T, H, W, D, root_grid))
      return fail(ctx, STTM_ERR_SHAPE, "shape differs from the one the statistics were computed for");
    if (!ctx->have_tau_s)
      return fail(ctx, STTM_ERR_STATE, "no spatial threshold chosen (call sttm_budget_threshold first)");
  }
  launch_spatial_decide(ctx->g, at<float>(ctx, ctx->lay.m), at<float>(ctx, ctx->lay.tau_s),
                        ctx->tau_s_pending ? at<SelState>(ctx, ctx->lay.sel_s) : nullptr, node_map_dev, node_level_dev,
                        ctx->stream);
  ctx->tau_s_pending = false;  // the kernel has left the threshold in the workspace
  return after_launch(ctx);
}

static int temporal_prepare(sttm_ctx* ctx, const void* feats_dev, const int32_t* node_map_dev,
                            const uint8_t** node_level_dev) {
  if (!node_map_dev) return fail(ctx, STTM_ERR_NULL, "node_map is NULL");
  if (!ctx->bound || !ctx->have_spatial)
    return fail(ctx, STTM_ERR_STATE, "temporal stage needs the spatial statistics of the same features");
  int rc = check_feats(ctx, feats_dev);
  if (rc) return rc;
  if (feats_dev != ctx->feats_spatial)  // norms, node sums and cell-to-cell dot products come from that pass
    return fail(ctx, STTM_ERR_STATE, "the spatial statistics in the workspace were computed from other features");
  if (!*node_level_dev) {
    launch_node_levels(ctx->g, node_map_dev, at<uint8_t>(ctx, ctx->lay.lvl), ctx->stream);
    *node_level_dev = at<uint8_t>(ctx, ctx->lay.lvl);
  }
  return STTM_OK;
}

int sttm_temporal_stats(sttm_ctx* ctx, const void* feats_dev, const int32_t* node_map_dev,
                        const uint8_t* node_level_dev) {
  if (!ctx) return STTM_ERR_NULL;
  STTM_HIP(ctx, hipSetDevice(ctx->device));
  int rc = temporal_prepare(ctx, feats_dev, node_map_dev, &node_level_dev);
  if (rc) return rc;
  return run_temporal_stats(ctx, feats_dev, node_map_dev, node_level_dev);
}

int sttm_temporal_merge(sttm_ctx* ctx, const void* feats_dev, const int32_t* node_map_dev,
                        const uint8_t* node_level_dev, const float* tau_t_host, int32_t* cluster_ids_dev) {
  if (!ctx) return STTM_ERR_NULL;
  if (!cluster_ids_dev) return fail(ctx, STTM_ERR_NULL, "cluster_ids is NULL");
  STTM_HIP(ctx, hipSetDevice(ctx->device));
  int rc = temporal_prepare(ctx, feats_dev, node_map_dev, &node_level_dev);
  if (rc) return rc;
  if (tau_t_host) {
    rc = upload_tau(ctx, tau_t_host, at<float>(ctx, ctx->lay.tau_t), &ctx->h_tau_t);
    if (rc) return rc;
    rc = run_temporal_stats(ctx, feats_dev, node_map_dev, node_level_dev);
    if (rc) return rc;
    ctx->have_tau_t = true;
  } else {
    if (!ctx->have_temporal)
      return fail(ctx, STTM_ERR_STATE, "no temporal statistics in the workspace (call sttm_temporal_stats first)");
    if (!ctx->have_tau_t)
      return fail(ctx, STTM_ERR_STATE, "no temporal threshold chosen (call sttm_budget_threshold first)");
    if (node_map_dev != ctx->node_map_temporal)
      return fail(ctx, STTM_ERR_STATE, "the temporal statistics in the workspace were computed for another node map");
  }
  launch_temporal_parent(ctx->g, ctx->match_mode, node_map_dev, node_level_dev, at<float>(ctx, ctx->lay.sig),
                         at<float>(ctx, ctx->lay.tau_t),
                         ctx->tau_t_pending ? at<SelState>(ctx, ctx->lay.sel_t) : nullptr,
                         at<int32_t>(ctx, ctx->lay.parent), at<int32_t>(ctx, ctx->lay.ptr_a), ctx->stream);
  ctx->tau_t_pending = false;
  launch_roots(ctx->g, at<int32_t>(ctx, ctx->lay.ptr_a), at<int32_t>(ctx, ctx->lay.ptr_b), node_map_dev,
               cluster_ids_dev, ctx->stream);
  return after_launch(ctx);
}

int sttm_budget_threshold(sttm_ctx* ctx, int stage, const double* target_keep_host, float* tau_out_host) {
  if (!ctx) return STTM_ERR_NULL;
  if (!target_keep_host) return fail(ctx, STTM_ERR_NULL, "target_keep is NULL");
  if (stage != STTM_STAGE_SPATIAL && stage != STTM_STAGE_TEMPORAL) return fail(ctx, STTM_ERR_ARG, "unknown stage");
  if (!ctx->bound || !ctx->have_spatial)
    return fail(ctx, STTM_ERR_STATE, "no spatial statistics in the workspace");
  if (stage == STTM_STAGE_TEMPORAL && !ctx->have_temporal)
    return fail(ctx, STTM_ERR_STATE, "no temporal statistics in the workspace");
  STTM_HIP(ctx, hipSetDevice(ctx->device));
  const Geo& g = ctx->g;
  const double thw = (double)g.T * g.HW;
  for (int b = 0; b < g.B; ++b) {
    const double k = target_keep_host[b];
    if (!(k > 0.0 && k <= 1.0)) return fail(ctx, STTM_ERR_ARG, "target_keep must be in (0, 1]");
  }
  const bool spatial = stage == STTM_STAGE_SPATIAL;
  std::vector<int>& h_target = spatial ? ctx->h_target_s : ctx->h_target_t;
  bool& on_device = spatial ? ctx->target_s_on_device : ctx->target_t_on_device;
  std::vector<int> want(g.B);
  for (int b = 0; b < g.B; ++b) {
    const double k = target_keep_host[b];
    want[b] = (int)std::floor((spatial ? std::sqrt(k) : k) * thw);
  }
  int rc;
  int* target_dev = at<int>(ctx, spatial ? ctx->lay.target_s : ctx->lay.target_t);
  if (!on_device || want != h_target) {  // the same targets as last time are already there
    h_target = want;
    STTM_HIP(ctx, hipMemcpyAsync(target_dev, h_target.data(), g.B * sizeof(int), hipMemcpyHostToDevice,
                                 ctx->stream));
    on_device = true;
  }
  float* tau_dev = at<float>(ctx, spatial ? ctx->lay.tau_s : ctx->lay.tau_t);
  // When the caller does not ask for the value, the last digit of the search is resolved by the kernel that uses the
  // threshold (one launch less); otherwise by a launch of its own.
  float* tau_now = tau_out_host ? tau_dev : nullptr;
  if (spatial) {
    launch_select_spatial(g, at<uint32_t>(ctx, ctx->lay.sel_key_s), at<uint8_t>(ctx, ctx->lay.sel_w_s),
                          target_dev, at<SelState>(ctx, ctx->lay.sel_s), ctx->sel_s_dirty, tau_now, ctx->stream);
    ctx->sel_s_dirty = true;
    ctx->tau_s_pending = tau_now == nullptr;
  } else {
    launch_select_temporal(g, ctx->node_map_temporal, at<uint32_t>(ctx, ctx->lay.sel_key_t), target_dev,
                           at<SelState>(ctx, ctx->lay.sel_t), ctx->sel_t_dirty, tau_now, ctx->stream);
    ctx->sel_t_dirty = true;
    ctx->tau_t_pending = tau_now == nullptr;
  }
  rc = after_launch(ctx);
  if (rc) return rc;
  if (stage == STTM_STAGE_SPATIAL) ctx->have_tau_s = true; else ctx->have_tau_t = true;
  if (tau_out_host) {
    STTM_HIP(ctx, hipMemcpyAsync(tau_out_host, tau_dev, g.B * sizeof(float), hipMemcpyDeviceToHost, ctx->stream));
    STTM_HIP(ctx, hipStreamSynchronize(ctx->stream));
  }
  return STTM_OK;
}

int sttm_reduce(sttm_ctx* ctx, const void* feats_dev, const int32_t* cluster_ids_dev,
                const int32_t* node_map_dev, const uint8_t* node_level_dev, int out_dtype, int64_t capacity,
                void* merged_dev, int32_t* counts_dev, int32_t* out_ids_dev, int64_t* offsets_dev,
                int64_t* n_out_host) {
  if (!ctx) return STTM_ERR_NULL;
  if (!cluster_ids_dev || !merged_dev || !offsets_dev)
    return fail(ctx, STTM_ERR_NULL, "cluster_ids, merged and offsets are required");
  if ((node_map_dev == nullptr) != (node_level_dev == nullptr))
    return fail(ctx, STTM_ERR_NULL, "node_map and node_level go together (both or neither)");
  if (out_dtype != STTM_F32 && out_dtype != STTM_BF16 && out_dtype != STTM_F16)
    return fail(ctx, STTM_ERR_DTYPE, "bad out_dtype");
  if (capacity < 0) return fail(ctx, STTM_ERR_ARG, "capacity < 0");
  if (!ctx->bound) return fail(ctx, STTM_ERR_STATE, "no shape bound (run the spatial stage first)");
  if (!reduce_io_supported(ctx->g.dtype, out_dtype))
    return fail(ctx, STTM_ERR_DTYPE, "a 16-bit input is written out in its own type or in fp32");
  int rc = check_feats(ctx, feats_dev);
  if (rc) return rc;
  if (node_map_dev && (!ctx->have_spatial || ctx->feats_spatial != feats_dev))
    return fail(ctx, STTM_ERR_STATE,
                "a partition was given but the workspace holds no stage-1 statistics of these features");
  if (reinterpret_cast<uintptr_t>(merged_dev) & 15) return fail(ctx, STTM_ERR_ARG, "merged must be 16-byte aligned");
  STTM_HIP(ctx, hipSetDevice(ctx->device));
  const ReduceBuffers rb = reduce_buffers(ctx->ws, ctx->lay);
  const bool zscan = ctx->order == STTM_ORDER_ZSCAN;
  ctx->cluster_ids_reduced = nullptr;
  launch_reduce_prepare(ctx->g, cluster_ids_dev, node_map_dev, node_level_dev, capacity, out_ids_dev, offsets_dev,
                        rb, zscan, ctx->stream);
  {
    Timed t(ctx, STTM_KERNEL_REDUCE_GATHER);
    launch_reduce_gather(ctx->g, feats_dev, at<float>(ctx, ctx->lay.nsum), node_map_dev, node_level_dev, out_dtype,
                         capacity, merged_dev, counts_dev, rb, zscan, ctx->stream);
  }
  launch_reduce_big(ctx->g, feats_dev, at<float>(ctx, ctx->lay.nsum), node_map_dev, node_level_dev, out_dtype,
                    capacity, merged_dev, counts_dev, rb, zscan, ctx->stream);
  rc = after_launch(ctx);
  if (rc) return rc;
  ctx->cluster_ids_reduced = cluster_ids_dev;
  ctx->reduced_zscan = zscan;
  if (n_out_host) {
    int32_t k = 0;
    STTM_HIP(ctx, hipMemcpyAsync(&k, rb.kdev, sizeof k, hipMemcpyDeviceToHost, ctx->stream));
    STTM_HIP(ctx, hipStreamSynchronize(ctx->stream));
    *n_out_host = k;
    if (k > capacity) {
      char buf[128];
      snprintf(buf, sizeof buf, "%d output tokens exceed the capacity of %lld rows", k, (long long)capacity);
      return fail(ctx, STTM_ERR_CAPACITY, buf);
    }
  }
  return STTM_OK;
}

int sttm_reduce_noalloc(sttm_ctx* ctx, const void* feats_dev, int dtype, int B, int T, int H, int W, int D,
                        const int32_t* cluster_ids_dev, int out_dtype, int64_t capacity, void* merged_dev,
                        int32_t* counts_dev, int32_t* out_ids_dev, int64_t* offsets_dev) {
  if (!ctx) return STTM_ERR_NULL;
  if (!cluster_ids_dev || !merged_dev || !offsets_dev)
    return fail(ctx, STTM_ERR_NULL, "cluster_ids, merged and offsets are required");
  if (dtype != STTM_F32 && dtype != STTM_BF16 && dtype != STTM_F16) return fail(ctx, STTM_ERR_DTYPE, "bad dtype");
  if (out_dtype != STTM_F32 && out_dtype != STTM_BF16 && out_dtype != STTM_F16)
    return fail(ctx, STTM_ERR_DTYPE, "bad out_dtype");
  if (!reduce_io_supported(dtype, out_dtype))
    return fail(ctx, STTM_ERR_DTYPE, "a 16-bit input is written out in its own type or in fp32");
  if (capacity < 0) return fail(ctx, STTM_ERR_ARG, "capacity < 0");
  int rc = check_feats(ctx, feats_dev);
  if (rc) return rc;
  if (reinterpret_cast<uintptr_t>(merged_dev) & 15) return fail(ctx, STTM_ERR_ARG, "merged must be 16-byte aligned");
  Geo g;
  std::memset(&g, 0, sizeof g);
  if (!make_geo(B, T, H, W, D, dtype, 1, &g))
    return fail(ctx, STTM_ERR_SHAPE, "need B,T >= 1, B*T <= 65535, 1 <= H,W <= 32, D % 8 == 0, B*T*H*W < 2^31");
  Layout l;
  std::memset(&l, 0, sizeof l);
  const size_t need = layout_reduce(g, 0, &l);
  if (need > kStaticScratchBytes) {
    char buf[160];
    snprintf(buf, sizeof buf, "shape needs %zu bytes of scratch, the static buffer holds %zu (use sttm_reduce)", need,
             kStaticScratchBytes);
    return fail(ctx, STTM_ERR_WORKSPACE, buf);
  }
  STTM_HIP(ctx, hipSetDevice(ctx->device));
  const ReduceBuffers rb = reduce_buffers(ctx->static_scratch, l);
  const bool zscan = ctx->order == STTM_ORDER_ZSCAN;
  launch_reduce_prepare(g, cluster_ids_dev, nullptr, nullptr, capacity, out_ids_dev, offsets_dev, rb, zscan,
                        ctx->stream);
  launch_reduce_gather(g, feats_dev, nullptr, nullptr, nullptr, out_dtype, capacity, merged_dev, counts_dev, rb, zscan,
                       ctx->stream);
  launch_reduce_big(g, feats_dev, nullptr, nullptr, nullptr, out_dtype, capacity, merged_dev, counts_dev, rb, zscan,
                    ctx->stream);
  return after_launch(ctx);
}

size_t sttm_reduce_noalloc_max_bytes(void) { return kStaticScratchBytes; }

size_t sttm_reduce_noalloc_bytes(int B, int T, int H, int W, int D, int dtype) {
  Geo g;
  if (!make_geo(B, T, H, W, D, dtype, 1, &g)) return 0;
  Layout l;
  std::memset(&l, 0, sizeof l);
  return layout_reduce(g, 0, &l);
}

int sttm_positions(sttm_ctx* ctx, const int32_t* cluster_ids_dev, const int32_t* node_map_dev,
                   const uint8_t* node_level_dev, const int64_t* offsets_dev, int64_t capacity, int32_t* survived_dev, int32_t* reassigned_dev,
                   float* merged_pos_dev, int32_t* root_tyxl_dev) {
  if (!ctx) return STTM_ERR_NULL;
  if (!cluster_ids_dev || !offsets_dev) return fail(ctx, STTM_ERR_NULL, "cluster_ids and offsets are required");
  if (capacity < 0) return fail(ctx, STTM_ERR_ARG, "capacity < 0");
  if (!ctx->bound || !ctx->cluster_ids_reduced || ctx->cluster_ids_reduced != cluster_ids_dev)
    return fail(ctx, STTM_ERR_STATE, "sttm_positions follows sttm_reduce on the same cluster_ids");
  if (ctx->reduced_zscan != (ctx->order == STTM_ORDER_ZSCAN))
    return fail(ctx, STTM_ERR_STATE, "the output order was changed after sttm_reduce");
  STTM_HIP(ctx, hipSetDevice(ctx->device));
  ReduceBuffers rb;
  std::memset(&rb, 0, sizeof rb);
  rb.rank = at<int32_t>(ctx, ctx->lay.rank);
  rb.order = at<int32_t>(ctx, ctx->lay.order);
  rb.seg = at<int32_t>(ctx, ctx->lay.seg);
  rb.kdev = at<int32_t>(ctx, ctx->lay.kdev);
  rb.zpos = at<int32_t>(ctx, ctx->lay.zpos);
  launch_positions(ctx->g, cluster_ids_dev, node_map_dev, node_level_dev, offsets_dev, capacity, rb,
                   ctx->reduced_zscan,
                   at<unsigned long long>(ctx, ctx->lay.possum), at<unsigned>(ctx, ctx->lay.poscnt), survived_dev,
                   reassigned_dev, merged_pos_dev, root_tyxl_dev, ctx->stream);
  return after_launch(ctx);
}

int sttm_export(sttm_ctx* ctx, int table, void* dst_dev, size_t bytes) {
  if (!ctx) return STTM_ERR_NULL;
  if (!dst_dev) return fail(ctx, STTM_ERR_NULL, "dst is NULL");
  if (!ctx->bound || !ctx->have_spatial) return fail(ctx, STTM_ERR_STATE, "nothing to export yet");
  const Geo& g = ctx->g;
  size_t off = 0, want = 0;
  bool temporal = false;
  switch (table) {
    case STTM_TBL_CHILD_SIM: off = ctx->lay.sim; want = (size_t)g.F * g.NN * 4; break;
    case STTM_TBL_MIN_SIM: off = ctx->lay.m; want = (size_t)g.F * g.NN * 4; break;
    case STTM_TBL_NORM2: off = ctx->lay.nrm2; want = (size_t)g.F * g.NN * 4; break;
    case STTM_TBL_PAIR_SIM: off = ctx->lay.sig; want = (size_t)g.N * 4; temporal = true; break;
    case STTM_TBL_BEST_SIM: off = ctx->lay.e; want = (size_t)g.N * 4; temporal = true; break;
    case STTM_TBL_PARENT: off = ctx->lay.parent; want = (size_t)g.N * 4; temporal = true; break;
    default: return fail(ctx, STTM_ERR_ARG, "unknown table");
  }
  if (temporal && !ctx->have_temporal) return fail(ctx, STTM_ERR_STATE, "no temporal statistics yet");
  if (bytes != want) return fail(ctx, STTM_ERR_ARG, "byte count does not match the table size");
  STTM_HIP(ctx, hipSetDevice(ctx->device));
  STTM_HIP(ctx, hipMemcpyAsync(dst_dev, ctx->ws + off, want, hipMemcpyDeviceToDevice, ctx->stream));
  return STTM_OK;
}

int sttm_profile_enable(sttm_ctx* ctx, int on) {
  if (!ctx) return STTM_ERR_NULL;
  ctx->profiling = on < 0 ? 0 : on;
  for (auto& u : ctx->ev_used) u = 0;
  for (auto& u : ctx->prof_seen) u = 0;
  return STTM_OK;
}

int sttm_profile_read(sttm_ctx* ctx, int kernel, double* total_ms, int64_t* launches) {
  if (!ctx) return STTM_ERR_NULL;
  if (!total_ms || !launches) return fail(ctx, STTM_ERR_NULL, "total_ms and launches are required");
  if (kernel < 0 || kernel >= STTM_KERNEL_COUNT) return fail(ctx, STTM_ERR_ARG, "unknown kernel id");
  STTM_HIP(ctx, hipStreamSynchronize(ctx->stream));
  double tot = 0.0;
  for (size_t i = 0; i < ctx->ev_used[kernel]; ++i) {
    float ms = 0.f;
    STTM_HIP(ctx, hipEventElapsedTime(&ms, ctx->ev[kernel][i].a, ctx->ev[kernel][i].b));
    tot += ms;
  }
  *total_ms = tot;
  *launches = (int64_t)ctx->ev_used[kernel];
  return STTM_OK;
}

}  // extern "C"
