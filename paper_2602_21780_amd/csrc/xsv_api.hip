// Host side of libxsv: context, argument validation, state machine, launch sequencing.
// Every step of the path runs in the kernels of attend.hip / score_select.hip / requant.hip; this
// file only decides WHICH launches a step needs (the cache lengths are known on the host: they
// depend on token counts alone) and owns the device memory.
#include "../../include/xsv.h"
#include "../../include/xsv_tune.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "xsv_internal.h"

using namespace xsv;

namespace {

enum Phase { kIdle = 0, kAttended = 1, kScored = 2 };

// The fork / join events only order the context's two streams on one device: no timing, and no system-scope
// fence (nothing here is read by the host or by another device at these points).
constexpr unsigned kOrderingEvent = hipEventDisableTiming | hipEventDisableSystemFence;

struct LayerState {
  int T = 0;        // cached tokens
  int frames = 0;   // frames seen
  int buf = 0;      // buffer holding the cache
  int phase = kIdle;
  int pending_Tn = 0;   // keep length decided by score_prune
  int last_P = 0;       // scores computed by the last score_prune (0 if none)
  int last_keep = 0;
};

}  // namespace

struct xsv_ctx {
  xsv_config cfg;
  hipStream_t stream;
  // xsv_step runs the score/select/re-quantize chain on `side` while the attention kernel runs on
  // `stream` (the chain only reads what attention reads and writes the OTHER cache buffer)
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  hipStream_t work = nullptr;  // stream the score/quantize launchers currently enqueue on
  int overlap = 1;             // 0: one stream; 1: side stream, joined before the call returns; 2: joined lazily
  // overlap == 2: ev_chain[l] is recorded on `side` behind the chain of a step that began at layer l;
  // pending[l] >= 0 names the event `stream` still has to wait for before it may touch layer l
  std::vector<hipEvent_t> ev_chain;
  std::vector<int> pending;
  // the side stream is in order, so a later record implies every earlier one: seq[e] numbers the records
  std::vector<long long> seq;
  long long next_seq = 1;
  CachePool pool;
  Workspace ws;
  uint8_t* stable_flag = nullptr;  // [L][H][Tcap / 64], see RequantArgs
  std::vector<LayerState> layers;
  std::vector<void*> allocs;
  int splits_single = 0, splits_batched = 0;
  int attend_variant = 3;  // 8 waves x 64 query rows per workgroup (xsv_create picks 8 x 32 where that wastes fewer rows)
  int last_attend_wgs = 0;  // grid of the most recent attention launch
  // optional timing of the attention launches: events before, between the two kernels, after, and one more
  // right behind (the span of the last two, with nothing between them, is what an event pair itself costs)
  bool timing = false;
  std::vector<hipEvent_t> timing_events;
  size_t timing_used = 0;
  std::vector<hipEvent_t> chain_events;  // triples on the chain's stream: before score, after select, after re-quantize
  size_t chain_used = 0;
  int frame_tile_cost = 95;  // cost of a key tile of the frame's own rows in percent of a cache tile's (attention range cut)
  int short_pct = -1; // xsv_step: length of one extra, short key range per unit, in percent of a long one (0 = none, -1 = by overlap mode)
  int side_cus = -1;  // compute units xsv_step leaves to the prune chain while attention runs (-1: by launch size)
  size_t part_rows = 0;  // rows the partial-output workspace holds
  int n_cu = 256;
  bool broken = false;
};

namespace {

int round_up(int a, int b) { return (a + b - 1) / b * b; }

bool tensor_ok(const xsv_tensor& t) {
  return t.ptr != nullptr && t.stride_token >= kD && t.stride_token <= (1ll << 24) && t.stride_head >= 0 &&
         (reinterpret_cast<uintptr_t>(t.ptr) % 16 == 0) && t.stride_token % 8 == 0 && t.stride_head % 8 == 0;
}

int hip_fail(xsv_ctx* ctx) {
  if (ctx) ctx->broken = true;
  return XSV_ERR_HIP;
}

template <typename T>
int dev_alloc(xsv_ctx* ctx, T** out, size_t count, bool zero) {
  void* p = nullptr;
  const size_t bytes = std::max<size_t>(count * sizeof(T), 256);
  if (hipMalloc(&p, bytes) != hipSuccess) {
    (void)hipGetLastError();
    return XSV_ERR_OOM;
  }
  ctx->allocs.push_back(p);
  if (zero && hipMemsetAsync(p, 0, bytes, ctx->stream) != hipSuccess) return XSV_ERR_HIP;
  *out = static_cast<T*>(p);
  return XSV_OK;
}

void free_all(xsv_ctx* ctx) {
  for (void* p : ctx->allocs) (void)hipFree(p);
  ctx->allocs.clear();
  if (ctx->side) (void)hipStreamDestroy(ctx->side);
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
  for (hipEvent_t e : ctx->ev_chain) (void)hipEventDestroy(e);
  for (hipEvent_t e : ctx->timing_events) (void)hipEventDestroy(e);
  ctx->timing_events.clear();
  for (hipEvent_t e : ctx->chain_events) (void)hipEventDestroy(e);
  ctx->chain_events.clear();
  ctx->ev_chain.clear();
  ctx->side = nullptr;
  ctx->ev_fork = ctx->ev_join = nullptr;
}

// An event that only orders streams.  A runtime that does not know the no-system-fence flag gets a plain
// untimed event (same ordering, a little more cost per record).
bool ordering_event(hipEvent_t* e) {
  if (hipEventCreateWithFlags(e, kOrderingEvent) == hipSuccess) return true;
  (void)hipGetLastError();
  *e = nullptr;
  if (hipEventCreateWithFlags(e, hipEventDisableTiming) == hipSuccess) return true;
  (void)hipGetLastError();
  *e = nullptr;
  return false;
}

// Orders the context's stream after the side-stream work still outstanding for layers [l0, l0 + n): ONE wait, for
// the latest of their records (the side stream runs in order), which also settles every layer recorded before it.
// A wait costs the waiting stream several microseconds even when the event has long fired, so a step that has to
// wait anyway waits for a NEWER record if there is one that is `settled_lag` records old or older - the chains
// behind such a record have had time to finish - and thereby settles the layers the following steps would each
// have waited for (one wait per frame instead of one per layer when the caller never calls xsv_join).
int join_layers(xsv_ctx* ctx, int l0, int n, int settled_lag = -1) {
  int latest = -1;
  for (int l = l0; l < l0 + n; ++l) {
    const int e = ctx->pending[l];
    if (e >= 0 && (latest < 0 || ctx->seq[e] > ctx->seq[latest])) latest = e;
  }
  if (latest < 0) return XSV_OK;
  if (settled_lag >= 0) {
    for (int e : ctx->pending)
      if (e >= 0 && ctx->seq[e] > ctx->seq[latest] && ctx->seq[e] <= ctx->next_seq - 1 - settled_lag) latest = e;
  }
  if (hipStreamWaitEvent(ctx->stream, ctx->ev_chain[latest], 0) != hipSuccess) return hip_fail(ctx);
  for (int& e : ctx->pending)
    if (e >= 0 && ctx->seq[e] <= ctx->seq[latest]) e = -1;
  return XSV_OK;
}

// For the synchronous introspection calls: the side stream's work on the layer is ordered into the context's
// stream AND waited for from the host, so that copies to the host made next see it whatever fence the ordering
// events carry.
int settle_layer(xsv_ctx* ctx, int layer) {
  const int rc = join_layers(ctx, layer, 1);
  if (rc != XSV_OK) return rc;
  if (ctx->side && hipStreamSynchronize(ctx->side) != hipSuccess) return hip_fail(ctx);
  return XSV_OK;
}

// What a step does to the cache length (paper Sec. 3.2: prune once T exceeds the budget; first and
// current frames always stay).  Pure token counting — known on the host without reading the GPU.
struct PrunePlan {
  int T;         // length after the append
  int T_first, T_cur, P, k;
  bool prune;    // keep list differs from "everything"
  bool score;    // scores are needed (0 < k < P)
  int Tn;        // keep length
};

PrunePlan plan_for(const xsv_config& c, const LayerState& L) {
  PrunePlan p{};
  const int n = c.tokens_per_frame;
  p.T = L.T + n;
  p.T_first = n;
  p.T_cur = n;
  p.prune = !(c.budget == 0 || p.T <= c.budget || L.frames == 0);
  if (!p.prune) {
    p.P = 0; p.k = 0; p.score = false; p.Tn = p.T;
    return p;
  }
  p.P = p.T - p.T_first - p.T_cur;
  p.k = std::min(std::max(0, c.budget - p.T_first - p.T_cur), p.P);
  p.score = p.k > 0 && p.k < p.P;
  p.Tn = p.T_first + p.k + p.T_cur;
  return p;
}

// Workgroups of one attention launch.  requested > 0: every unit is cut into that many equal key
// ranges.  Otherwise one workgroup per slot of the chip (2 per compute unit for the 4-wave shapes, 1
// for the 8-wave ones), minus the compute units left to kernels running beside it.
AttendPlan choose_grid(const xsv_ctx* ctx, int n_layers, int Tc, int requested, int spare_cus) {
  const xsv_config& c = ctx->cfg;
  const int rows = attend_rows_per_workgroup(ctx->attend_variant);
  const int n_units = ((c.tokens_per_frame + rows - 1) / rows) * c.n_heads * n_layers;
  const int per_cu = ctx->attend_variant >= 2 ? 1 : 2;
  int want = requested > 0 ? n_units * requested : per_cu * std::max(ctx->n_cu / 2, ctx->n_cu - spare_cus);
  // a grid that cuts every unit into the same number of ranges has no workgroup that ends one unit
  // and begins another (two pipeline fills, two sets of partials); prefer it when it is nearly as large
  if (requested <= 0 && want / n_units >= 1 && (want / n_units) * n_units * 8 >= want * 7) want = (want / n_units) * n_units;
  return plan_attend(ctx->attend_variant, n_layers, c.n_heads, c.tokens_per_frame, Tc, want, ctx->part_rows);
}

int fill_batch(xsv_ctx* ctx, Batch& b, int layer0, int n_layers, const xsv_tensor* q, const xsv_tensor* k,
               const xsv_tensor* v, void* const* out) {
  std::memset(&b, 0, sizeof(b));
  b.n_layers = n_layers;
  b.layer0 = layer0;
  // the frame's K and V rows of one head are read through a buffer resource with 32-bit byte offsets: the rows of a
  // head must lie within 2 GiB of its first one
  const long long n_rows = ctx->cfg.tokens_per_frame;
  auto span_ok = [&](const xsv_tensor& t) { return ((n_rows - 1) * t.stride_token + kD) * 2 <= (1ll << 31); };
  if ((k && n_layers > 0 && !span_ok(k[0])) || (v && n_layers > 0 && !span_ok(v[0]))) return XSV_ERR_ARG;
  for (int i = 0; i < n_layers; ++i) {
    if (ctx->layers[layer0 + i].buf) b.bufsel |= 1u << i;
    if (q) {
      if (!tensor_ok(q[i]) || q[i].stride_head != q[0].stride_head || q[i].stride_token != q[0].stride_token) return XSV_ERR_ARG;
      b.q[i] = static_cast<const uint16_t*>(q[i].ptr);
    }
    if (k) {
      if (!tensor_ok(k[i]) || k[i].stride_head != k[0].stride_head || k[i].stride_token != k[0].stride_token) return XSV_ERR_ARG;
      b.k[i] = static_cast<const uint16_t*>(k[i].ptr);
    }
    if (v) {
      if (!tensor_ok(v[i]) || v[i].stride_head != v[0].stride_head || v[i].stride_token != v[0].stride_token) return XSV_ERR_ARG;
      b.v[i] = static_cast<const uint16_t*>(v[i].ptr);
    }
    if (out) {
      if (out[i] == nullptr || reinterpret_cast<uintptr_t>(out[i]) % 16 != 0) return XSV_ERR_ARG;
      b.out[i] = static_cast<uint16_t*>(out[i]);
    }
  }
  if (q) { b.q_sh = q[0].stride_head; b.q_st = q[0].stride_token; }
  if (k) { b.k_sh = k[0].stride_head; b.k_st = k[0].stride_token; }
  if (v) { b.v_sh = v[0].stride_head; b.v_st = v[0].stride_token; }
  return XSV_OK;
}

// Where the R key ranges of a unit begin (begin[0] = 0 .. begin[R] = all tiles), so that every range costs the same:
// a cache tile costs 100, a tile of the frame's own rows frame_cost; the last range gets last_pct percent of a
// full share.  Every range holds at least one tile (R <= tiles).
void range_starts(int n_ct, int n_ft, int R, int last_pct, int frame_cost, int32_t* begin) {
  const int n_tiles = n_ct + n_ft;
  const long long total = 100ll * n_ct + (long long)frame_cost * n_ft;
  const long long shares = 100ll * (R - 1) + last_pct;  // in percent of a full share
  begin[0] = 0;
  long long acc = 0;
  int t = 0;
  for (int p = 1; p < R; ++p) {
    const long long target = total * (100ll * p) / shares;  // cost in front of range p
    while (t < n_tiles - (R - p)) {                         // leave one tile for each range still to come
      const int c = t < n_ct ? 100 : frame_cost;
      if (t > begin[p - 1] && acc + c / 2 >= target) break;  // not empty, and nearer to the target without this tile
      acc += c;
      ++t;
    }
    begin[p] = t;
  }
  begin[R] = n_tiles;
}

// The three stages for layers [layer0, layer0 + n_layers), which must be in step with each other.
// frame_only: the frame's own tokens are the only keys (no cache tiles, no change of state).
int do_attend(xsv_ctx* ctx, int layer0, int n_layers, const xsv_tensor* q, const xsv_tensor* k, const xsv_tensor* v,
              void* const* out, int splits_req, int spare_cus, bool frame_only = false) {
  AttendArgs a{};
  {
    Batch b;
    int rc = fill_batch(ctx, b, layer0, n_layers, q, k, v, out);
    if (rc != XSV_OK) return rc;
    const CachePool& p = ctx->pool;
    for (int i = 0; i < n_layers; ++i) {
      const LayerCache lc = layer_cache(p, b.src_buf(i), layer0 + i);
      AttendLayer& ly = a.layer[i];
      ly.kc = reinterpret_cast<const uint32_t*>(lc.kc); ly.ks = lc.ks; ly.kz = lc.kz;
      ly.vc = reinterpret_cast<const uint32_t*>(lc.vc); ly.vs = lc.vs; ly.vz = lc.vz;
      ly.q = b.q[i]; ly.k = b.k[i]; ly.v = b.v[i]; ly.out = b.out[i];
    }
    a.n_layers = n_layers; a.H = p.H; a.bits = p.bits; a.G = p.G; a.Tcap = p.Tcap;
    a.code_head = (uint32_t)((size_t)p.Tcap * (kD * p.bits / 32));
    a.kparam_head = (uint32_t)((size_t)(p.Tcap / p.G) * kD);
    a.vparam_head = (uint32_t)((size_t)p.Tcap * (kD / p.G));
    a.q_sh = b.q_sh; a.q_st = b.q_st; a.k_sh = b.k_sh; a.k_st = b.k_st; a.v_sh = b.v_sh; a.v_st = b.v_st;
    a.attn_o = ctx->ws.attn_o; a.attn_ml = ctx->ws.attn_ml;
  }
  a.Tc = frame_only ? 0 : ctx->layers[layer0].T;
  a.n = ctx->cfg.tokens_per_frame;
  a.variant = ctx->attend_variant;
  AttendPlan plan = choose_grid(ctx, n_layers, a.Tc, splits_req, spare_cus);
  const int n_ct = (a.Tc + kTile - 1) / kTile, n_ft = (a.n + kTile - 1) / kTile, n_tiles = n_ct + n_ft;
  bool short_last = false;
  // with deferred joins the chain only has to keep up, so the short range can be longer (the long ones shorter) than
  // when every step waits for its chain before it returns
  const int short_pct = ctx->short_pct >= 0 ? ctx->short_pct : (ctx->overlap == 2 ? 50 : 35);
  if (splits_req <= 0 && spare_cus > 0 && short_pct > 0) {
    // beside the overlapped chain: the equal cut that leaves spare units, plus one short range per unit
    const int rows = attend_rows_per_workgroup(ctx->attend_variant);
    const int n_units = ((a.n + rows - 1) / rows) * ctx->cfg.n_heads * n_layers;
    const int S = plan.n_wgs % n_units == 0 ? plan.n_wgs / n_units : 0;
    if (S >= 1 && (S + 1) * n_units <= ctx->n_cu - 8 && S + 1 <= kMaxPieces && S + 1 <= n_tiles) {
      const AttendPlan more = plan_attend(ctx->attend_variant, n_layers, ctx->cfg.n_heads, a.n, a.Tc, (S + 1) * n_units, ctx->part_rows);
      if (more.n_wgs == (S + 1) * n_units) {
        plan = more;
        short_last = true;
      }
    }
  }
  a.n_wgs = plan.n_wgs;
  a.rows_wg = plan.rows_wg;
  a.cut = plan.max_pieces > 1;
  {
    const int n_units = ((a.n + plan.rows_wg - 1) / plan.rows_wg) * ctx->cfg.n_heads * n_layers;
    const int ranges = plan.n_wgs % n_units == 0 ? plan.n_wgs / n_units : 0;
    a.equal_ranges = (ranges > 1 && ranges <= kMaxPieces && ranges <= n_tiles) ? ranges : 0;
    a.xcd_ranges = (ranges > 0 && (ctx->cfg.n_heads * n_layers * ranges) % 8 == 0) ? ranges : 0;
    if (a.equal_ranges > 0) range_starts(n_ct, n_ft, a.equal_ranges, short_last ? short_pct : 100, ctx->frame_tile_cost, a.range_begin);
  }
  ctx->last_attend_wgs = plan.n_wgs;
  a.qscale = ctx->cfg.softmax_scale * 1.4426950408889634f;
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  if (ctx->timing) {
    while (ctx->timing_events.size() < ctx->timing_used + 4) {
      hipEvent_t e = nullptr;
      if (hipEventCreate(&e) != hipSuccess) return hip_fail(ctx);
      ctx->timing_events.push_back(e);
    }
    for (int i = 0; i < 4; ++i) ev[i] = ctx->timing_events[ctx->timing_used + i];
    ctx->timing_used += 4;
    if (hipEventRecord(ev[0], ctx->stream) != hipSuccess) return hip_fail(ctx);
  }
  if (launch_attend(a, ctx->stream, ev[1]) != hipSuccess) return hip_fail(ctx);
  if (ev[2] && (hipEventRecord(ev[2], ctx->stream) != hipSuccess || hipEventRecord(ev[3], ctx->stream) != hipSuccess))
    return hip_fail(ctx);
  for (int i = 0; i < n_layers && !frame_only; ++i) ctx->layers[layer0 + i].phase = kAttended;
  return XSV_OK;
}

int do_score_prune(xsv_ctx* ctx, int layer0, int n_layers, const xsv_tensor* q) {
  const PrunePlan p = plan_for(ctx->cfg, ctx->layers[layer0]);
  // the lists of layers [layer0, layer0 + n_layers) are contiguous: sets per layer
  const int sets = ctx->ws.sets, n_lists = n_layers * sets;
  int32_t* keep = ctx->ws.keep + list_index(sets, layer0, 0) * ctx->ws.scores_stride;
  if (!p.prune) {
    if (launch_fill_keep(keep, ctx->ws.scores_stride, n_lists, p.T, 0, 0, true, ctx->work) != hipSuccess) return hip_fail(ctx);
  } else if (!p.score) {
    // k == 0: first ∪ current;  k == P: everything (cannot happen once T > budget, kept for completeness)
    if (launch_fill_keep(keep, ctx->ws.scores_stride, n_lists, p.T_first, p.P, p.T_cur, p.k == p.P, ctx->work) != hipSuccess)
      return hip_fail(ctx);
  } else {
    ScoreArgs s{};
    int rc = fill_batch(ctx, s.b, layer0, n_layers, q, nullptr, nullptr, nullptr);
    if (rc != XSV_OK) return rc;
    s.pool = ctx->pool;
    s.ws = ctx->ws;
    s.Tc = ctx->layers[layer0].T;
    s.n = ctx->cfg.tokens_per_frame;
    s.n_special = ctx->cfg.n_special;
    s.pool_size = ctx->cfg.pool_size;
    s.T_first = p.T_first;
    s.P = p.P;
    s.k_plain = nullptr;
    s.per_head = ctx->cfg.score_mode == 1;
    if (launch_pool_query(s, ctx->work) != hipSuccess) return hip_fail(ctx);
    if (launch_score(s, ctx->work) != hipSuccess) return hip_fail(ctx);
    SelectArgs sel{};
    sel.scores = ctx->ws.scores + list_index(sets, layer0, 0) * ctx->ws.scores_stride;
    sel.keep = keep;
    sel.scores_stride = sel.keep_stride = ctx->ws.scores_stride;
    sel.n_lists = n_lists;
    sel.P = p.P; sel.k = p.k; sel.T_first = p.T_first; sel.T_cur = p.T_cur;
    if (launch_select(sel, ctx->work) != hipSuccess) return hip_fail(ctx);
  }
  for (int i = 0; i < n_layers; ++i) {
    LayerState& L = ctx->layers[layer0 + i];
    L.phase = kScored;
    L.pending_Tn = p.Tn;
    L.last_P = p.score ? p.P : 0;
    L.last_keep = p.Tn;
  }
  return XSV_OK;
}

int do_quantize(xsv_ctx* ctx, int layer0, int n_layers, const xsv_tensor* k, const xsv_tensor* v) {
  RequantArgs r{};
  int rc = fill_batch(ctx, r.b, layer0, n_layers, nullptr, k, v, nullptr);
  if (rc != XSV_OK) return rc;
  r.pool = ctx->pool;
  r.ws = ctx->ws;
  r.Tc = ctx->layers[layer0].T;
  r.n = ctx->cfg.tokens_per_frame;
  r.Tn = ctx->layers[layer0].pending_Tn;
  r.frame_id = ctx->layers[layer0].frames;
  {
    const PrunePlan p = plan_for(ctx->cfg, ctx->layers[layer0]);
    r.identity_end = p.prune ? std::min(p.T_first, r.Tc) : r.Tc;
    r.stable_blocks = r.identity_end / kTile;
    r.stable_flag = ctx->stable_flag;
    r.carry_values = ctx->cfg.value_mode == 1;
  }
  if (launch_requant(r, ctx->work) != hipSuccess) return hip_fail(ctx);
  for (int i = 0; i < n_layers; ++i) {
    LayerState& L = ctx->layers[layer0 + i];
    L.T = r.Tn;
    L.frames += 1;
    if (ctx->pool.buffers == 2) L.buf ^= 1;
    L.phase = kIdle;
  }
  return XSV_OK;
}

int check_layer(xsv_ctx* ctx, int layer) {
  if (!ctx) return XSV_ERR_ARG;
  if (ctx->broken) return XSV_ERR_HIP;
  if (layer < 0 || layer >= ctx->cfg.n_layers) return XSV_ERR_ARG;
  return XSV_OK;
}

int check_capacity(xsv_ctx* ctx, int layer) {
  // the cache must hold what the step retains; only an unbounded cache can run out of room
  if (plan_for(ctx->cfg, ctx->layers[layer]).Tn > ctx->pool.Tcap) return XSV_ERR_STATE;
  return XSV_OK;
}

}  // namespace

// device temporaries → host copies for the export and the stateless entry points
namespace {
struct Temp {
  std::vector<void*> ptrs;
  ~Temp() { for (void* p : ptrs) (void)hipFree(p); }
  template <typename T> T* get(size_t count) {
    void* p = nullptr;
    if (hipMalloc(&p, std::max<size_t>(count * sizeof(T), 256)) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    ptrs.push_back(p);
    return static_cast<T*>(p);
  }
};
}  // namespace

extern "C" {

const char* xsv_strerror(int code) {
  switch (code) {
    case XSV_OK: return "ok";
    case XSV_ERR_ARG: return "invalid argument";
    case XSV_ERR_UNSUPPORTED: return "configuration not supported by this build";
    case XSV_ERR_OOM: return "device allocation failed";
    case XSV_ERR_STATE: return "call order violated or layers out of step";
    case XSV_ERR_HIP: return "HIP call failed";
    default: return "unknown error";
  }
}

int xsv_create(const xsv_config* cfg, void* hip_stream, xsv_ctx** out) {
  if (!cfg || !out) return XSV_ERR_ARG;
  *out = nullptr;
  xsv_config c = *cfg;
  if (c.n_layers < 1 || c.n_heads < 1 || c.tokens_per_frame < 1 || c.n_special < 0 || c.n_special > c.tokens_per_frame ||
      c.budget < 0 || c.pool_size < 1 || !(c.softmax_scale >= 0.0f) || !std::isfinite(c.softmax_scale))
    return XSV_ERR_ARG;
  if (c.kv_bits != 2 && c.kv_bits != 4 && c.kv_bits != 16) return XSV_ERR_ARG;
  if (c.score_mode != 0 && c.score_mode != 1) return XSV_ERR_ARG;
  if (c.value_mode != 0 && c.value_mode != 1) return XSV_ERR_ARG;
  if (c.head_dim != kD) return XSV_ERR_UNSUPPORTED;
  if (c.kv_bits == 16) c.group_size = 64;
  if (c.group_size != 32 && c.group_size != 64) return c.group_size > 0 ? XSV_ERR_UNSUPPORTED : XSV_ERR_ARG;
  if (c.budget == 0 && c.max_frames < 1) return XSV_ERR_ARG;
  if (c.softmax_scale == 0.0f) c.softmax_scale = 1.0f / std::sqrt((float)c.head_dim);
  const long long n = c.tokens_per_frame;
  // after a step the cache holds at most max(budget, first + current) tokens
  const long long cap_tokens = c.budget > 0 ? std::max<long long>(c.budget, 2 * n) : n * c.max_frames;
  if (cap_tokens > (1ll << 24) || (long long)c.n_heads * c.n_layers > (1 << 16)) return XSV_ERR_UNSUPPORTED;

  xsv_ctx* ctx = new (std::nothrow) xsv_ctx;
  if (!ctx) return XSV_ERR_OOM;
  ctx->cfg = c;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  ctx->work = ctx->stream;
  ctx->layers.resize(c.n_layers);
  // the device is queried before anything is created, so this failure has nothing to release
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    (void)hipGetLastError();
    delete ctx;
    return XSV_ERR_HIP;
  }
  if (hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking) != hipSuccess || !ordering_event(&ctx->ev_fork) ||
      !ordering_event(&ctx->ev_join)) {
    free_all(ctx);
    delete ctx;
    return XSV_ERR_HIP;
  }
  // workgroups of 512 query rows unless blocks of 256 leave fewer padding rows in a frame's last block
  // (1041 tokens: 1280 against 1536 rows)
  ctx->attend_variant = round_up(c.tokens_per_frame, 256) < round_up(c.tokens_per_frame, 512) ? 2 : 3;
  ctx->pending.assign(c.n_layers, -1);
  ctx->seq.assign(c.n_layers, 0);
  for (int l = 0; l < c.n_layers; ++l) {
    hipEvent_t e = nullptr;
    if (!ordering_event(&e)) {
      free_all(ctx);
      delete ctx;
      return XSV_ERR_HIP;
    }
    ctx->ev_chain.push_back(e);
  }
  ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

  CachePool& p = ctx->pool;
  std::memset(&p, 0, sizeof(p));
  p.L = c.n_layers; p.H = c.n_heads; p.bits = c.kv_bits; p.G = c.group_size;
  p.Tcap = round_up((int)cap_tokens, kTile);
  p.sets = c.score_mode == 1 ? c.n_heads : 1;
  // a cache that is never pruned keeps every row where it is: one buffer, rewritten in place where a step touches it
  p.buffers = c.budget == 0 ? 1 : 2;
  const size_t slabs = (size_t)p.buffers * c.n_layers;
  int rc = XSV_OK;
  auto A = [&](auto** ptr, size_t count, bool zero) { if (rc == XSV_OK) rc = dev_alloc(ctx, ptr, count, zero); };
  // zero-filled: padding rows of a ragged last block are read (masked) by the attention kernel
  A(&p.kc, slabs * p.code_slab(), true);
  A(&p.vc, slabs * p.code_slab(), true);
  if (c.kv_bits != 16) {
    A(&p.ks, slabs * p.kparam_slab(), true);
    A(&p.kz, slabs * p.kparam_slab(), true);
    A(&p.vs, slabs * p.vparam_slab(), true);
    A(&p.vz, slabs * p.vparam_slab(), true);
  }
  A(&p.tok_frame, slabs * p.tok_slab(), true);
  A(&p.tok_index, slabs * p.tok_slab(), true);

  Workspace& w = ctx->ws;
  std::memset(&w, 0, sizeof(w));
  w.scores_stride = p.Tcap + (int)n;
  w.qpart_rows = c.n_heads * kPoolSeg;
  w.sets = p.sets;
  A(&ctx->stable_flag, (size_t)c.n_layers * c.n_heads * (p.Tcap / kTile), true);
  A(&w.scores, (size_t)c.n_layers * w.sets * w.scores_stride, true);
  A(&w.keep, (size_t)c.n_layers * w.sets * w.scores_stride, true);
  A(&w.qpart, (size_t)c.n_layers * w.qpart_rows * kD, true);
  // partial attention outputs: up to 16 key ranges for one layer, or 2 per layer when batched
  // (partials are stored in blocks of 32 query rows per head)
  const size_t part_rows = (size_t)std::max(16, 2 * std::min(c.n_layers, kMaxBatch)) * c.n_heads * round_up((int)n, 32);
  ctx->part_rows = part_rows;
  A(&w.attn_o, part_rows * kD, false);
  A(&w.attn_ml, part_rows * 4, false);
  if (rc == XSV_OK && hipStreamSynchronize(ctx->stream) != hipSuccess) rc = XSV_ERR_HIP;
  if (rc != XSV_OK) {
    free_all(ctx);
    delete ctx;
    return rc;
  }
  *out = ctx;
  return XSV_OK;
}

int xsv_destroy(xsv_ctx* ctx) {
  if (!ctx) return XSV_OK;
  (void)hipStreamSynchronize(ctx->stream);
  if (ctx->side) (void)hipStreamSynchronize(ctx->side);
  free_all(ctx);
  delete ctx;
  return XSV_OK;
}

int xsv_reset(xsv_ctx* ctx) {
  if (!ctx) return XSV_ERR_ARG;
  if (ctx->broken) return XSV_ERR_HIP;
  const int rc = join_layers(ctx, 0, ctx->cfg.n_layers);
  if (rc != XSV_OK) return rc;
  for (LayerState& L : ctx->layers) L = LayerState();
  const size_t flags = (size_t)ctx->cfg.n_layers * ctx->cfg.n_heads * (ctx->pool.Tcap / kTile);
  if (launch_zero_bytes(ctx->stable_flag, flags, ctx->stream) != hipSuccess) return hip_fail(ctx);
  return XSV_OK;
}

int xsv_join(xsv_ctx* ctx) {
  if (!ctx) return XSV_ERR_ARG;
  if (ctx->broken) return XSV_ERR_HIP;
  return join_layers(ctx, 0, ctx->cfg.n_layers);
}

int xsv_set_attend_splits(xsv_ctx* ctx, int per_layer_calls, int batched_calls) {
  if (!ctx || per_layer_calls < 0 || per_layer_calls > 16 || batched_calls < 0 || batched_calls > 16) return XSV_ERR_ARG;
  ctx->splits_single = per_layer_calls;
  ctx->splits_batched = batched_calls;
  return XSV_OK;
}

int xsv_set_attend_timing(xsv_ctx* ctx, int enabled) {
  if (!ctx) return XSV_ERR_ARG;
  ctx->timing = enabled != 0;
  ctx->timing_used = 0;
  ctx->chain_used = 0;
  return XSV_OK;
}

int xsv_attend_times(xsv_ctx* ctx, int32_t* launches, float* attend_ms, float* merge_ms, float* event_ms) {
  if (!ctx || !launches || !attend_ms || !merge_ms) return XSV_ERR_ARG;
  if (ctx->broken) return XSV_ERR_HIP;
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) return hip_fail(ctx);
  double a = 0.0, m = 0.0, own = 0.0;
  const size_t n = ctx->timing_used / 4;
  for (size_t i = 0; i < n; ++i) {
    float t0 = 0.f, t1 = 0.f, t2 = 0.f;
    hipEvent_t* e = &ctx->timing_events[4 * i];
    if (hipEventElapsedTime(&t0, e[0], e[1]) != hipSuccess || hipEventElapsedTime(&t1, e[1], e[2]) != hipSuccess ||
        hipEventElapsedTime(&t2, e[2], e[3]) != hipSuccess)
      return hip_fail(ctx);
    a += t0;
    m += t1;
    own += t2;
  }
  *launches = (int32_t)n;
  *attend_ms = n ? (float)(a / n) : 0.f;
  *merge_ms = n ? (float)(m / n) : 0.f;
  if (event_ms) *event_ms = n ? (float)(own / n) : 0.f;
  ctx->timing_used = 0;
  return XSV_OK;
}

int xsv_chain_times(xsv_ctx* ctx, int32_t* steps, float* score_prune_ms, float* quantize_ms) {
  if (!ctx || !steps || !score_prune_ms || !quantize_ms) return XSV_ERR_ARG;
  if (ctx->broken) return XSV_ERR_HIP;
  if (hipStreamSynchronize(ctx->stream) != hipSuccess || hipStreamSynchronize(ctx->side) != hipSuccess) return hip_fail(ctx);
  double a = 0.0, b = 0.0;
  const size_t n = ctx->chain_used / 3;
  for (size_t i = 0; i < n; ++i) {
    float t0 = 0.f, t1 = 0.f;
    hipEvent_t* e = &ctx->chain_events[3 * i];
    if (hipEventElapsedTime(&t0, e[0], e[1]) != hipSuccess || hipEventElapsedTime(&t1, e[1], e[2]) != hipSuccess)
      return hip_fail(ctx);
    a += t0;
    b += t1;
  }
  *steps = (int32_t)n;
  *score_prune_ms = n ? (float)(a / n) : 0.f;
  *quantize_ms = n ? (float)(b / n) : 0.f;
  ctx->chain_used = 0;
  return XSV_OK;
}

int xsv_last_attend_workgroups(xsv_ctx* ctx, int32_t* workgroups) {
  if (!ctx || !workgroups) return XSV_ERR_ARG;
  *workgroups = ctx->last_attend_wgs;
  return XSV_OK;
}

int xsv_set_short_range(xsv_ctx* ctx, int percent) {
  if (!ctx || percent < -1 || percent > 100) return XSV_ERR_ARG;
  ctx->short_pct = percent;
  return XSV_OK;
}

int xsv_settled_blocks(xsv_ctx* ctx, int layer, int32_t* settled, int32_t* total) {
  int rc = check_layer(ctx, layer);
  if (rc != XSV_OK) return rc;
  if (!settled || !total) return XSV_ERR_ARG;
  if ((rc = settle_layer(ctx, layer)) != XSV_OK) return rc;
  const size_t per_layer = (size_t)ctx->cfg.n_heads * (ctx->pool.Tcap / kTile);
  std::vector<uint8_t> flags(per_layer);
  if (hipMemcpyAsync(flags.data(), ctx->stable_flag + (size_t)layer * per_layer, per_layer, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
      hipStreamSynchronize(ctx->stream) != hipSuccess)
    return hip_fail(ctx);
  int32_t count = 0;
  for (uint8_t f : flags) count += f != 0;
  *settled = count;
  *total = ctx->cfg.n_heads * ((ctx->layers[layer].T + kTile - 1) / kTile);
  return XSV_OK;
}

int xsv_set_frame_tile_cost(xsv_ctx* ctx, int percent) {
  if (!ctx || percent < 25 || percent > 400) return XSV_ERR_ARG;
  ctx->frame_tile_cost = percent;
  return XSV_OK;
}

int xsv_set_side_cus(xsv_ctx* ctx, int compute_units) {
  if (!ctx || compute_units < -1 || compute_units > ctx->n_cu / 2) return XSV_ERR_ARG;
  ctx->side_cus = compute_units;
  return XSV_OK;
}

int xsv_key_ranges(int cache_tiles, int frame_tiles, int ranges, int last_percent, int frame_tile_cost, int32_t* begin) {
  if (!begin || cache_tiles < 0 || frame_tiles < 0 || ranges < 1 || ranges > kMaxPieces || ranges > cache_tiles + frame_tiles ||
      last_percent < 1 || last_percent > 100 || frame_tile_cost < 25 || frame_tile_cost > 400)
    return XSV_ERR_ARG;
  range_starts(cache_tiles, frame_tiles, ranges, last_percent, frame_tile_cost, begin);
  return XSV_OK;
}

int xsv_step_plan(const xsv_config* cfg, int cache_tokens, int frames_seen, int32_t* middle, int32_t* keep, int32_t* new_len) {
  if (!cfg || cfg->tokens_per_frame < 1 || cfg->budget < 0 || cache_tokens < 0 || frames_seen < 0) return XSV_ERR_ARG;
  LayerState L;
  L.T = cache_tokens;
  L.frames = frames_seen;
  const PrunePlan p = plan_for(*cfg, L);
  if (middle) *middle = p.P;
  if (keep) *keep = p.k;
  if (new_len) *new_len = p.Tn;
  return XSV_OK;
}

int xsv_line_partition(int64_t units, int tiles, int workgroups, int workgroup, int64_t* begin, int64_t* end, int64_t unit,
                       int32_t* first, int32_t* last) {
  if (units < 1 || tiles < 1 || workgroups < 1 || workgroup < 0 || workgroup >= workgroups || unit < 0 || unit >= units ||
      units > (1ll << 40) / tiles)
    return XSV_ERR_ARG;
  long long b = 0, e = 0;
  int f = 0, l = 0;
  partition_query(units, tiles, workgroups, workgroup, &b, &e);
  partition_unit_query(units, tiles, workgroups, (int)unit, &f, &l);
  if (begin) *begin = b;
  if (end) *end = e;
  if (first) *first = f;
  if (last) *last = l;
  return XSV_OK;
}

int xsv_set_attend_variant(xsv_ctx* ctx, int variant) {
  if (!ctx || variant < 0 || variant > 3) return XSV_ERR_ARG;
  ctx->attend_variant = variant;
  return XSV_OK;
}

int xsv_dequant_attend(xsv_ctx* ctx, int layer, xsv_tensor q, xsv_tensor k_new, xsv_tensor v_new, void* out) {
  int rc = check_layer(ctx, layer);
  if (rc != XSV_OK) return rc;
  if (ctx->layers[layer].phase != kIdle) return XSV_ERR_STATE;
  if ((rc = check_capacity(ctx, layer)) != XSV_OK) return rc;
  if ((rc = join_layers(ctx, layer, 1)) != XSV_OK) return rc;
  void* outs[1] = {out};
  return do_attend(ctx, layer, 1, &q, &k_new, &v_new, outs, ctx->splits_single, 0);
}

int xsv_frame_attend(xsv_ctx* ctx, xsv_tensor q, xsv_tensor k, xsv_tensor v, void* out) {
  if (!ctx) return XSV_ERR_ARG;
  if (ctx->broken) return XSV_ERR_HIP;
  if (!tensor_ok(q) || !tensor_ok(k) || !tensor_ok(v) || !out) return XSV_ERR_ARG;
  void* outs[1] = {out};
  return do_attend(ctx, 0, 1, &q, &k, &v, outs, ctx->splits_single, 0, true);
}

int xsv_score_prune(xsv_ctx* ctx, int layer, xsv_tensor q) {
  int rc = check_layer(ctx, layer);
  if (rc != XSV_OK) return rc;
  if (ctx->layers[layer].phase != kAttended) return XSV_ERR_STATE;
  if (!tensor_ok(q)) return XSV_ERR_ARG;
  return do_score_prune(ctx, layer, 1, &q);
}

int xsv_quantize(xsv_ctx* ctx, int layer, xsv_tensor k_new, xsv_tensor v_new) {
  int rc = check_layer(ctx, layer);
  if (rc != XSV_OK) return rc;
  if (ctx->layers[layer].phase != kScored) return XSV_ERR_STATE;
  return do_quantize(ctx, layer, 1, &k_new, &v_new);
}

// attention on the context's stream, score → select → re-quantize concurrently on the side stream.
// overlap 1: on return the context's stream is ordered after both.  overlap 2: the context's stream
// only waits for a layer's chain when it next needs that layer (or in xsv_join).
static int step_layers(xsv_ctx* ctx, int layer0, int n_layers, const xsv_tensor* q, const xsv_tensor* k,
                       const xsv_tensor* v, void* const* out, int splits) {
  // (a one-buffer cache is rewritten in place by the chain, so the chain must not run beside the attention that reads it)
  const bool fork = ctx->overlap != 0 && ctx->pool.buffers == 2;
  {  // every tensor of the batch is checked before the first launch (the stages check again as they marshal)
    Batch probe;
    const int bad = fill_batch(ctx, probe, layer0, n_layers, q, k, v, out);
    if (bad != XSV_OK) return bad;
  }
  int rc = join_layers(ctx, layer0, n_layers, 2);  // the previous frame's chain wrote the cache read now
  if (rc != XSV_OK) return rc;
  if (fork) {
    if (hipEventRecord(ctx->ev_fork, ctx->stream) != hipSuccess || hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0) != hipSuccess)
      return hip_fail(ctx);
  }
  hipEvent_t cev[3] = {nullptr, nullptr, nullptr};
  if (ctx->timing) {
    while (ctx->chain_events.size() < ctx->chain_used + 3) {
      hipEvent_t e = nullptr;
      if (hipEventCreate(&e) != hipSuccess) return hip_fail(ctx);
      ctx->chain_events.push_back(e);
    }
    for (int i = 0; i < 3; ++i) cev[i] = ctx->chain_events[ctx->chain_used + i];
    ctx->chain_used += 3;
  }
  hipStream_t chain = fork ? ctx->side : ctx->stream;
  auto mark = [&](hipEvent_t e) { return !e || hipEventRecord(e, chain) == hipSuccess; };
  if (fork) {
    // the chain is enqueued first: its launches then do not queue up behind the host time of the
    // attention launches, and it starts as soon as the fork event fires
    ctx->work = ctx->side;
    if (!mark(cev[0])) return hip_fail(ctx);
    rc = do_score_prune(ctx, layer0, n_layers, q);
    if (!mark(cev[1])) return hip_fail(ctx);
    ctx->work = ctx->stream;
    if (rc == XSV_OK) {
      // The chain takes about the same time whatever the attention launch takes, so the longer the
      // attention, the smaller the share of the chip worth leaving to it: a quarter of the compute units
      // up to about 24 key tiles per attention workgroup, an eighth beyond.
      int spare = ctx->side_cus;
      if (spare < 0) {
        const xsv_config& c = ctx->cfg;
        const int rows = attend_rows_per_workgroup(ctx->attend_variant);
        const long long units = (long long)((c.tokens_per_frame + rows - 1) / rows) * c.n_heads * n_layers;
        const long long tiles = (ctx->layers[layer0].T + kTile - 1) / kTile + (c.tokens_per_frame + kTile - 1) / kTile;
        const int per_cu = ctx->attend_variant >= 2 ? 1 : 2;
        const long long wgs = (long long)per_cu * (ctx->n_cu - ctx->n_cu / 4);
        spare = units * tiles > 24 * wgs ? ctx->n_cu / 8 : ctx->n_cu / 4;
      }
      rc = do_attend(ctx, layer0, n_layers, q, k, v, out, splits, spare);
    }
    ctx->work = ctx->side;
    if (rc == XSV_OK) rc = do_quantize(ctx, layer0, n_layers, k, v);
    if (!mark(cev[2])) return hip_fail(ctx);
    ctx->work = ctx->stream;
  } else {
    rc = do_attend(ctx, layer0, n_layers, q, k, v, out, splits, 0);
    if (!mark(cev[0])) return hip_fail(ctx);
    if (rc == XSV_OK) rc = do_score_prune(ctx, layer0, n_layers, q);
    if (!mark(cev[1])) return hip_fail(ctx);
    if (rc == XSV_OK) rc = do_quantize(ctx, layer0, n_layers, k, v);
    if (!mark(cev[2])) return hip_fail(ctx);
  }
  if (fork && ctx->overlap == 2) {
    if (hipEventRecord(ctx->ev_chain[layer0], ctx->side) != hipSuccess) return hip_fail(ctx);
    ctx->seq[layer0] = ctx->next_seq++;
    for (int l = layer0; l < layer0 + n_layers; ++l) ctx->pending[l] = layer0;
  } else if (fork) {  // join even after an error so the streams stay ordered
    if (hipEventRecord(ctx->ev_join, ctx->side) != hipSuccess || hipStreamWaitEvent(ctx->stream, ctx->ev_join, 0) != hipSuccess)
      return hip_fail(ctx);
  }
  return rc;
}

int xsv_step(xsv_ctx* ctx, int layer, xsv_tensor q, xsv_tensor k_new, xsv_tensor v_new, void* out) {
  int rc = check_layer(ctx, layer);
  if (rc != XSV_OK) return rc;
  if (ctx->layers[layer].phase != kIdle) return XSV_ERR_STATE;
  if ((rc = check_capacity(ctx, layer)) != XSV_OK) return rc;
  if (!tensor_ok(q) || !tensor_ok(k_new) || !tensor_ok(v_new) || !out) return XSV_ERR_ARG;
  void* outs[1] = {out};
  return step_layers(ctx, layer, 1, &q, &k_new, &v_new, outs, ctx->splits_single);
}

int xsv_step_all_layers(xsv_ctx* ctx, const xsv_tensor* q, const xsv_tensor* k_new, const xsv_tensor* v_new,
                        void* const* out) {
  if (!ctx || !q || !k_new || !v_new || !out) return XSV_ERR_ARG;
  if (ctx->broken) return XSV_ERR_HIP;
  const int L = ctx->cfg.n_layers;
  if (L > kMaxBatch) return XSV_ERR_UNSUPPORTED;
  for (int l = 0; l < L; ++l) {
    const LayerState& a = ctx->layers[l];
    if (a.phase != kIdle || a.T != ctx->layers[0].T || a.frames != ctx->layers[0].frames) return XSV_ERR_STATE;
    if (!tensor_ok(q[l]) || !tensor_ok(k_new[l]) || !tensor_ok(v_new[l]) || !out[l]) return XSV_ERR_ARG;
  }
  int rc = check_capacity(ctx, 0);
  if (rc != XSV_OK) return rc;
  return step_layers(ctx, 0, L, q, k_new, v_new, out, ctx->splits_batched);
}

int xsv_set_overlap(xsv_ctx* ctx, int mode) {
  if (!ctx || mode < 0 || mode > 2) return XSV_ERR_ARG;
  const int rc = join_layers(ctx, 0, ctx->cfg.n_layers);
  if (rc != XSV_OK) return rc;
  ctx->overlap = mode;
  return XSV_OK;
}

int xsv_cache_len(xsv_ctx* ctx, int layer, int32_t* T) {
  int rc = check_layer(ctx, layer);
  if (rc != XSV_OK) return rc;
  if (!T) return XSV_ERR_ARG;
  *T = ctx->layers[layer].T;
  return XSV_OK;
}


int xsv_cache_export(xsv_ctx* ctx, int layer, uint8_t* k_codes, float* k_scale, float* k_zero, uint8_t* v_codes,
                     float* v_scale, float* v_zero, uint16_t* k_bf16, uint16_t* v_bf16, int32_t* token_frame,
                     int32_t* token_index) {
  int rc = check_layer(ctx, layer);
  if (rc != XSV_OK) return rc;
  const LayerState& L = ctx->layers[layer];
  if (L.phase != kIdle) return XSV_ERR_STATE;
  if ((rc = settle_layer(ctx, layer)) != XSV_OK) return rc;
  const xsv_config& c = ctx->cfg;
  const bool quant = c.kv_bits != 16;
  if (!quant && (k_codes || k_scale || k_zero || v_codes || v_scale || v_zero)) return XSV_ERR_ARG;
  const int T = L.T, H = c.n_heads, G = c.group_size;
  if (T == 0) return XSV_OK;
  const size_t n_el = (size_t)H * T * kD, n_kp = (size_t)H * ((T + G - 1) / G) * kD, n_vp = (size_t)H * T * (kD / G);
  Temp tmp;
  UnpackArgs u{};
  u.pool = ctx->pool; u.buf = L.buf; u.layer = layer; u.T = T;
  bool ok = true;
  auto want = [&](auto*& dev, const void* host, size_t count) {
    using P = std::remove_reference_t<decltype(dev)>;
    dev = nullptr;
    if (host) { dev = tmp.get<std::remove_pointer_t<P>>(count); ok = ok && dev != nullptr; }
  };
  want(u.k_codes, k_codes, n_el); want(u.v_codes, v_codes, n_el);
  want(u.k_scale, k_scale, n_kp); want(u.k_zero, k_zero, n_kp);
  want(u.v_scale, v_scale, n_vp); want(u.v_zero, v_zero, n_vp);
  want(u.k_bf16, k_bf16, n_el); want(u.v_bf16, v_bf16, n_el);
  if (!ok) return XSV_ERR_OOM;
  if (launch_unpack(u, ctx->stream) != hipSuccess) return hip_fail(ctx);
  bool good = true;
  auto back = [&](void* host, const void* dev, size_t bytes) {
    if (host && good) good = hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, ctx->stream) == hipSuccess;
  };
  back(k_codes, u.k_codes, n_el); back(v_codes, u.v_codes, n_el);
  back(k_scale, u.k_scale, n_kp * 4); back(k_zero, u.k_zero, n_kp * 4);
  back(v_scale, u.v_scale, n_vp * 4); back(v_zero, u.v_zero, n_vp * 4);
  back(k_bf16, u.k_bf16, n_el * 2); back(v_bf16, u.v_bf16, n_el * 2);
  const LayerCache lc = layer_cache(ctx->pool, L.buf, layer);
  for (int st = 0; st < ctx->pool.sets; ++st) {  // device rows are Tcap apart, host rows T
    back(token_frame ? token_frame + (size_t)st * T : nullptr, lc.tok_frame + (size_t)st * ctx->pool.Tcap, (size_t)T * 4);
    back(token_index ? token_index + (size_t)st * T : nullptr, lc.tok_index + (size_t)st * ctx->pool.Tcap, (size_t)T * 4);
  }
  if (!good || hipStreamSynchronize(ctx->stream) != hipSuccess) return hip_fail(ctx);
  return XSV_OK;
}

int xsv_cache_import(xsv_ctx* ctx, int layer, int32_t T, int32_t frames_seen, const uint8_t* k_codes,
                     const float* k_scale, const float* k_zero, const uint8_t* v_codes, const float* v_scale,
                     const float* v_zero, const uint16_t* k_bf16, const uint16_t* v_bf16, const int32_t* token_frame,
                     const int32_t* token_index) {
  int rc = check_layer(ctx, layer);
  if (rc != XSV_OK) return rc;
  LayerState& L = ctx->layers[layer];
  const xsv_config& c = ctx->cfg;
  const CachePool& p = ctx->pool;
  if (L.phase != kIdle) return XSV_ERR_STATE;
  if (T < 0 || T > p.Tcap || frames_seen < 0 || (T > 0 && frames_seen < 1) || (T > 0 && T < c.tokens_per_frame)) return XSV_ERR_ARG;
  const bool quant = c.kv_bits != 16;
  if (T > 0) {
    if (quant && (!k_codes || !k_scale || !k_zero || !v_codes || !v_scale || !v_zero)) return XSV_ERR_ARG;
    if (!quant && (!k_bf16 || !v_bf16)) return XSV_ERR_ARG;
    if (!token_frame || !token_index) return XSV_ERR_ARG;
  }
  const int H = c.n_heads, G = c.group_size, bits = c.kv_bits;
  const LayerCache lc = layer_cache(p, L.buf, layer);
  if ((rc = settle_layer(ctx, layer)) != XSV_OK) return rc;
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) return hip_fail(ctx);
  // pack on the host into the library's private layout (layout marshalling only)
  const size_t row_bytes = p.code_row_bytes();
  std::vector<uint8_t> kc((size_t)H * p.Tcap * row_bytes, 0), vc((size_t)H * p.Tcap * row_bytes, 0);
  const int ng = (T + G - 1) / G;
  for (int h = 0; h < H; ++h)
    for (int t = 0; t < T; ++t)
      for (int ch = 0; ch < kD; ++ch) {
        const size_t src = ((size_t)h * T + t) * kD + ch;
        if (quant) {
          const size_t kbit = (size_t)ch * bits, vbit = (size_t)(t % kTile) * bits;
          kc[((size_t)h * p.Tcap + t) * row_bytes + kbit / 8] |= (uint8_t)((k_codes[src] & ((1 << bits) - 1)) << (kbit % 8));
          vc[((size_t)h * p.Tcap + (size_t)(t / kTile) * kTile + ch) * row_bytes + vbit / 8] |=
              (uint8_t)((v_codes[src] & ((1 << bits) - 1)) << (vbit % 8));
        } else {
          std::memcpy(&kc[((size_t)h * p.Tcap + t) * row_bytes + ch * 2], &k_bf16[src], 2);
          std::memcpy(&vc[((size_t)h * p.Tcap + (size_t)(t / kTile) * kTile + ch) * row_bytes + (t % kTile) * 2], &v_bf16[src], 2);
        }
      }
  bool good = hipMemcpy(lc.kc, kc.data(), kc.size(), hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(lc.vc, vc.data(), vc.size(), hipMemcpyHostToDevice) == hipSuccess;
  if (quant && T > 0) {
    std::vector<float> ks(p.kparam_slab(), 0.f), kz(p.kparam_slab(), 0.f), vs(p.vparam_slab(), 0.f), vz(p.vparam_slab(), 0.f);
    for (int h = 0; h < H; ++h) {
      for (int g = 0; g < ng; ++g)
        for (int ch = 0; ch < kD; ++ch) {
          ks[((size_t)h * (p.Tcap / G) + g) * kD + ch] = k_scale[((size_t)h * ng + g) * kD + ch];
          kz[((size_t)h * (p.Tcap / G) + g) * kD + ch] = k_zero[((size_t)h * ng + g) * kD + ch];
        }
      for (int t = 0; t < T; ++t)
        for (int g = 0; g < kD / G; ++g) {
          vs[((size_t)h * p.Tcap + t) * (kD / G) + g] = v_scale[((size_t)h * T + t) * (kD / G) + g];
          vz[((size_t)h * p.Tcap + t) * (kD / G) + g] = v_zero[((size_t)h * T + t) * (kD / G) + g];
        }
    }
    good = good && hipMemcpy(lc.ks, ks.data(), ks.size() * 4, hipMemcpyHostToDevice) == hipSuccess &&
           hipMemcpy(lc.kz, kz.data(), kz.size() * 4, hipMemcpyHostToDevice) == hipSuccess &&
           hipMemcpy(lc.vs, vs.data(), vs.size() * 4, hipMemcpyHostToDevice) == hipSuccess &&
           hipMemcpy(lc.vz, vz.data(), vz.size() * 4, hipMemcpyHostToDevice) == hipSuccess;
  }
  for (int st = 0; T > 0 && st < p.sets; ++st)
    good = good && hipMemcpy(lc.tok_frame + (size_t)st * p.Tcap, token_frame + (size_t)st * T, (size_t)T * 4, hipMemcpyHostToDevice) == hipSuccess &&
           hipMemcpy(lc.tok_index + (size_t)st * p.Tcap, token_index + (size_t)st * T, (size_t)T * 4, hipMemcpyHostToDevice) == hipSuccess;
  {  // nothing is known about the imported blocks
    const size_t per_layer = (size_t)c.n_heads * (p.Tcap / kTile);
    good = good && hipMemset(ctx->stable_flag + (size_t)layer * per_layer, 0, per_layer) == hipSuccess;
  }
  if (!good) return hip_fail(ctx);
  L.T = T;
  L.frames = frames_seen;
  L.last_P = 0;
  L.last_keep = 0;
  return XSV_OK;
}

int xsv_last_selection(xsv_ctx* ctx, int layer, int32_t* n_scores, float* scores, int32_t* n_keep, int32_t* keep) {
  int rc = check_layer(ctx, layer);
  if (rc != XSV_OK) return rc;
  const LayerState& L = ctx->layers[layer];
  if ((rc = settle_layer(ctx, layer)) != XSV_OK) return rc;
  if (n_scores) *n_scores = L.last_P;
  if (n_keep) *n_keep = L.last_keep;
  bool good = true;
  const int sets = ctx->ws.sets;
  for (int st = 0; st < sets && good; ++st) {  // device lists are scores_stride apart, host lists packed
    const size_t row = (list_index(sets, layer, 0) + st) * ctx->ws.scores_stride;
    if (scores && L.last_P > 0)
      good = hipMemcpyAsync(scores + (size_t)st * L.last_P, ctx->ws.scores + row, (size_t)L.last_P * 4, hipMemcpyDeviceToHost,
                            ctx->stream) == hipSuccess;
    if (keep && L.last_keep > 0 && good)
      good = hipMemcpyAsync(keep + (size_t)st * L.last_keep, ctx->ws.keep + row, (size_t)L.last_keep * 4, hipMemcpyDeviceToHost,
                            ctx->stream) == hipSuccess;
  }
  if (!good || hipStreamSynchronize(ctx->stream) != hipSuccess) return hip_fail(ctx);
  return XSV_OK;
}

// ---- stateless entry points: a throw-away one-layer context around the same kernels ----------------

static int quantize_plain(void* hip_stream, const void* x, int H, int T, int d, int bits, int G, void* codes, float* scale,
                          float* zero, bool keys) {
  if (!x || !codes || !scale || !zero || H < 1 || T < 1) return XSV_ERR_ARG;
  if (d != kD) return XSV_ERR_UNSUPPORTED;
  if (bits != 2 && bits != 4) return XSV_ERR_ARG;
  if (G != 32 && G != 64) return XSV_ERR_UNSUPPORTED;
  xsv_config c{};
  c.n_layers = 1; c.n_heads = H; c.head_dim = d; c.tokens_per_frame = T; c.n_special = 0; c.budget = 0;
  c.kv_bits = bits; c.group_size = G; c.pool_size = 1; c.max_frames = 1;
  xsv_ctx* ctx = nullptr;
  int rc = xsv_create(&c, hip_stream, &ctx);
  if (rc != XSV_OK) return rc;
  // the whole tensor is "the current frame" of an empty cache: keep everything, quantize
  const xsv_tensor t{x, (int64_t)T * d, d};
  ctx->layers[0].phase = kAttended;
  rc = do_score_prune(ctx, 0, 1, nullptr);
  if (rc == XSV_OK) rc = do_quantize(ctx, 0, 1, &t, &t);
  if (rc == XSV_OK) {
    UnpackArgs u{};
    u.pool = ctx->pool; u.buf = ctx->layers[0].buf; u.layer = 0; u.T = T;
    if (keys) { u.k_codes = static_cast<uint8_t*>(codes); u.k_scale = scale; u.k_zero = zero; }
    else { u.v_codes = static_cast<uint8_t*>(codes); u.v_scale = scale; u.v_zero = zero; }
    if (launch_unpack(u, ctx->stream) != hipSuccess) rc = XSV_ERR_HIP;
  }
  xsv_destroy(ctx);  // synchronizes
  return rc;
}

int xsv_quantize_k(void* hip_stream, const void* k_bf16, int H, int T, int d, int bits, int G, void* codes_u8,
                   float* scale, float* zero) {
  return quantize_plain(hip_stream, k_bf16, H, T, d, bits, G, codes_u8, scale, zero, true);
}

int xsv_quantize_v(void* hip_stream, const void* v_bf16, int H, int T, int d, int bits, int G, void* codes_u8,
                   float* scale, float* zero) {
  return quantize_plain(hip_stream, v_bf16, H, T, d, bits, G, codes_u8, scale, zero, false);
}

int xsv_score(void* hip_stream, xsv_tensor q, const void* k_mid_bf16, int H, int n, int n_s, int P, int d, int g,
              float* scores) {
  if (!tensor_ok(q) || !k_mid_bf16 || !scores || H < 1 || n < 1 || n_s < 0 || n_s > n || P < 1 || g < 1) return XSV_ERR_ARG;
  if (d != kD) return XSV_ERR_UNSUPPORTED;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  Temp tmp;
  ScoreArgs s{};
  s.pool.H = H; s.pool.L = 1; s.pool.bits = 16; s.pool.G = 64; s.pool.Tcap = round_up(P, kTile);
  s.b.n_layers = 1; s.b.layer0 = 0;
  s.b.q[0] = static_cast<const uint16_t*>(q.ptr);
  s.b.q_sh = q.stride_head; s.b.q_st = q.stride_token;
  s.ws.qpart_rows = H * kPoolSeg;
  s.ws.sets = 1;
  s.ws.qpart = tmp.get<float>((size_t)s.ws.qpart_rows * kD);
  if (!s.ws.qpart) return XSV_ERR_OOM;
  s.ws.scores = scores;
  s.ws.scores_stride = P;
  s.Tc = P; s.n = n; s.n_special = n_s; s.pool_size = g; s.T_first = 0; s.P = P;
  s.k_plain = static_cast<const uint16_t*>(k_mid_bf16);
  if (launch_pool_query(s, stream) != hipSuccess || launch_score(s, stream) != hipSuccess) return XSV_ERR_HIP;
  return hipStreamSynchronize(stream) == hipSuccess ? XSV_OK : XSV_ERR_HIP;
}

// ---- the entry point that allocates nothing ---------------------------------------------------------
// xsv_score needs one scratch buffer: the per-head partial sums of the pooled query that pool_query_kernel
// writes and score_kernel folds.  Here it lives in a file-scope device array instead of a hipMalloc'ed
// temporary.  The array's name is only a host-side handle: its device address is looked up once per device
// (each device holds its own copy) and that pointer is what the kernels get.
constexpr int kNoAllocMaxHeads = XSV_NOALLOC_MAX_HEADS;
constexpr int kNoAllocMaxDevices = 64;
static __device__ __align__(256) float scratch[kNoAllocMaxHeads * kPoolSeg * kD];

static std::mutex g_scratch_mutex;
static float* g_scratch_ptr[kNoAllocMaxDevices];  // device address of `scratch` on device i, once resolved

// The current device's copy of `scratch`; nullptr (and *rc set) on failure.
static float* scratch_of_current_device(int* rc) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); *rc = XSV_ERR_HIP; return nullptr; }
  if (dev < 0 || dev >= kNoAllocMaxDevices) { *rc = XSV_ERR_UNSUPPORTED; return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      *rc = XSV_ERR_HIP;
      return nullptr;
    }
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  return g_scratch_ptr[dev];
}

int xsv_score_noalloc(void* hip_stream, xsv_tensor q, const void* k_mid_bf16, int H, int n, int n_s, int P, int d, int g,
                      float* scores) {
  if (!tensor_ok(q) || !k_mid_bf16 || !scores || H < 1 || n < 1 || n_s < 0 || n_s > n || P < 1 || g < 1) return XSV_ERR_ARG;
  if (d != kD) return XSV_ERR_UNSUPPORTED;
  if (H > kNoAllocMaxHeads) return XSV_ERR_UNSUPPORTED;  // the scratch array holds kNoAllocMaxHeads partial sums
  int rc = XSV_OK;
  float* qpart = scratch_of_current_device(&rc);
  if (!qpart) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  ScoreArgs s{};
  s.pool.H = H; s.pool.L = 1; s.pool.bits = 16; s.pool.G = 64; s.pool.Tcap = round_up(P, kTile);
  s.b.n_layers = 1; s.b.layer0 = 0;
  s.b.q[0] = static_cast<const uint16_t*>(q.ptr);
  s.b.q_sh = q.stride_head; s.b.q_st = q.stride_token;
  s.ws.qpart_rows = H * kPoolSeg;
  s.ws.sets = 1;
  s.ws.qpart = qpart;  // every entry a call reads is written by that call's pooling kernel first: nothing to clear
  s.ws.scores = scores;
  s.ws.scores_stride = P;
  s.Tc = P; s.n = n; s.n_special = n_s; s.pool_size = g; s.T_first = 0; s.P = P;
  s.k_plain = static_cast<const uint16_t*>(k_mid_bf16);
  if (launch_pool_query(s, stream) != hipSuccess || launch_score(s, stream) != hipSuccess) return XSV_ERR_HIP;
  return XSV_OK;
}

int xsv_topk_keep(void* hip_stream, const float* scores, int P, int k, int T_first, int T_cur, int32_t* keep) {
  if (!keep || P < 0 || k < 0 || k > P || T_first < 0 || T_cur < 0 || (P > 0 && !scores)) return XSV_ERR_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (k == 0 || k == P) {
    e = launch_fill_keep(keep, 0, 1, T_first, P, T_cur, k == P, stream);
  } else {
    SelectArgs s{};
    s.scores = scores; s.keep = keep; s.n_lists = 1; s.P = P; s.k = k; s.T_first = T_first; s.T_cur = T_cur;
    e = launch_select(s, stream);
  }
  if (e != hipSuccess) return XSV_ERR_HIP;
  return hipStreamSynchronize(stream) == hipSuccess ? XSV_OK : XSV_ERR_HIP;
}

}  // extern "C"
