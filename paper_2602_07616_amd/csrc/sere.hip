// Host side of the C ABI declared in include/sere.h: argument validation,
// workspace layout and kernel launches.  Nothing here synchronises the device.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>

#include "common.hpp"
#include "ffn_generic.hpp"
#include "ffn_mfma.hpp"
#include "route_kernels.hpp"
#include "similarity_kernels.hpp"

namespace sere {

// ---------------------------------------------------------------- layout ---
struct Layout {
  size_t list_key, list_id, topk_ids, topk_w, rerouted, cnt_before, cnt_after, primary, num_active, offsets,
      sorted_token, sorted_slot, slot_pos, work_expert, work_off, work_cnt, n_work, ticket, h, y, total;
  int rows;      // A + n_sh*T rows of the sorted slot list
  int ksplit;    // slices of d_m in the down projection
  int max_work;  // upper bound on FFN work items (the FFN grids are sized for it)
};

static size_t align_up(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

// bf16 down projection: d_m is cut into slices of at most 2048 so that one
// wavefront streams at most 64 KB of weights whatever the expert width
static int down_ksplit(const sere_config& c) {
  return c.dtype == SERE_BF16 ? (c.inter + 2047) / 2048 : 1;
}

static Layout make_layout(const sere_config& c) {
  Layout l{};
  const size_t T = c.num_tokens, M = c.num_experts, K = c.top_k, A = T * K;
  const size_t R = A + static_cast<size_t>(c.num_shared) * T;
  // an expert's rows are cut into items of <= kItemRows: at most one partial item per expert, and
  // never more items than rows (small batches: far fewer than M)
  const size_t routed_items = M + A / kItemRows < A ? M + A / kItemRows : A;
  const size_t W = routed_items + c.num_shared * ((T + kItemRows - 1) / kItemRows);
  l.rows = static_cast<int>(R);
  l.ksplit = down_ksplit(c);
  l.max_work = static_cast<int>(W);
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o = align_up(o + bytes);
    return at;
  };
  const size_t lists = (M + 15) / 16;  // sorted 16-expert lists per token
  l.list_key = take(T * lists * 16 * sizeof(uint64_t));
  l.list_id = take(T * lists * 16);
  l.topk_ids = take(A * 4);
  l.topk_w = take(A * 4);
  l.rerouted = take(A * 4);
  l.cnt_before = take(M * 4);
  l.cnt_after = take(M * 4);
  l.primary = take(M * 4);
  l.num_active = take(2 * 4);
  l.offsets = take((M + 1) * 4);
  l.sorted_token = take(R * 4);
  l.sorted_slot = take(A * 4);
  l.slot_pos = take(A * 4);
  l.work_expert = take(W * 4);
  l.work_off = take(W * 4);
  l.work_cnt = take(W * 4);
  l.n_work = take(8);
  l.ticket = take(4);
  l.h = take(R * c.inter * sizeof(float));
  l.y = take(static_cast<size_t>(l.ksplit) * R * c.hidden * sizeof(float));
  l.total = o;
  return l;
}

// ------------------------------------------------------------ validation ---
static int check_config(const sere_config* c) {
  if (c == nullptr) return SERE_ERR_NULL_PTR;
  if (c->dtype != SERE_F32 && c->dtype != SERE_BF16) return SERE_ERR_BAD_DTYPE;
  if ((c->flags & ~(SERE_FLAG_RESIDUAL | SERE_FLAG_SIM_COSINE | SERE_FLAG_SIM_CKA_LINEAR)) != 0) return SERE_ERR_BAD_FLAGS;
  if ((c->flags & SERE_FLAG_SIM_COSINE) && (c->flags & SERE_FLAG_SIM_CKA_LINEAR)) return SERE_ERR_BAD_FLAGS;
  if (c->num_tokens < 1 || c->num_tokens > SERE_MAX_TOKENS) return SERE_ERR_BAD_SHAPE;
  if (c->hidden < 64 || c->hidden % 64 != 0 || c->hidden > (1 << 16)) return SERE_ERR_BAD_SHAPE;
  if (c->inter < 64 || c->inter % 64 != 0 || c->inter > (1 << 18)) return SERE_ERR_BAD_SHAPE;
  if (c->num_experts < 1 || c->num_experts > SERE_MAX_EXPERTS) return SERE_ERR_BAD_SHAPE;
  if (c->num_shared < 0 || c->num_shared > SERE_MAX_SHARED) return SERE_ERR_BAD_SHAPE;
  if (c->top_k < 1 || c->top_k > c->num_experts) return SERE_ERR_BAD_TOPK;
  if (c->select_top_k < 1 || c->select_top_k > c->top_k) return SERE_ERR_BAD_TOPK;
  if (!std::isfinite(c->threshold)) return SERE_ERR_NONFINITE_THRESHOLD;
  // one work item per 32 rows of the sorted slot list at most, and the FFN grids carry the items in
  // their y dimension (at most 65535)
  const int64_t rows = static_cast<int64_t>(c->num_tokens) * (c->top_k + c->num_shared);
  if (rows > SERE_MAX_ROWS) return SERE_ERR_BAD_SHAPE;
  return SERE_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct PtrCheck {
  int status = SERE_OK;
  void need(const void* p) {
    if (status != SERE_OK) return;
    if (p == nullptr)
      status = SERE_ERR_NULL_PTR;
    else if (!aligned16(p))
      status = SERE_ERR_MISALIGNED;
  }
  void optional(const void* p) {
    if (status == SERE_OK && p != nullptr && !aligned16(p)) status = SERE_ERR_MISALIGNED;
  }
};

static void check_route_out(PtrCheck& pc, const sere_route_out* o) {
  if (o == nullptr) return;
  pc.optional(o->topk_ids);
  pc.optional(o->topk_weights);
  pc.optional(o->rerouted_ids);
  pc.optional(o->count_before);
  pc.optional(o->count_after);
  pc.optional(o->primary_mask);
  pc.optional(o->num_active);
  pc.optional(o->expert_offsets);
  pc.optional(o->sorted_token);
  pc.optional(o->sorted_slot);
}

static int check_workspace(const Layout& l, const void* ws, size_t bytes) {
  if (ws == nullptr) return SERE_ERR_NULL_PTR;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return SERE_ERR_MISALIGNED;
  if (bytes < l.total) return SERE_ERR_WORKSPACE_TOO_SMALL;
  return SERE_OK;
}

// ---------------------------------------------------------------- timing ---
struct Timing {
  bool enabled = false;
  int n = 0;
  int created = 0;
  hipEvent_t start[SERE_TIMING_MAX_RECORDS];
  hipEvent_t stop[SERE_TIMING_MAX_RECORDS];
  int stage[SERE_TIMING_MAX_RECORDS];
};
static Timing g_timing;

// Event pair for the next launch of `stage`, if timing is on and a record is free.
static bool timing_slot(int stage, hipEvent_t* start, hipEvent_t* stop) {
  Timing& t = g_timing;
  if (!t.enabled || t.n >= SERE_TIMING_MAX_RECORDS) return false;
  if (t.n >= t.created) {
    if (hipEventCreate(&t.start[t.created]) != hipSuccess) return false;
    if (hipEventCreate(&t.stop[t.created]) != hipSuccess) {
      (void)hipEventDestroy(t.start[t.created]);
      return false;
    }
    ++t.created;
  }
  t.stage[t.n] = stage;
  *start = t.start[t.n];
  *stop = t.stop[t.n];
  return true;
}

// One kernel launch of a stage.  With timing on, the two events are attached to the dispatch
// itself (they take the kernel's own start and end time stamps, as a profiler's kernel trace
// does), not recorded around it on the stream.
template <typename Kernel, typename... Args>
static void launch_stage(int stage, hipStream_t s, Kernel kernel, dim3 grid, dim3 block, Args... args) {
  hipEvent_t e0, e1;
  if (timing_slot(stage, &e0, &e1)) {
    hipExtLaunchKernelGGL(kernel, grid, block, 0, s, e0, e1, 0, args...);
    ++g_timing.n;
  } else {
    hipLaunchKernelGGL(kernel, grid, block, 0, s, args...);
  }
}

// --------------------------------------------------------------- launches ---
struct Pointers {
  uint64_t* list_key;
  uint8_t* list_id;
  int32_t* ticket;
  int32_t* topk_ids;
  float* topk_w;
  RouteArgs route;
  float* h;
  float* y;
};

static Pointers bind(const sere_config& c, const Layout& l, void* workspace, const sere_route_out* o) {
  char* ws = static_cast<char*>(workspace);
  auto pick = [&](void* user, size_t off) { return user != nullptr ? user : static_cast<void*>(ws + off); };
  static const sere_route_out none{};
  if (o == nullptr) o = &none;
  Pointers p{};
  p.list_key = reinterpret_cast<uint64_t*>(ws + l.list_key);
  p.list_id = reinterpret_cast<uint8_t*>(ws + l.list_id);
  p.ticket = reinterpret_cast<int32_t*>(ws + l.ticket);
  p.topk_ids = static_cast<int32_t*>(pick(o->topk_ids, l.topk_ids));
  p.topk_w = static_cast<float*>(pick(o->topk_weights, l.topk_w));
  RouteArgs& r = p.route;
  r.topk_ids = p.topk_ids;
  r.T = c.num_tokens;
  r.K = c.top_k;
  r.M = c.num_experts;
  r.S = c.select_top_k;
  r.n_sh = c.num_shared;
  r.rho = c.threshold;
  r.rerouted_ids = static_cast<int32_t*>(pick(o->rerouted_ids, l.rerouted));
  r.count_before = static_cast<int32_t*>(pick(o->count_before, l.cnt_before));
  r.count_after = static_cast<int32_t*>(pick(o->count_after, l.cnt_after));
  r.primary_mask = static_cast<int32_t*>(pick(o->primary_mask, l.primary));
  r.num_active = static_cast<int32_t*>(pick(o->num_active, l.num_active));
  r.expert_offsets = static_cast<int32_t*>(pick(o->expert_offsets, l.offsets));
  r.sorted_token = reinterpret_cast<int32_t*>(ws + l.sorted_token);  // holds shared rows too
  r.sorted_slot = static_cast<int32_t*>(pick(o->sorted_slot, l.sorted_slot));
  r.slot_pos = reinterpret_cast<int32_t*>(ws + l.slot_pos);
  r.work_expert = reinterpret_cast<int32_t*>(ws + l.work_expert);
  r.work_off = reinterpret_cast<int32_t*>(ws + l.work_off);
  r.work_cnt = reinterpret_cast<int32_t*>(ws + l.work_cnt);
  r.n_work = reinterpret_cast<int32_t*>(ws + l.n_work);
  // top-K: one workgroup (ids handed on through LDS) while the merge needs at most kTopkLoneThreads
  // threads; else groups of 256 threads while that gives at most kTopkMaxSmallGroups workgroups;
  // else groups of 1024
  const int lists = (c.num_experts + 15) / 16;
  const long long merge_threads = static_cast<long long>(c.num_tokens) * (lists <= 4 ? 4 : (lists <= 8 ? 8 : 16));
  r.topk_threads = (merge_threads > kTopkLoneThreads && merge_threads <= kTopkMaxSmallGroups * kTopkThreadsMulti)
                       ? kTopkThreadsMulti
                       : kRouteThreads;
  r.fine_items = kFineCutBlocks / (c.inter / (2 * kGateUpJ * kWavesPerBlock));
  // many rows per expert on average (prefill-sized batches): items of 64, 128 or 256 rows, served in
  // one pass over the weights each
  const long long slots = static_cast<long long>(c.num_tokens) * c.top_k;
  r.item_rows = slots >= 96ll * c.num_experts   ? kWideItemRows
                : slots >= 48ll * c.num_experts ? 4 * kItemRows
                : slots >= 24ll * c.num_experts ? 2 * kItemRows
                                                : kItemRows;
  p.h = reinterpret_cast<float*>(ws + l.h);
  p.y = reinterpret_cast<float*>(ws + l.y);
  return p;
}

static int hip_status() { return hipGetLastError() == hipSuccess ? SERE_OK : SERE_ERR_HIP; }

constexpr int kGateUpEightWavesRows = 12;  // average rows per expert from which on gate/up workgroups have 8 wavefronts
constexpr int kRouterMfmaTokens = 256;   // batches from this size on: router logits on the fp64 matrix cores

static int launch_router(const sere_config& c, const Pointers& p, const void* hidden,
                         const void* router_w, hipStream_t s) {
  const int lists = (c.num_experts + 15) / 16;
#define SERE_LAUNCH_ROUTER_TOKENS(TB)                                                                            \
  do {                                                                                                          \
    const dim3 grid(lists, (c.num_tokens + TB - 1) / TB);                                                       \
    if (c.dtype == SERE_F32)                                                                                    \
      launch_stage(SERE_STAGE_ROUTER, s, router_logits_tokens_kernel<SERE_F32, TB>, grid, dim3(256), hidden,    \
                   router_w, p.list_key, p.list_id, c.num_tokens, c.num_experts, c.hidden, p.ticket);           \
    else                                                                                                        \
      launch_stage(SERE_STAGE_ROUTER, s, router_logits_tokens_kernel<SERE_BF16, TB>, grid, dim3(256), hidden,   \
                   router_w, p.list_key, p.list_id, c.num_tokens, c.num_experts, c.hidden, p.ticket);           \
    return hip_status();                                                                                        \
  } while (0)
  if (c.num_tokens >= kRouterMfmaTokens) {  // a dense contraction: the fp64 matrix cores
    const dim3 grid(lists, (c.num_tokens + 15) / 16);
    if (c.dtype == SERE_F32)
      launch_stage(SERE_STAGE_ROUTER, s, router_logits_mfma_kernel<SERE_F32>, grid, dim3(256), hidden, router_w,
                   p.list_key, p.list_id, c.num_tokens, c.num_experts, c.hidden, p.ticket);
    else
      launch_stage(SERE_STAGE_ROUTER, s, router_logits_mfma_kernel<SERE_BF16>, grid, dim3(256), hidden, router_w,
                   p.list_key, p.list_id, c.num_tokens, c.num_experts, c.hidden, p.ticket);
    return hip_status();
  }
  // fewer tokens: two per fetch, if that still leaves a workgroup for every compute unit
  if (c.num_tokens >= 64 && lists * ((c.num_tokens + 1) / 2) >= 256) SERE_LAUNCH_ROUTER_TOKENS(2);
#undef SERE_LAUNCH_ROUTER_TOKENS
  const dim3 grid(lists, c.num_tokens);
  if (c.dtype == SERE_F32)
    launch_stage(SERE_STAGE_ROUTER, s, router_logits_kernel<SERE_F32>, grid, dim3(256), hidden, router_w, p.list_key,
                 p.list_id, c.num_tokens, c.num_experts, c.hidden, p.ticket);
  else
    launch_stage(SERE_STAGE_ROUTER, s, router_logits_kernel<SERE_BF16>, grid, dim3(256), hidden, router_w,
                 p.list_key, p.list_id, c.num_tokens, c.num_experts, c.hidden, p.ticket);
  return hip_status();
}

static int launch_route(const sere_config& c, const Pointers& p, bool with_topk, hipStream_t s,
                        const sere_route_out* o, size_t sorted_token_bytes) {
  if (with_topk) {
    // lanes per token = lists per token rounded up to 4, 8 or 16; K <= KS * lanes
    const int lists = (c.num_experts + 15) / 16;
    const int lp = lists <= 4 ? 4 : (lists <= 8 ? 8 : 16);
    const bool small_k = c.top_k <= 2 * lp;
    const dim3 grid((c.num_tokens * lp + p.route.topk_threads - 1) / p.route.topk_threads);
#define SERE_LAUNCH_TOPK(LP, KS, KEEP)                                                                          \
  launch_stage(SERE_STAGE_ROUTE, s, topk_route_kernel<LP, KS, KEEP>, grid, dim3(kRouteThreads), p.list_key, \
               p.list_id, p.topk_ids, p.topk_w, p.ticket, p.route)
    const bool half_lists = c.top_k <= 8;  // no list can give more than K entries
    if (lp == 4) {
      if (small_k) SERE_LAUNCH_TOPK(4, 2, 8); else SERE_LAUNCH_TOPK(4, 16, 16);
    } else if (lp == 8) {
      if (half_lists) SERE_LAUNCH_TOPK(8, 2, 8);
      else if (small_k) SERE_LAUNCH_TOPK(8, 2, 16);
      else SERE_LAUNCH_TOPK(8, 16, 16);
    } else {
      if (half_lists) SERE_LAUNCH_TOPK(16, 2, 8);
      else if (small_k) SERE_LAUNCH_TOPK(16, 2, 16);
      else SERE_LAUNCH_TOPK(16, 16, 16);
    }
#undef SERE_LAUNCH_TOPK
  } else {
    launch_stage(SERE_STAGE_ROUTE, s, route_kernel, dim3(1), dim3(kRouteThreads), p.route);
  }
  // the internal sorted_token list also carries the shared experts' rows; a
  // caller-visible copy holds the routed part only
  if (o != nullptr && o->sorted_token != nullptr)
    (void)hipMemcpyAsync(o->sorted_token, p.route.sorted_token, sorted_token_bytes, hipMemcpyDeviceToDevice, s);
  return hip_status();
}

static void launch_combine(const sere_config& c, const Layout& l, const Pointers& p, const void* hidden, void* out,
                           hipStream_t s) {
  CombineArgs ca{p.y, p.topk_w, p.route.slot_pos, (c.flags & SERE_FLAG_RESIDUAL) ? hidden : nullptr, out,
                 c.num_tokens, c.hidden, c.top_k, c.num_shared, l.ksplit, l.rows};
  const dim3 grid(static_cast<unsigned>((c.hidden + 255) / 256) * c.num_tokens);
  if (c.dtype == SERE_F32)
    launch_stage(SERE_STAGE_COMBINE, s, combine_kernel<SERE_F32>, grid, dim3(256), ca);
  else
    launch_stage(SERE_STAGE_COMBINE, s, combine_kernel<SERE_BF16>, grid, dim3(256), ca);
}

// fp32 layers: vector-ALU kernels.  bf16 layers: matrix-core kernels; `wide`: the variants for
// batches whose work items hold 128 rows (prefill-sized).
static void launch_gateup_down(int dtype, int inter, int hidden, int max_work, int ksplit, const FfnArgs& f,
                               hipStream_t s, bool wide = false, bool waves8 = false) {
  if (dtype == SERE_BF16 && wide) {
    constexpr int kGateUpPerBlock = kWideGateUpJ * kWideWaves, kDownPerBlock = kWideDownRows * kWideWaves;
    launch_stage(SERE_STAGE_GATE_UP, s, ffn_gateup_mfma_wide, dim3((inter + kGateUpPerBlock - 1) / kGateUpPerBlock, max_work),
                 dim3(kWideThreads), f);
    launch_stage(SERE_STAGE_DOWN, s, ffn_down_mfma_wide,
                 dim3(((hidden + kDownPerBlock - 1) / kDownPerBlock) * ksplit, max_work), dim3(kWideThreads), f);
    return;
  }
  if (dtype == SERE_F32) {
    launch_stage(SERE_STAGE_GATE_UP, s, ffn_gateup_generic<SERE_F32>, dim3((inter + kGenJB - 1) / kGenJB, max_work),
                 dim3(256), f);
    launch_stage(SERE_STAGE_DOWN, s, ffn_down_generic<SERE_F32>, dim3((hidden + kGenRB - 1) / kGenRB, max_work),
                 dim3(256), f);
  } else {
    if (waves8)
      launch_stage(SERE_STAGE_GATE_UP, s, ffn_gateup_mfma<8>, dim3(inter / (kGateUpJ * 8), max_work), dim3(512), f);
    else
      launch_stage(SERE_STAGE_GATE_UP, s, ffn_gateup_mfma<4>, dim3(inter / (kGateUpJ * 4), max_work), dim3(256), f);
    launch_stage(SERE_STAGE_DOWN, s, ffn_down_mfma,
                 dim3(((hidden + kDownRows * kWavesPerBlock - 1) / (kDownRows * kWavesPerBlock)) * ksplit, max_work),
                 dim3(256), f);
  }
}

static void launch_ffn(const sere_config& c, const Layout& l, const Pointers& p, const FfnArgs& f, void* out,
                       hipStream_t s) {
  const bool wide = c.dtype == SERE_BF16 && !f.split_h && p.route.item_rows >= 2 * kItemRows;
  // a dozen rows per expert and more: the gate/up workgroups of eight wavefronts (the routing
  // kernel's choice of the cut counts workgroups of four; both cuts halve alike)
  const bool waves8 = static_cast<long long>(c.num_tokens) * c.top_k >= kGateUpEightWavesRows * c.num_experts;
  launch_gateup_down(c.dtype, c.inter, c.hidden, l.max_work, l.ksplit, f, s, wide, waves8);
  launch_combine(c, l, p, f.hidden, out, s);
}

// --------------------------------------------------------- static scratch ---
// Workspace of sere_moe_decode_static: part of the library image, one copy per GPU.  In host code
// the array's name is only a handle for the runtime; the device address of the current GPU's copy
// comes from hipGetSymbolAddress and is what every kernel argument is built from.
static __device__ __align__(256) unsigned char scratch[SERE_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];  // per device, looked up on the first call with that device current

static int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SERE_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return SERE_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SERE_OK;
}

// wide experts: h keeps its bf16 rounding residual in a second plane (see decode())
static int wants_split_h(const sere_config& c) { return (c.dtype == SERE_BF16 && c.inter >= 4096) ? 1 : 0; }

static int decode(const sere_config* cfg, const void* hidden, const void* router_w, const void* w_gate_up,
                  const void* w_down, const void* shared_gate_up, const void* shared_down, const float* sim,
                  void* out, const sere_route_out* dbg, void* workspace, size_t workspace_bytes, void* stream,
                  bool reroute, bool static_workspace = false) {
  int st = check_config(cfg);
  if (st != SERE_OK) return st;
  PtrCheck pc;
  pc.need(hidden);
  pc.need(router_w);
  pc.need(w_gate_up);
  pc.need(w_down);
  pc.need(out);
  if (reroute) pc.need(sim);
  if (cfg->num_shared > 0) {
    pc.need(shared_gate_up);
    pc.need(shared_down);
  }
  check_route_out(pc, dbg);
  if (pc.status != SERE_OK) return pc.status;
  const Layout l = make_layout(*cfg);
  if (static_workspace) {  // the library's own array instead of a caller's buffer
    if (l.total > SERE_STATIC_SCRATCH_BYTES) return SERE_ERR_SCRATCH_TOO_SMALL;
    st = static_scratch(&workspace);
    if (st != SERE_OK) return st;
    workspace_bytes = SERE_STATIC_SCRATCH_BYTES;
  }
  st = check_workspace(l, workspace, workspace_bytes);
  if (st != SERE_OK) return st;

  hipStream_t s = static_cast<hipStream_t>(stream);
  Pointers p = bind(*cfg, l, workspace, dbg);
  p.route.sim = sim;
  p.route.reroute = reroute ? 1 : 0;
  if (!reroute) p.route.S = cfg->top_k;  // every slot is a primary slot: identity map
  st = launch_router(*cfg, p, hidden, router_w, s);
  if (st != SERE_OK) return st;
  st = launch_route(*cfg, p, true, s, dbg, static_cast<size_t>(cfg->num_tokens) * cfg->top_k * 4);
  if (st != SERE_OK) return st;

  FfnArgs f{};
  f.hidden = hidden;
  f.w_gate_up = w_gate_up;
  f.w_down = w_down;
  f.shared_gate_up = shared_gate_up;
  f.shared_down = shared_down;
  f.sorted_token = p.route.sorted_token;
  f.work_expert = p.route.work_expert;
  f.work_off = p.route.work_off;
  f.work_cnt = p.route.work_cnt;
  f.n_work = p.route.n_work;
  f.h = p.h;
  f.y = p.y;
  f.T = cfg->num_tokens;
  f.dh = cfg->hidden;
  f.dm = cfg->inter;
  f.M = cfg->num_experts;
  f.K = cfg->top_k;
  f.n_sh = cfg->num_shared;
  f.ksplit = l.ksplit;
  f.rows = l.rows;
  // Rounding h to bf16 perturbs every term of the down projection by up to
  // 2^-9 relative; the sum of d_m such terms stays far inside the output
  // tolerance for narrow experts, but not for very wide ones whose outputs
  // reach several units.  From d_m = 4096 on, h keeps its rounding residual in
  // a second bf16 plane and the down projection multiplies both.
  f.split_h = wants_split_h(*cfg);
  launch_ffn(*cfg, l, p, f, out, s);
  return hip_status();
}

// ------------------------------------------------------------ stream read ---
constexpr int kStreamReadUnroll = 8;  // 128-bit loads in flight per thread

// A workgroup reads 256 * kStreamReadUnroll consecutive 16-byte pieces, thread t the pieces
// t, t + 256, ...: every load instruction of a wavefront covers 1 KB of consecutive memory.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, size_t pieces,
                                                          uint32_t* __restrict__ sink) {
  const size_t base = static_cast<size_t>(blockIdx.x) * 256 * kStreamReadUnroll + threadIdx.x;
  u32x4 v[kStreamReadUnroll];
#pragma unroll
  for (int u = 0; u < kStreamReadUnroll; ++u) {
    const size_t at = base + static_cast<size_t>(u) * 256;
    v[u] = at < pieces ? __builtin_nontemporal_load(src + at) : u32x4{0u, 0u, 0u, 0u};
  }
  uint32_t acc = 0;
#pragma unroll
  for (int u = 0; u < kStreamReadUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  if (acc == 0x9e3779b9u && blockIdx.x == 0xfffffffeu) sink[0] = acc;  // keeps the loads alive; never true
}

// ------------------------------------------------------------- similarity ---
struct SimLayout {
  size_t sorted_token, work_expert, work_off, work_cnt, n_work, h, y, dist, acc, gram, rowsum, diag, gram_part, max_bits,
      total;
  int rows, ksplit;
  int gram_splits;      // Frobenius metric: slices of the flattened outputs in the Gram kernel
  long long gram_chunk; // ... and their length
};

static SimLayout make_sim_layout(const sere_config& c, int n) {
  SimLayout l{};
  const size_t M = c.num_experts, R = M * static_cast<size_t>(n);
  l.rows = static_cast<int>(R);
  l.ksplit = down_ksplit(c);
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o = align_up(o + bytes);
    return at;
  };
  l.sorted_token = take(R * 4);
  l.work_expert = take(M * 4);
  l.work_off = take(M * 4);
  l.work_cnt = take(M * 4);
  l.n_work = take(8);
  l.h = take(R * c.inter * sizeof(float));
  l.y = take(static_cast<size_t>(l.ksplit) * R * c.hidden * sizeof(float));
  l.dist = take(M * M * sizeof(double));
  l.acc = take(M * M * sizeof(double));
  l.max_bits = take(8);
  if (c.flags & SERE_FLAG_SIM_CKA_LINEAR) {  // Gram matrix and its row sums per expert
    l.gram = take(R * n * sizeof(double));
    l.rowsum = take(R * sizeof(double));
    l.diag = take(R * sizeof(double));
  }
  if ((c.flags & (SERE_FLAG_SIM_CKA_LINEAR | SERE_FLAG_SIM_COSINE)) == 0) {  // Frobenius: partial Gram matrices of the experts
    const long long L = static_cast<long long>(n) * c.hidden;
    // enough splits that blocks x splits fill the chip (about 512 workgroups), 16 .. 128 of them,
    // each a multiple of the Gram kernel's 64-wide load group
    const int nb = static_cast<int>((M + kGramBlock - 1) / kGramBlock);
    const int want = std::min(128, std::max(16, 512 / (nb * (nb + 1) / 2)));
    long long chunk = (L + want - 1) / want;
    chunk = std::max<long long>(256, (chunk + 63) / 64 * 64);
    l.gram_chunk = chunk;
    l.gram_splits = static_cast<int>((L + chunk - 1) / chunk);
    l.gram_part = take(static_cast<size_t>(l.gram_splits) * gram_part_stride(static_cast<int>(M)) * sizeof(double));
    l.gram = take(kGramGroups * M * M * sizeof(double));
  }
  l.total = o;
  return l;
}

constexpr int kCkaMinTokens = 4, kCkaMaxTokens = 512;  // the estimator's lower limit; M*n*n doubles of workspace

static int check_similarity_sizes(const sere_config& c, int32_t num_batches, int32_t n) {
  if (num_batches < 1 || num_batches > 4096 || n < 1 || n > 4096) return SERE_ERR_BAD_SHAPE;
  if ((c.flags & SERE_FLAG_SIM_CKA_LINEAR) && (n < kCkaMinTokens || n > kCkaMaxTokens)) return SERE_ERR_BAD_SHAPE;
  return SERE_OK;
}

static int similarity(const sere_config* cfg, const void* calib, int32_t num_batches, int32_t batch_tokens,
                      const void* w_gate_up, const void* w_down, int cka_kernel, double p0, double p1, float* sim,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  int st = check_config(cfg);
  if (st != SERE_OK) return st;
  st = check_similarity_sizes(*cfg, num_batches, batch_tokens);
  if (st != SERE_OK) return st;
  PtrCheck pc;
  pc.need(calib);
  pc.need(w_gate_up);
  pc.need(w_down);
  pc.need(sim);
  if (pc.status != SERE_OK) return pc.status;
  const SimLayout l = make_sim_layout(*cfg, batch_tokens);
  if (workspace == nullptr) return SERE_ERR_NULL_PTR;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SERE_ERR_MISALIGNED;
  if (workspace_bytes < l.total) return SERE_ERR_WORKSPACE_TOO_SMALL;

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  const int M = cfg->num_experts, n = batch_tokens;
  FfnArgs f{};
  f.w_gate_up = w_gate_up;
  f.w_down = w_down;
  f.sorted_token = reinterpret_cast<int32_t*>(ws + l.sorted_token);
  f.work_expert = reinterpret_cast<int32_t*>(ws + l.work_expert);
  f.work_off = reinterpret_cast<int32_t*>(ws + l.work_off);
  f.work_cnt = reinterpret_cast<int32_t*>(ws + l.work_cnt);
  f.n_work = reinterpret_cast<int32_t*>(ws + l.n_work);
  f.h = reinterpret_cast<float*>(ws + l.h);
  f.y = reinterpret_cast<float*>(ws + l.y);
  f.T = n;
  f.dh = cfg->hidden;
  f.dm = cfg->inter;
  f.M = M;
  f.K = 1;
  f.n_sh = 0;
  f.ksplit = l.ksplit;
  f.rows = l.rows;
  f.split_h = wants_split_h(*cfg);
  hipLaunchKernelGGL(similarity_worklist_kernel, dim3((M * n + 255) / 256), dim3(256), 0, s, M, n,
                     const_cast<int32_t*>(f.sorted_token), const_cast<int32_t*>(f.work_expert),
                     const_cast<int32_t*>(f.work_off), const_cast<int32_t*>(f.work_cnt),
                     const_cast<int32_t*>(f.n_work));
  const size_t eb = cfg->dtype == SERE_F32 ? 4 : 2;
  const int metric = (cfg->flags & SERE_FLAG_SIM_COSINE)
                         ? kMetricCosine
                         : ((cfg->flags & SERE_FLAG_SIM_CKA_LINEAR) ? kMetricCkaLinear : kMetricFrobenius);
  double* dist = reinterpret_cast<double*>(ws + l.dist);
  unsigned long long* max_bits = reinterpret_cast<unsigned long long*>(ws + l.max_bits);
  for (int b = 0; b < num_batches; ++b) {
    f.hidden = static_cast<const char*>(calib) + static_cast<size_t>(b) * n * cfg->hidden * eb;
    launch_gateup_down(cfg->dtype, cfg->inter, cfg->hidden, M, l.ksplit, f, s);
    if (metric == kMetricCosine) {
      hipLaunchKernelGGL(pair_cosine_kernel, dim3(M, M), dim3(256), 0, s, f.y, l.ksplit, l.rows, n, cfg->hidden, M,
                         dist);
    } else if (metric == kMetricCkaLinear) {
      double* gram = reinterpret_cast<double*>(ws + l.gram);
      double* rowsum = reinterpret_cast<double*>(ws + l.rowsum);
      if (cka_kernel == kCkaLinear) {
        hipLaunchKernelGGL(gram_kernel, dim3(n, M), dim3(256), 0, s, f.y, l.ksplit, l.rows, n, cfg->hidden, gram,
                           rowsum, static_cast<double*>(nullptr));
      } else {
        double* diag = reinterpret_cast<double*>(ws + l.diag);
        hipLaunchKernelGGL(gram_kernel, dim3(n, M), dim3(256), 0, s, f.y, l.ksplit, l.rows, n, cfg->hidden, gram,
                           static_cast<double*>(nullptr), diag);
        hipLaunchKernelGGL(gram_transform_kernel, dim3(n, M), dim3(256), 0, s, gram, diag, n, cka_kernel, p0,
                           static_cast<int>(p1), rowsum);
      }
      hipLaunchKernelGGL(pair_hsic_kernel, dim3(M, M), dim3(256), 0, s, gram, rowsum, n, M, dist);
    } else {
      double* part = reinterpret_cast<double*>(ws + l.gram_part);
      double* gram = reinterpret_cast<double*>(ws + l.gram);
      const int nb = (M + kGramBlock - 1) / kGramBlock;
      const dim3 per_pair((M * M + 255) / 256);
      launch_stage(SERE_STAGE_SIM_PAIRS, s, frobenius_gram_kernel, dim3(nb * (nb + 1) / 2, l.gram_splits), dim3(256), f.y,
                   l.ksplit, l.rows, n, cfg->hidden, M, l.gram_chunk, part, max_bits);
      launch_stage(SERE_STAGE_SIM_PAIRS, s, gram_reduce_kernel, dim3(per_pair.x, kGramGroups), dim3(256),
                   static_cast<const double*>(part), l.gram_splits, M, gram);
      launch_stage(SERE_STAGE_SIM_PAIRS, s, frobenius_distance_kernel, per_pair, dim3(256),
                   static_cast<const double*>(gram), static_cast<const float*>(f.y), l.ksplit, l.rows, n, cfg->hidden,
                   M, dist, max_bits);
    }
    launch_stage(SERE_STAGE_SIM_PAIRS, s, similarity_accumulate_kernel, dim3((M * M + 255) / 256), dim3(256),
                 static_cast<const double*>(dist), M, b, static_cast<int>(num_batches), metric,
                 static_cast<const unsigned long long*>(max_bits), reinterpret_cast<double*>(ws + l.acc), sim);
  }
  return hip_status();
}

}  // namespace sere

using namespace sere;

extern "C" {

size_t sere_workspace_bytes(const sere_config* cfg) {
  if (check_config(cfg) != SERE_OK) return 0;
  return make_layout(*cfg).total;
}

int sere_route(const sere_config* cfg, const void* hidden, const void* router_w, const float* sim,
               const sere_route_out* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int st = check_config(cfg);
  if (st != SERE_OK) return st;
  PtrCheck pc;
  pc.need(hidden);
  pc.need(router_w);
  pc.need(sim);
  check_route_out(pc, out);
  if (pc.status != SERE_OK) return pc.status;
  const Layout l = make_layout(*cfg);
  st = check_workspace(l, workspace, workspace_bytes);
  if (st != SERE_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  Pointers p = bind(*cfg, l, workspace, out);
  p.route.sim = sim;
  p.route.reroute = 1;
  st = launch_router(*cfg, p, hidden, router_w, s);
  if (st != SERE_OK) return st;
  return launch_route(*cfg, p, true, s, out, static_cast<size_t>(cfg->num_tokens) * cfg->top_k * 4);
}

int sere_reroute(const sere_config* cfg, const int32_t* topk_ids, const float* sim, const sere_route_out* out,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  int st = check_config(cfg);
  if (st != SERE_OK) return st;
  PtrCheck pc;
  pc.need(topk_ids);
  pc.need(sim);
  check_route_out(pc, out);
  if (pc.status != SERE_OK) return pc.status;
  const Layout l = make_layout(*cfg);
  st = check_workspace(l, workspace, workspace_bytes);
  if (st != SERE_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  sere_route_out o{};
  if (out != nullptr) o = *out;
  o.topk_ids = nullptr;
  o.topk_weights = nullptr;
  Pointers p = bind(*cfg, l, workspace, &o);
  p.route.topk_ids = topk_ids;
  p.route.sim = sim;
  p.route.reroute = 1;
  return launch_route(*cfg, p, false, s, &o, static_cast<size_t>(cfg->num_tokens) * cfg->top_k * 4);
}

int sere_moe_decode(const sere_config* cfg, const void* hidden, const void* router_w, const void* w_gate_up,
                    const void* w_down, const void* shared_gate_up, const void* shared_down, const float* sim,
                    void* out, const sere_route_out* dbg, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
  return decode(cfg, hidden, router_w, w_gate_up, w_down, shared_gate_up, shared_down, sim, out, dbg, workspace,
                workspace_bytes, hip_stream, true);
}

int sere_moe_decode_static(const sere_config* cfg, const void* hidden, const void* router_w,
                           const void* w_gate_up, const void* w_down, const void* shared_gate_up,
                           const void* shared_down, const float* sim, void* out, const sere_route_out* dbg,
                           void* hip_stream) {
  return decode(cfg, hidden, router_w, w_gate_up, w_down, shared_gate_up, shared_down, sim, out, dbg, nullptr, 0,
                hip_stream, true, true);
}

int sere_moe_decode_baseline(const sere_config* cfg, const void* hidden, const void* router_w,
                             const void* w_gate_up, const void* w_down, const void* shared_gate_up,
                             const void* shared_down, void* out, const sere_route_out* dbg, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
  return decode(cfg, hidden, router_w, w_gate_up, w_down, shared_gate_up, shared_down, nullptr, out, dbg,
                workspace, workspace_bytes, hip_stream, false);
}

size_t sere_similarity_workspace_bytes(const sere_config* cfg, int32_t batch_tokens) {
  if (check_config(cfg) != SERE_OK || check_similarity_sizes(*cfg, 1, batch_tokens) != SERE_OK) return 0;
  return make_sim_layout(*cfg, batch_tokens).total;
}

int sere_similarity(const sere_config* cfg, const void* calib, int32_t num_batches, int32_t batch_tokens,
                    const void* w_gate_up, const void* w_down, float* sim, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  return similarity(cfg, calib, num_batches, batch_tokens, w_gate_up, w_down, kCkaLinear, 0.0, 0.0, sim, workspace,
                    workspace_bytes, hip_stream);
}

// cfg with the linear-CKA flag in place of any other metric flag (workspace layout and checks)
static sere_config with_cka_flag(const sere_config* cfg) {
  sere_config c = *cfg;
  c.flags = (c.flags & ~SERE_FLAG_SIM_COSINE) | SERE_FLAG_SIM_CKA_LINEAR;
  return c;
}

size_t sere_similarity_cka_workspace_bytes(const sere_config* cfg, int32_t batch_tokens) {
  if (cfg == nullptr) return 0;
  const sere_config c = with_cka_flag(cfg);
  return sere_similarity_workspace_bytes(&c, batch_tokens);
}

int sere_similarity_cka(const sere_config* cfg, const void* calib, int32_t num_batches, int32_t batch_tokens,
                        const void* w_gate_up, const void* w_down, int32_t kernel, double param0, double param1,
                        float* sim, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (cfg == nullptr) return SERE_ERR_NULL_PTR;
  if (kernel != SERE_CKA_LINEAR && kernel != SERE_CKA_RBF && kernel != SERE_CKA_POLY) return SERE_ERR_BAD_KERNEL;
  if (kernel == SERE_CKA_RBF && !(std::isfinite(param0) && param0 > 0.0)) return SERE_ERR_BAD_KERNEL;
  if (kernel == SERE_CKA_POLY &&
      !(std::isfinite(param0) && param1 >= 1.0 && param1 <= 16.0 && param1 == std::floor(param1)))
    return SERE_ERR_BAD_KERNEL;
  const sere_config c = with_cka_flag(cfg);
  return similarity(&c, calib, num_batches, batch_tokens, w_gate_up, w_down, kernel, param0, param1, sim, workspace,
                    workspace_bytes, hip_stream);
}

int sere_stream_read(const void* src, size_t bytes, uint32_t* sink, void* hip_stream) {
  if (src == nullptr || sink == nullptr) return SERE_ERR_NULL_PTR;
  if (!aligned16(src)) return SERE_ERR_MISALIGNED;
  if (bytes == 0 || bytes % 16 != 0) return SERE_ERR_BAD_SHAPE;
  const size_t pieces = bytes / 16;
  const size_t per_block = static_cast<size_t>(256) * kStreamReadUnroll;
  const size_t blocks = (pieces + per_block - 1) / per_block;
  if (blocks > 0x7fffffffull) return SERE_ERR_BAD_SHAPE;
  hipLaunchKernelGGL(stream_read_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const u32x4*>(src), pieces, sink);
  return hip_status();
}

int sere_stage_timing(int enable) {
  g_timing.enabled = enable != 0;
  g_timing.n = 0;
  return SERE_OK;
}

int sere_stage_timing_read(double* total_ms, int32_t* launches) {
  if (total_ms == nullptr || launches == nullptr) return SERE_ERR_NULL_PTR;
  for (int i = 0; i < SERE_NUM_STAGES; ++i) {
    total_ms[i] = 0.0;
    launches[i] = 0;
  }
  Timing& t = g_timing;
  int status = SERE_OK;
  for (int i = 0; i < t.n; ++i) {
    float ms = 0.0f;
    if (hipEventSynchronize(t.stop[i]) != hipSuccess ||
        hipEventElapsedTime(&ms, t.start[i], t.stop[i]) != hipSuccess) {
      status = SERE_ERR_HIP;
      continue;
    }
    total_ms[t.stage[i]] += ms;
    launches[t.stage[i]] += 1;
  }
  t.n = 0;
  return status;
}

const char* sere_status_string(int status) {
  switch (status) {
    case SERE_OK: return "ok";
    case SERE_ERR_NULL_PTR: return "a required pointer is NULL";
    case SERE_ERR_BAD_SHAPE: return "a size is outside the supported range";
    case SERE_ERR_BAD_TOPK: return "top_k > num_experts or select_top_k outside [1, top_k]";
    case SERE_ERR_BAD_DTYPE: return "dtype is neither SERE_F32 nor SERE_BF16";
    case SERE_ERR_MISALIGNED: return "a pointer is not sufficiently aligned";
    case SERE_ERR_WORKSPACE_TOO_SMALL: return "workspace is smaller than sere_workspace_bytes()";
    case SERE_ERR_BAD_FLAGS: return "flags has an unknown bit";
    case SERE_ERR_NONFINITE_THRESHOLD: return "threshold is NaN or infinite";
    case SERE_ERR_HIP: return "a HIP call reported an error";
    case SERE_ERR_BAD_KERNEL: return "unknown CKA kernel, or a kernel parameter outside its range";
    case SERE_ERR_SCRATCH_TOO_SMALL: return "the configuration needs more than SERE_STATIC_SCRATCH_BYTES of scratch";
    default: return "unknown status";
  }
}

}  // extern "C"
