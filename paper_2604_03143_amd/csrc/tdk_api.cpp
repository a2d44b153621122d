// Host side of libtdk: argument validation, the round planner (rotation tables, block-table
// slices, work list), device memory owned by a round, event timing and the C ABI itself.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "tdk_internal.h"
#include "tdk_bench.h"
#include "tdk_plan.h"

using namespace tdk;

// Flag scratch of tdk_diff_encode_static: one byte per (agent, master page) of the round being encoded.
// Every GPU the library runs on holds its own copy of this array until the process ends.  In host code
// the name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[TDK_STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_last_error;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};     // device address of `scratch` on each device, once resolved

tdk_status fail(tdk_status st, const std::string& msg) {
  g_last_error = msg;
  return st;
}

tdk_status hip_fail(hipError_t e, const char* what) {
  return fail(TDK_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// No exception leaves the library: host allocations that fail become TDK_ERR_NOMEM.
template <typename F>
tdk_status guarded(F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    try { g_last_error = "out of memory"; } catch (...) {}   // short enough to need no allocation
    return TDK_ERR_NOMEM;
  } catch (...) {
    try { g_last_error = "internal error"; } catch (...) {}
    return TDK_ERR_INVALID_ARG;
  }
}

using HostSession = tdk::PlanSession;

struct EventPair {
  hipEvent_t start, stop;
  int kernel;
};

}  // namespace

struct tdk_round {
  tdk_model model{};
  int device = -1;
  int32_t n_cus = 256;             // compute units of that device
  std::vector<HostSession> sessions;
  int32_t n_agents = 0;
  int64_t max_phys_page = -1;      // largest page number any shared span maps to
  int64_t total_pages = 0;         // sum over agents of their session's page count
  int64_t total_master_pages = 0;  // sum over sessions of pages
  int32_t group = 0;               // agents per work item (resolved)
  int32_t flags = TDK_TUNE_DEFAULT;

  void*  blob = nullptr;           // one device allocation for everything below
  size_t blob_bytes = 0;
  size_t work_capacity = 0;        // WorkItems the work region can hold
  RoundDev rd{};

  // ping-pong restore: one "loaded" and one "free" event per staging buffer, one "done" per call
  hipEvent_t ev_loaded[2] = {nullptr, nullptr};
  hipEvent_t ev_free[2] = {nullptr, nullptr};
  bool free_recorded[2] = {false, false};
  int64_t total_master_rows = 0;
  int64_t total_tokens = 0;        // sum over agents of their session's span
  int32_t max_segments = 1;        // most segments any agent has (1 for identity layouts)
  bool seg_moved = false;          // a segmented agent's stored diff sits at other positions
  bool diff_moved = false;         // some agent's stored diff sits at other positions (segmented or not)

  bool timing = false;
  std::vector<EventPair> pending;
  std::vector<EventPair> free_events;
  double  total_ms[TDK_KERNEL_KINDS] = {0};
  int64_t launches[TDK_KERNEL_KINDS] = {0};
};

namespace {

// group: agents per work item; read_group: the same for the kernels that only read (equal when the caller named one)
tdk_status upload_work(tdk_round* r, int group, int read_group) {
  std::vector<WorkItem> work, rwork;
  plan_work(r->sessions, group, (r->flags & TDK_TUNE_TAPER) != 0, work);
  plan_work(r->sessions, read_group, false, rwork);
  if (work.size() > r->work_capacity || rwork.size() > r->work_capacity) return fail(TDK_ERR_INVALID_ARG, "work list larger than reserved");
  std::vector<WorkItem> queued;
  plan_queues(work, queued, r->rd.q_begin);
  if (!work.empty()) {
    hipError_t e = hipMemcpy(const_cast<WorkItem*>(r->rd.work), work.data(), work.size() * sizeof(WorkItem),
                             hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(const_cast<WorkItem*>(r->rd.qwork), queued.data(), queued.size() * sizeof(WorkItem),
                                       hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(const_cast<WorkItem*>(r->rd.rwork), rwork.data(), rwork.size() * sizeof(WorkItem),
                                       hipMemcpyHostToDevice);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpy(work list)");
  }
  r->rd.n_work = (int32_t)work.size();
  r->rd.n_rwork = (int32_t)rwork.size();
  r->rd.dyn_begin = r->rd.n_work;   // (a launch that shares its tail sets these in its own copy)
  r->rd.dyn_count = 0;
  r->group = group;
  return TDK_OK;
}

tdk_status check_step(const tdk_round* r, int32_t layer, const tdk_layer_io* io) {
  if (!r) return fail(TDK_ERR_INVALID_ARG, "round is NULL");
  if (!io) return fail(TDK_ERR_INVALID_ARG, "layer io is NULL");
  if (layer < 0 || layer >= r->model.num_layers) return fail(TDK_ERR_INVALID_ARG, "layer out of range");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != r->device)
    return fail(TDK_ERR_INVALID_ARG, "the round was created on another device than the current one");
  if (io->pool_pages < 0) return fail(TDK_ERR_INVALID_ARG, "pool_pages is negative");
  if (r->rd.n_work > 0) {
    if (!io->master_k || !io->master_v || !io->pool_k || !io->pool_v)
      return fail(TDK_ERR_INVALID_ARG, "layer io holds a NULL buffer");
    if (io->pool_pages <= r->max_phys_page)
      return fail(TDK_ERR_INVALID_ARG, "pool_pages is smaller than a page number in the block tables");
    const uintptr_t bits = (uintptr_t)io->master_k | (uintptr_t)io->master_v | (uintptr_t)io->pool_k | (uintptr_t)io->pool_v;
    if (bits & 15) return fail(TDK_ERR_INVALID_ARG, "layer io buffers must be 16-byte aligned");
  }
  return TDK_OK;
}

tdk_status check_diff(const tdk_round* r, const tdk_diff* d, bool for_encode) {
  if (!d) return fail(TDK_ERR_INVALID_ARG, "diff is NULL");
  if (!d->count || !d->offset) return fail(TDK_ERR_INVALID_ARG, "diff.count / diff.offset is NULL");
  if (for_encode && !d->overflow) return fail(TDK_ERR_INVALID_ARG, "diff.overflow is NULL");
  if (d->capacity_pages < 0) return fail(TDK_ERR_INVALID_ARG, "diff.capacity_pages is negative");
  if (d->capacity_pages > 0 && (!d->idx || !d->payload))
    return fail(TDK_ERR_INVALID_ARG, "diff.idx / diff.payload is NULL with capacity_pages > 0");
  if ((uintptr_t)d->payload & 15) return fail(TDK_ERR_INVALID_ARG, "diff.payload must be 16-byte aligned");
  if ((uintptr_t)d->offset & 7) return fail(TDK_ERR_INVALID_ARG, "diff.offset must be 8-byte aligned");
  (void)r;
  return TDK_OK;
}

LayerDev layer_dev(const tdk_layer_io* io) {
  LayerDev l;
  l.master_k = static_cast<const u32x4*>(io->master_k);
  l.master_v = static_cast<const u32x4*>(io->master_v);
  l.pool_k = static_cast<u32x4*>(io->pool_k);
  l.pool_v = static_cast<u32x4*>(io->pool_v);
  return l;
}

DiffDev diff_dev(const tdk_diff* d) {
  DiffDev x;
  x.count = d->count;
  x.offset = d->offset;
  x.idx = d->idx;
  x.payload = static_cast<u32x4*>(d->payload);
  x.capacity = d->capacity_pages;
  x.overflow = d->overflow;
  return x;
}

// brackets one kernel launch with events when timing is on
struct Timed {
  tdk_round* r;
  hipStream_t st;
  EventPair ev{};
  bool on;
  hipError_t err = hipSuccess;
  Timed(tdk_round* r_, int kernel, hipStream_t st_) : r(r_), st(st_), on(r_->timing) {
    if (!on) return;
    if (!r->free_events.empty()) {
      ev = r->free_events.back();
      r->free_events.pop_back();
    } else {
      err = hipEventCreate(&ev.start);
      if (err == hipSuccess) {
        err = hipEventCreate(&ev.stop);
        if (err != hipSuccess) (void)hipEventDestroy(ev.start);
      }
      if (err != hipSuccess) { on = false; return; }
    }
    ev.kernel = kernel;
    err = hipEventRecord(ev.start, st);
  }
  void done() {
    if (!on) return;
    hipError_t e = hipEventRecord(ev.stop, st);
    if (err == hipSuccess) err = e;
    r->pending.push_back(ev);
  }
};

#define TDK_LAUNCH(R, KIND, ST, CALL)                                     \
  do {                                                                    \
    Timed timed_((R), (KIND), (ST));                                      \
    hipError_t e_ = (CALL);                                               \
    timed_.done();                                                        \
    if (e_ != hipSuccess) return hip_fail(e_, "kernel launch " #KIND);     \
    if (timed_.err != hipSuccess) return hip_fail(timed_.err, "event record"); \
  } while (0)

}  // namespace

extern "C" {

const char* tdk_status_str(tdk_status s) {
  switch (s) {
    case TDK_OK: return "ok";
    case TDK_ERR_INVALID_ARG: return "invalid argument";
    case TDK_ERR_UNSUPPORTED: return "unsupported";
    case TDK_ERR_CAPACITY: return "capacity exceeded";
    case TDK_ERR_HIP: return "HIP runtime error";
    case TDK_ERR_NOMEM: return "out of memory";
  }
  return "unknown status";
}

const char* tdk_last_error(void) { return g_last_error.c_str(); }

const char* tdk_version(void) { return "tdk 0.1 (gfx950)"; }

const char* tdk_kernel_name(int32_t kernel) {
  switch (kernel) {
    case TDK_KERNEL_REROTATE: return "tdk_rerotate_kernel";
    case TDK_KERNEL_FLAG: return "tdk_flag_kernel";
    case TDK_KERNEL_COMPACT: return "tdk_compact_kernel";
    case TDK_KERNEL_GATHER: return "tdk_gather_kernel";
    case TDK_KERNEL_DECODE: return "tdk_decode_kernel";
    case TDK_KERNEL_SCATTER: return "tdk_scatter_kernel";
    case TDK_KERNEL_KEYDIFF: return "tdk_keydiff_kernel";
    case TDK_KERNEL_SELECT: return "tdk_select_kernel";
    case TDK_KERNEL_MASTER: return "tdk_master_kernel";
    case TDK_KERNEL_ATTEND_QROT: return "tdk_attend_qrot_kernel";
    case TDK_KERNEL_ATTEND_MASTER: return "tdk_attend_master_kernel";
    case TDK_KERNEL_ATTEND_DIFF: return "tdk_attend_diff_kernel";
    case TDK_KERNEL_ATTEND_MERGE: return "tdk_attend_merge_kernel";
  }
  return "";
}

}  // extern "C"

namespace {

struct RoundDeleter {
  void operator()(tdk_round* r) const { tdk_round_destroy(r); }
};

tdk_status round_create(const tdk_model* model, const tdk_session* sessions, int32_t n_sessions,
                        const tdk_agent* agents, int32_t n_agents, tdk_round** out) {
  if (!out) return fail(TDK_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  tdk_status st = TDK_OK;
  std::unique_ptr<tdk_round, RoundDeleter> holder(new tdk_round());   // released on every early return
  tdk_round* r = holder.get();

  // ---- host-side validation and planning (tdk_plan.cpp; no HIP call before this block is through) ----
  RoundPlan p;
  {
    std::string err;
    const tdk_status ps = plan_round(model, sessions, n_sessions, agents, n_agents, p, err);
    if (ps != TDK_OK) return fail(ps, err);
  }
  r->sessions = p.sessions;
  r->max_phys_page = p.max_phys_page;
  r->total_pages = p.total_pages;
  r->rd.agent_pages = p.total_pages;
  r->total_master_pages = p.total_master_pages;
  r->total_master_rows = p.total_master_rows;
  r->total_tokens = p.total_tokens;
  r->max_segments = p.max_segments;
  r->seg_moved = p.seg_moved;
  r->diff_moved = p.diff_moved;
  r->work_capacity = p.work_capacity;
  r->model = *model;
  r->n_agents = n_agents;
  const int T = model->page_tokens;
  const bool any_segments = p.any_segments;
  const size_t work_cap = p.work_capacity;
  const int64_t flag_off = p.total_pages;
  const auto& sess_dev = p.sess;
  const auto& agent_dev = p.agents;
  const auto& order = p.order;
  const auto& bt = p.bt;
  const auto& tab = p.tab;
  const auto& tab_diff = p.tab_diff;
  const auto& rowmap = p.rowmap;
  const auto& pagetab = p.pagetab;
  const auto& segtab = p.segtab;
  const auto& segtab_diff = p.segtab_diff;
  const auto& seg_off = p.seg_off;
  const auto& seg_src = p.seg_src;

  // ---- device memory: one allocation ----
  size_t off = 0;
  auto place = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  const size_t o_work = place(work_cap * sizeof(WorkItem));
  const size_t o_qwork = place(work_cap * sizeof(WorkItem));
  const size_t o_rwork = place(work_cap * sizeof(WorkItem));
  const size_t o_sess = place(sess_dev.size() * sizeof(SessionDev));
  const size_t o_agents = place(agent_dev.size() * sizeof(AgentDev));
  const size_t o_order = place(order.size() * sizeof(int32_t));
  const size_t o_bt = place(bt.size() * sizeof(int32_t));
  const size_t o_tab = place(tab.size() * sizeof(float));
  const size_t o_tab_diff = place(tab_diff.size() * sizeof(float));
  const size_t o_rowmap = place(any_segments ? rowmap.size() * sizeof(int32_t) : 0);
  const size_t o_pagetab = place(any_segments ? pagetab.size() * sizeof(PageTab) : 0);
  const size_t o_segtab = place(any_segments ? segtab.size() * sizeof(float) : 0);
  const size_t o_segtab_diff = place(any_segments ? segtab_diff.size() * sizeof(float) : 0);
  const size_t o_seg_off = place(any_segments ? seg_off.size() * sizeof(int32_t) : 0);
  const size_t o_seg_src = place(any_segments ? seg_src.size() * sizeof(int32_t) : 0);
  const size_t o_flags = place((size_t)flag_off);
  const size_t o_qstate = place(16 * sizeof(int32_t));
  r->blob_bytes = std::max<size_t>(off, 256);

  hipError_t e = hipGetDevice(&r->device);
  if (e != hipSuccess) { return hip_fail(e, "hipGetDevice"); }
  {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, r->device) == hipSuccess && cus > 0) r->n_cus = cus;
  }
  e = hipMalloc(&r->blob, r->blob_bytes);
  if (e != hipSuccess) { return e == hipErrorOutOfMemory ? fail(TDK_ERR_NOMEM, "device allocation failed") : hip_fail(e, "hipMalloc"); }
  char* base = static_cast<char*>(r->blob);
  auto up = [&](size_t o, const void* src, size_t bytes) -> hipError_t {
    return bytes ? hipMemcpy(base + o, src, bytes, hipMemcpyHostToDevice) : hipSuccess;
  };
  e = up(o_sess, sess_dev.data(), sess_dev.size() * sizeof(SessionDev));
  if (e == hipSuccess) e = up(o_agents, agent_dev.data(), agent_dev.size() * sizeof(AgentDev));
  if (e == hipSuccess) e = up(o_order, order.data(), order.size() * sizeof(int32_t));
  if (e == hipSuccess) e = up(o_bt, bt.data(), bt.size() * sizeof(int32_t));
  if (e == hipSuccess) e = up(o_tab, tab.data(), tab.size() * sizeof(float));
  if (e == hipSuccess) e = up(o_tab_diff, tab_diff.data(), tab_diff.size() * sizeof(float));
  if (e == hipSuccess && any_segments) e = up(o_rowmap, rowmap.data(), rowmap.size() * sizeof(int32_t));
  if (e == hipSuccess && any_segments) e = up(o_pagetab, pagetab.data(), pagetab.size() * sizeof(PageTab));
  if (e == hipSuccess && any_segments) e = up(o_segtab, segtab.data(), segtab.size() * sizeof(float));
  if (e == hipSuccess && any_segments) e = up(o_segtab_diff, segtab_diff.data(), segtab_diff.size() * sizeof(float));
  if (e == hipSuccess && any_segments) e = up(o_seg_off, seg_off.data(), seg_off.size() * sizeof(int32_t));
  if (e == hipSuccess && any_segments) e = up(o_seg_src, seg_src.data(), seg_src.size() * sizeof(int32_t));
  if (e == hipSuccess && flag_off) e = hipMemset(base + o_flags, 0, (size_t)flag_off);
  if (e == hipSuccess) e = hipMemset(base + o_qstate, 0, 16 * sizeof(int32_t));
  if (e != hipSuccess) return hip_fail(e, "upload of round descriptors");

  r->rd.work = reinterpret_cast<const WorkItem*>(base + o_work);
  r->rd.qwork = reinterpret_cast<const WorkItem*>(base + o_qwork);
  r->rd.rwork = reinterpret_cast<const WorkItem*>(base + o_rwork);
  r->rd.sess = reinterpret_cast<const SessionDev*>(base + o_sess);
  r->rd.agents = reinterpret_cast<const AgentDev*>(base + o_agents);
  r->rd.order = reinterpret_cast<const int32_t*>(base + o_order);
  r->rd.bt = reinterpret_cast<const int32_t*>(base + o_bt);
  r->rd.tab = reinterpret_cast<const float*>(base + o_tab);
  r->rd.tab_diff = reinterpret_cast<const float*>(base + o_tab_diff);
  r->rd.flags = reinterpret_cast<uint8_t*>(base + o_flags);
  r->rd.q_state = reinterpret_cast<int32_t*>(base + o_qstate);
  r->rd.n_cus = r->n_cus;
  r->rd.seg = any_segments ? 1 : 0;
  r->rd.rowmap = any_segments ? reinterpret_cast<const int32_t*>(base + o_rowmap) : nullptr;
  r->rd.pagetab = any_segments ? reinterpret_cast<const PageTab*>(base + o_pagetab) : nullptr;
  r->rd.segtab = any_segments ? reinterpret_cast<const float*>(base + o_segtab) : nullptr;
  r->rd.segtab_diff = any_segments ? reinterpret_cast<const float*>(base + o_segtab_diff) : nullptr;
  r->rd.seg_off = any_segments ? reinterpret_cast<const int32_t*>(base + o_seg_off) : nullptr;
  r->rd.seg_src = any_segments ? reinterpret_cast<const int32_t*>(base + o_seg_src) : nullptr;
  r->rd.n_agents = n_agents;
  r->rd.master_rows = r->total_master_rows;
  r->rd.n_sessions = n_sessions;
  r->rd.heads = model->num_kv_heads;
  r->rd.page_tokens = T;
  r->rd.interleaved = model->rope_style == TDK_ROPE_INTERLEAVED;
  r->rd.nontemporal = r->flags & TDK_TUNE_ALL;

  st = upload_work(r, plan_auto_group(r->sessions), plan_auto_group(r->sessions, true));
  if (st != TDK_OK) return st;
  for (int b = 0; b < 2 && e == hipSuccess; ++b) {
    e = hipEventCreateWithFlags(&r->ev_loaded[b], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&r->ev_free[b], hipEventDisableTiming);
  }
  if (e != hipSuccess) return hip_fail(e, "hipEventCreate");
  *out = holder.release();
  return TDK_OK;
}

// The two halves of skip-or-correct: the page kernel writes every page that no diff lists from the re-rotated
// master, the slot kernel copies the listed pages from the payload (in a launch of its own, or, on small rounds,
// as extra workgroups of the page kernel's launch).
tdk_status launch_restore(tdk_round* r, const LayerDev& l, const DiffDev& d, int planes, int64_t capacity_pages, hipStream_t s) {
  // the number of listed pages is known on the device only: a fixed number of workgroups strides over them
  const int slots = (int)std::min<int64_t>(std::min<int64_t>(capacity_pages, r->total_pages), 1 << 20);
  bool scattered = false;
  TDK_LAUNCH(r, TDK_KERNEL_DECODE, s, launch_decode(r->rd, l, d, planes, slots, &scattered, s));
  if (!scattered) TDK_LAUNCH(r, TDK_KERNEL_SCATTER, s, launch_scatter(r->rd, l, d, planes, slots, s));
  return TDK_OK;
}

}  // namespace

extern "C" {

tdk_status tdk_round_create(const tdk_model* model, const tdk_session* sessions, int32_t n_sessions,
                            const tdk_agent* agents, int32_t n_agents, tdk_round** out) {
  return guarded([&] { return round_create(model, sessions, n_sessions, agents, n_agents, out); });
}

void tdk_round_destroy(tdk_round* r) {
  if (!r) return;
  for (auto& ev : r->pending) { (void)hipEventDestroy(ev.start); (void)hipEventDestroy(ev.stop); }
  for (auto& ev : r->free_events) { (void)hipEventDestroy(ev.start); (void)hipEventDestroy(ev.stop); }
  for (int b = 0; b < 2; ++b) {
    if (r->ev_loaded[b]) (void)hipEventDestroy(r->ev_loaded[b]);
    if (r->ev_free[b]) (void)hipEventDestroy(r->ev_free[b]);
  }
  if (r->blob) (void)hipFree(r->blob);
  delete r;
}

size_t tdk_scratch_bytes(const tdk_round* r) { return r ? r->blob_bytes : 0; }

tdk_status tdk_round_tune(tdk_round* r, int32_t agents_per_group, int32_t flags) {
  return guarded([&]() -> tdk_status {
    if (!r) return fail(TDK_ERR_INVALID_ARG, "round is NULL");
    if (agents_per_group < 0 || agents_per_group > kMaxGroup)
      return fail(TDK_ERR_INVALID_ARG, "agents_per_group must be 0 (automatic) or 1..32");
    if (flags & ~TDK_TUNE_ALL) return fail(TDK_ERR_INVALID_ARG, "unknown tuning flag");
    // the work list is read by kernels already enqueued: wait for them before replacing it
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return hip_fail(e, "hipDeviceSynchronize");
    r->flags = flags;
    r->rd.nontemporal = flags & TDK_TUNE_ALL;
    return upload_work(r, agents_per_group ? agents_per_group : plan_auto_group(r->sessions),
                       agents_per_group ? agents_per_group : plan_auto_group(r->sessions, true));
  });
}

int32_t tdk_round_agents_per_group(const tdk_round* r) { return r ? r->group : 0; }

tdk_status tdk_rerotate_round(tdk_round* r, int32_t layer, const tdk_layer_io* io, void* hip_stream) {
  return guarded([&]() -> tdk_status {
    tdk_status st = check_step(r, layer, io);
    if (st != TDK_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    TDK_LAUNCH(r, TDK_KERNEL_REROTATE, s, launch_rerotate(r->rd, layer_dev(io), s));
    return TDK_OK;
  });
}

static tdk_status check_encode(const tdk_round* r, int32_t layer, const tdk_layer_io* io, float eps, const tdk_diff* out) {
  tdk_status st = check_step(r, layer, io);
  if (st != TDK_OK) return st;
  st = check_diff(r, out, true);
  if (st != TDK_OK) return st;
  if (!(eps >= 0.0f) || !std::isfinite(eps)) return fail(TDK_ERR_INVALID_ARG, "eps must be finite and >= 0");
  return TDK_OK;
}

static tdk_status encode_planes(tdk_round* r, int32_t layer, const tdk_layer_io* io, float eps, int planes,
                                const tdk_diff* out, void* hip_stream) {
  return guarded([&]() -> tdk_status {
    tdk_status st = check_encode(r, layer, io, eps, out);
    if (st != TDK_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const LayerDev l = layer_dev(io);
    const DiffDev d = diff_dev(out);
    TDK_LAUNCH(r, TDK_KERNEL_FLAG, s, launch_flag(r->rd, l, eps, planes, s));
    TDK_LAUNCH(r, TDK_KERNEL_COMPACT, s, launch_compact(r->rd, d, s));
    // the number of listed pages is known on the device only: a fixed grid strides over them
    const int grid = (int)std::min<int64_t>(std::min<int64_t>(out->capacity_pages, r->total_pages), 1 << 20);
    TDK_LAUNCH(r, TDK_KERNEL_GATHER, s, launch_gather(r->rd, l, d, planes, grid, s));
    return TDK_OK;
  });
}

// Device address of the static flag scratch on the current device, resolved once per device.
static tdk_status static_scratch(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return fail(TDK_ERR_UNSUPPORTED, "device ordinal beyond the static scratch table");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return TDK_OK;
}

tdk_status tdk_diff_encode_static(tdk_round* r, int32_t layer, const tdk_layer_io* io, float eps,
                                  const tdk_diff* out, void* hip_stream) {
  return guarded([&]() -> tdk_status {
    tdk_status st = check_encode(r, layer, io, eps, out);     // includes: the round's device is the current one
    if (st != TDK_OK) return st;
    if (r->total_pages > (int64_t)TDK_STATIC_SCRATCH_BYTES)
      return fail(TDK_ERR_CAPACITY, "round has more (agent, page) pairs than TDK_STATIC_SCRATCH_BYTES");
    void* flags = nullptr;
    st = static_scratch(r->device, &flags);
    if (st != TDK_OK) return st;
    // the same kernels as tdk_diff_encode, their flag bytes in the static array instead of the round's own
    // allocation; the compare kernel writes the flag of every (agent, page) of the round before compaction
    // reads any, so nothing of an earlier call is ever read and nothing needs clearing
    RoundDev rd = r->rd;
    rd.flags = static_cast<uint8_t*>(flags);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const LayerDev l = layer_dev(io);
    const DiffDev d = diff_dev(out);
    const int planes = TDK_PLANE_K | TDK_PLANE_V;
    hipError_t e = launch_flag(rd, l, eps, planes, s);
    if (e == hipSuccess) e = launch_compact(rd, d, s);
    const int grid = (int)std::min<int64_t>(std::min<int64_t>(out->capacity_pages, r->total_pages), 1 << 20);
    if (e == hipSuccess) e = launch_gather(rd, l, d, planes, grid, s);
    if (e != hipSuccess) return hip_fail(e, "kernel launch (tdk_diff_encode_static)");
    return TDK_OK;
  });
}

static tdk_status decode_planes(tdk_round* r, int32_t layer, const tdk_layer_io* io, int planes,
                                const tdk_diff* in, void* hip_stream) {
  return guarded([&]() -> tdk_status {
    tdk_status st = check_step(r, layer, io);
    if (st != TDK_OK) return st;
    st = check_diff(r, in, false);
    if (st != TDK_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const LayerDev l = layer_dev(io);
    const DiffDev d = diff_dev(in);
    st = launch_restore(r, l, d, planes, in->capacity_pages, s);
    return st;
  });
}

tdk_status tdk_diff_encode(tdk_round* r, int32_t layer, const tdk_layer_io* io, float eps,
                           const tdk_diff* out, void* hip_stream) {
  return encode_planes(r, layer, io, eps, TDK_PLANE_K | TDK_PLANE_V, out, hip_stream);
}

tdk_status tdk_diff_decode(tdk_round* r, int32_t layer, const tdk_layer_io* io, const tdk_diff* in,
                           void* hip_stream) {
  return decode_planes(r, layer, io, TDK_PLANE_K | TDK_PLANE_V, in, hip_stream);
}

tdk_status tdk_diff_encode_plane(tdk_round* r, int32_t layer, const tdk_layer_io* io, float eps, int32_t plane,
                                 const tdk_diff* out, void* hip_stream) {
  if (plane != TDK_PLANE_K && plane != TDK_PLANE_V) return fail(TDK_ERR_INVALID_ARG, "plane must be TDK_PLANE_K or TDK_PLANE_V");
  return encode_planes(r, layer, io, eps, plane, out, hip_stream);
}

tdk_status tdk_diff_decode_plane(tdk_round* r, int32_t layer, const tdk_layer_io* io, int32_t plane,
                                 const tdk_diff* in, void* hip_stream) {
  if (plane != TDK_PLANE_K && plane != TDK_PLANE_V) return fail(TDK_ERR_INVALID_ARG, "plane must be TDK_PLANE_K or TDK_PLANE_V");
  return decode_planes(r, layer, io, plane, in, hip_stream);
}

tdk_status tdk_check_layer(tdk_round* r, int32_t layer, const tdk_layer_io* io, float ratio, float min_score,
                           const tdk_reuse_plan* out, void* hip_stream) {
  return guarded([&]() -> tdk_status {
    tdk_status st = check_step(r, layer, io);
    if (st != TDK_OK) return st;
    if (!out) return fail(TDK_ERR_INVALID_ARG, "reuse plan is NULL");
    if (!(ratio > 0.0f) || !(ratio <= 1.0f)) return fail(TDK_ERR_INVALID_ARG, "ratio must be in (0, 1]");
    if (!(min_score >= 0.0f) || !std::isfinite(min_score)) return fail(TDK_ERR_INVALID_ARG, "min_score must be finite and >= 0");
    if (out->k_stride < 0) return fail(TDK_ERR_INVALID_ARG, "k_stride is negative");
    if (r->n_agents && (!out->n_important || !out->total)) return fail(TDK_ERR_INVALID_ARG, "plan.n_important / plan.total is NULL");
    if (r->total_tokens && !out->score) return fail(TDK_ERR_INVALID_ARG, "plan.score is NULL");
    if (r->n_agents && out->k_stride > 0 && !out->important) return fail(TDK_ERR_INVALID_ARG, "plan.important is NULL");
    if (!r->sessions.empty() && !out->master) return fail(TDK_ERR_INVALID_ARG, "plan.master is NULL");
    for (const auto& hs : r->sessions) {
      const int64_t k = (int64_t)std::ceil((double)ratio * (double)hs.span);
      if (!hs.agents.empty() && k > out->k_stride) return fail(TDK_ERR_INVALID_ARG, "k_stride is smaller than ceil(ratio * span)");
    }
    PlanDev pl;
    pl.score = out->score; pl.important = out->important; pl.n_important = out->n_important;
    pl.total = out->total; pl.master = out->master; pl.k_stride = out->k_stride;
    pl.ratio = ratio; pl.min_score = min_score;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    TDK_LAUNCH(r, TDK_KERNEL_KEYDIFF, s, launch_keydiff(r->rd, layer_dev(io), pl, s));
    TDK_LAUNCH(r, TDK_KERNEL_SELECT, s, launch_select(r->rd, pl, s));
    TDK_LAUNCH(r, TDK_KERNEL_MASTER, s, launch_master(r->rd, pl, s));
    return TDK_OK;
  });
}

namespace {

// Shape of the attention pass for a round: tokens per workgroup of the master pass, parts per query
// row, and the layout of the caller's workspace.
struct AttendPlan {
  int32_t chunk_tokens = 0, n_chunks = 0, n_parts = 0, max_rows = 0, n_pieces = 1, piece_tokens = 0;
  int64_t rows = 0;
  size_t o_qrot = 0, o_qdiff = 0, o_part_o = 0, o_part_m = 0, o_part_l = 0, bytes = 0;
};

bool attend_plan(const tdk_round* r, int32_t n_q, int32_t n_q_heads, AttendPlan& p) {
  if (!r || n_q < 1 || n_q_heads < 1 || n_q_heads % r->model.num_kv_heads) return false;
  const int32_t G = n_q_heads / r->model.num_kv_heads;
  int64_t max_span = 0, max_agents = 0;
  for (const auto& hs : r->sessions) {
    if (hs.agents.empty()) continue;
    max_span = std::max<int64_t>(max_span, hs.span);
    max_agents = std::max<int64_t>(max_agents, (int64_t)hs.agents.size());
  }
  const int64_t max_rows = max_agents * n_q * G;
  if (max_rows >= (int64_t)1 << 30) return false;
  p.max_rows = (int32_t)max_rows;
  p.rows = (int64_t)r->n_agents * n_q * n_q_heads;
  // Tokens per workgroup of the master pass.  A workgroup walks its chunk in steps of 64 tokens; two
  // workgroups fit a compute unit at a time, so the pass takes about ceil(workgroups / slots) rounds of
  // (steps per chunk + a fixed start-up cost of about two steps).  Of the chunk sizes that the 128-bit page
  // mask per query row can cover, the one with the lowest such cost wins; ties go to the larger chunk
  // (fewer partial results to merge).
  const int64_t row_blocks = std::max<int64_t>(1, (max_rows + 127) / 128);
  const int64_t slots = 2 * (int64_t)r->n_cus;
  const int32_t max_chunk = std::min<int32_t>(128 * r->model.page_tokens, 4096);
  // Chunks shorter than 512 tokens are not tried (unless the span is): a workgroup's start-up (page masks,
  // query rotation, first rows) costs about as much as three steps, every chunk adds a partial result per row
  // for the merge, and rounds small enough to consider such chunks are bounded by the listed-pages pass anyway
  // (one session of 25 agents: 44 us with chunks of 128 tokens, 32 us with 512).
  const int32_t min_chunk = (int32_t)std::min<int64_t>(512, (max_span + 63) / 64 * 64);
  int32_t chunk = std::max(min_chunk, 64);
  int64_t best = -1;
  for (int32_t c = max_chunk; c >= std::max(min_chunk, 64); c -= 64) {
    int64_t wgs = 0;
    for (const auto& hs : r->sessions)
      if (!hs.agents.empty()) wgs += ((int64_t)hs.span + c - 1) / c;
    wgs *= r->model.num_kv_heads * row_blocks;
    if (wgs == 0) break;
    const int64_t cost = ((wgs + slots - 1) / slots) * (std::min<int64_t>(c, max_span + 63) / 64 + 2);
    if (best < 0 || cost < best) { best = cost; chunk = c; }
  }
  p.chunk_tokens = chunk;
  p.n_chunks = (int32_t)((max_span + chunk - 1) / chunk);
  // the listed-pages pass: one wavefront takes a piece of an agent's list and every piece has its own partial result
  {
    int64_t max_pages = 0;
    for (const auto& hs : r->sessions)
      if (!hs.agents.empty()) max_pages = std::max<int64_t>(max_pages, hs.pages);
    p.piece_tokens = attend_piece_tokens((int64_t)r->n_agents * r->model.num_kv_heads, r->n_cus);
    p.n_pieces = (int32_t)std::max<int64_t>(1, (max_pages * r->model.page_tokens + p.piece_tokens - 1) / p.piece_tokens);
  }
  p.n_parts = p.n_chunks + p.n_pieces;
  size_t off = 0;
  auto place = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  p.o_qrot = place((size_t)p.rows * r->max_segments * kHeadDim * 2);
  p.o_qdiff = place((size_t)p.rows * (r->rd.seg && r->seg_moved ? r->max_segments : 1) * kHeadDim * 2);
  p.o_part_o = place((size_t)p.rows * p.n_parts * kHeadDim * sizeof(float));
  p.o_part_m = place((size_t)p.rows * p.n_parts * sizeof(float));
  p.o_part_l = place((size_t)p.rows * p.n_parts * sizeof(float));
  p.bytes = std::max<size_t>(off, 256);
  return true;
}

}  // namespace

size_t tdk_attend_workspace_bytes(const tdk_round* r, int32_t n_q, int32_t n_q_heads) {
  AttendPlan p;
  return attend_plan(r, n_q, n_q_heads, p) ? p.bytes : 0;
}

tdk_status tdk_attend_shared(tdk_round* r, int32_t layer, const tdk_layer_io* io, const tdk_diff* in,
                             const tdk_attend_io* a, void* hip_stream) {
  return guarded([&]() -> tdk_status {
    if (!r) return fail(TDK_ERR_INVALID_ARG, "round is NULL");
    if (!io || !a) return fail(TDK_ERR_INVALID_ARG, "layer io / attend io is NULL");
    if (layer < 0 || layer >= r->model.num_layers) return fail(TDK_ERR_INVALID_ARG, "layer out of range");
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != r->device)
      return fail(TDK_ERR_INVALID_ARG, "the round was created on another device than the current one");
    tdk_status st = check_diff(r, in, false);
    if (st != TDK_OK) return st;
    AttendPlan p;
    if (!attend_plan(r, a->n_q, a->n_q_heads, p))
      return fail(TDK_ERR_INVALID_ARG, "n_q must be >= 1 and n_q_heads a positive multiple of the KV heads");
    if (!std::isfinite(a->scale)) return fail(TDK_ERR_INVALID_ARG, "scale must be finite");
    if (p.rows == 0) return TDK_OK;
    if (!a->q || !a->out || !a->lse || !a->workspace) return fail(TDK_ERR_INVALID_ARG, "attend io holds a NULL buffer");
    if (((uintptr_t)a->q & 15) || ((uintptr_t)a->out & 15) || ((uintptr_t)a->workspace & 255))
      return fail(TDK_ERR_INVALID_ARG, "q / out must be 16-byte aligned, the workspace 256-byte aligned");
    if (a->workspace_bytes < p.bytes) return fail(TDK_ERR_INVALID_ARG, "workspace smaller than tdk_attend_workspace_bytes()");
    if (r->total_master_rows > 0) {
      if (!io->master_k || !io->master_v) return fail(TDK_ERR_INVALID_ARG, "layer io holds a NULL master");
      if (((uintptr_t)io->master_k | (uintptr_t)io->master_v) & 15) return fail(TDK_ERR_INVALID_ARG, "masters must be 16-byte aligned");
    }
    AttendDev at;
    char* ws = static_cast<char*>(a->workspace);
    at.q = a->q;
    at.qrot = ws + p.o_qrot;
    at.qdiff = ws + p.o_qdiff;
    at.part_o = reinterpret_cast<float*>(ws + p.o_part_o);
    at.part_m = reinterpret_cast<float*>(ws + p.o_part_m);
    at.part_l = reinterpret_cast<float*>(ws + p.o_part_l);
    at.out = a->out;
    at.lse = a->lse;
    at.n_q = a->n_q;
    at.n_q_heads = a->n_q_heads;
    at.group = a->n_q_heads / r->model.num_kv_heads;
    at.chunk_tokens = p.chunk_tokens;
    at.n_chunks = p.n_chunks;
    at.n_parts = p.n_parts;
    at.n_pieces = p.n_pieces;
    at.piece_tokens = p.piece_tokens;
    // most lists are far shorter than a whole session's pages: a few wavefronts per list walk its pieces in turn,
    // instead of one launched wavefront per possible piece (nearly all of which would find nothing)
    at.piece_grid = std::min<int32_t>(p.n_pieces, 4);
    // the kernels take a positive scale: the sign travels with the query copies, and a zero scale (uniform
    // weights) becomes one so small that every scaled score rounds to zero
    at.scale = std::fmax(std::fabs(a->scale), 1e-30f);
    at.q_flip = std::signbit(a->scale) ? 1 : 0;
    at.max_seg = r->max_segments;
    at.diff_seg = r->rd.seg && r->seg_moved ? r->max_segments : 1;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const LayerDev l = layer_dev(io);
    const DiffDev d = diff_dev(in);
    // blocks of the two passes share one launch when the round allows it (timed as the master pass)
    const int64_t fused_blocks = (int64_t)r->model.num_kv_heads * r->rd.n_sessions * p.n_chunks * ((p.max_rows + 127) / 128) +
                                 (int64_t)r->n_agents * ((r->model.num_kv_heads + 3) / 4) * std::min<int32_t>(p.n_pieces, 4);
    if (!r->rd.seg && !r->diff_moved && (int64_t)a->n_q * at.group <= 32 && r->total_master_rows > 0 && fused_blocks < (1 << 30)) {
      // (this launch rotates the query rows itself: no qrot kernel)
      TDK_LAUNCH(r, TDK_KERNEL_ATTEND_MASTER, s, launch_attend_fused(r->rd, l, d, at, p.max_rows, s));
    } else {
      TDK_LAUNCH(r, TDK_KERNEL_ATTEND_QROT, s, launch_attend_qrot(r->rd, at, s));
      TDK_LAUNCH(r, TDK_KERNEL_ATTEND_MASTER, s, launch_attend_master(r->rd, l, d, at, p.max_rows, s));
      TDK_LAUNCH(r, TDK_KERNEL_ATTEND_DIFF, s, launch_attend_diff(r->rd, d, at, s));
    }
    TDK_LAUNCH(r, TDK_KERNEL_ATTEND_MERGE, s, launch_attend_merge(r->rd, d, at, s));
    return TDK_OK;
  });
}

tdk_status tdk_restore_layers(tdk_round* r, int32_t first_layer, int32_t n_layers,
                              const void* const* host_master_k, const void* const* host_master_v,
                              const tdk_layer_io* io, const tdk_diff* diffs, const tdk_pingpong* pp,
                              void* compute_stream, void* copy_stream) {
  return guarded([&]() -> tdk_status {
    if (!r) return fail(TDK_ERR_INVALID_ARG, "round is NULL");
    if (n_layers < 0 || first_layer < 0 || (int64_t)first_layer + n_layers > r->model.num_layers)
      return fail(TDK_ERR_INVALID_ARG, "layer range out of bounds");
    if (n_layers == 0) return TDK_OK;
    if (!host_master_k || !host_master_v || !io || !diffs || !pp)
      return fail(TDK_ERR_INVALID_ARG, "NULL argument");
    const size_t master_bytes = (size_t)r->total_master_rows * r->model.num_kv_heads * r->model.head_dim * 2;
    if (pp->stage_bytes < master_bytes) return fail(TDK_ERR_INVALID_ARG, "staging buffers smaller than one layer of masters");
    for (int b = 0; b < 2; ++b) {
      if (master_bytes && (!pp->stage_k[b] || !pp->stage_v[b])) return fail(TDK_ERR_INVALID_ARG, "staging buffer is NULL");
      if (((uintptr_t)pp->stage_k[b] | (uintptr_t)pp->stage_v[b]) & 15) return fail(TDK_ERR_INVALID_ARG, "staging buffers must be 16-byte aligned");
    }
    if (pp->stage_k[0] == pp->stage_k[1] || pp->stage_v[0] == pp->stage_v[1])
      return fail(TDK_ERR_INVALID_ARG, "the two staging buffers must be distinct");
    // validate every layer before anything is enqueued
    std::vector<tdk_layer_io> lio(n_layers);
    for (int32_t k = 0; k < n_layers; ++k) {
      if (master_bytes && (!host_master_k[k] || !host_master_v[k])) return fail(TDK_ERR_INVALID_ARG, "host master pointer is NULL");
      lio[k] = io[k];
      lio[k].master_k = pp->stage_k[k & 1];
      lio[k].master_v = pp->stage_v[k & 1];
      tdk_status st = check_step(r, first_layer + k, &lio[k]);
      if (st != TDK_OK) return st;
      st = check_diff(r, &diffs[k], false);
      if (st != TDK_OK) return st;
    }
    hipStream_t cs = static_cast<hipStream_t>(compute_stream);
    hipStream_t xs = static_cast<hipStream_t>(copy_stream);
    hipError_t e = hipSuccess;
    for (int32_t k = 0; k < n_layers; ++k) {
      const int b = k & 1;
      // load side: wait until the restore that last read this buffer (in this call or an earlier one)
      // is through, then stage layer k
      if (r->free_recorded[b]) {
        e = hipStreamWaitEvent(xs, r->ev_free[b], 0);
        if (e != hipSuccess) return hip_fail(e, "hipStreamWaitEvent(free)");
      }
      if (master_bytes) {
        e = hipMemcpyAsync(pp->stage_k[b], host_master_k[k], master_bytes, hipMemcpyHostToDevice, xs);
        if (e == hipSuccess) e = hipMemcpyAsync(pp->stage_v[b], host_master_v[k], master_bytes, hipMemcpyHostToDevice, xs);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(master chunk)");
      }
      e = hipEventRecord(r->ev_loaded[b], xs);
      if (e != hipSuccess) return hip_fail(e, "hipEventRecord(loaded)");
      // compute side: sync on the load, swap roles, apply the diff / recover positions / write back
      e = hipStreamWaitEvent(cs, r->ev_loaded[b], 0);
      if (e != hipSuccess) return hip_fail(e, "hipStreamWaitEvent(loaded)");
      const LayerDev l = layer_dev(&lio[k]);
      const DiffDev d = diff_dev(&diffs[k]);
      tdk_status rs = launch_restore(r, l, d, 3, diffs[k].capacity_pages, cs);
      if (rs != TDK_OK) return rs;
      e = hipEventRecord(r->ev_free[b], cs);
      if (e != hipSuccess) return hip_fail(e, "hipEventRecord(free)");
      r->free_recorded[b] = true;
    }
    return TDK_OK;
  });
}

tdk_status tdk_timing_enable(tdk_round* r, int32_t on) {
  if (!r) return fail(TDK_ERR_INVALID_ARG, "round is NULL");
  r->timing = on != 0;
  return TDK_OK;
}

static tdk_status drain_events(tdk_round* r) {
  return guarded([&]() -> tdk_status {
    for (auto& ev : r->pending) {
      hipError_t e = hipEventSynchronize(ev.stop);
      if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
      float ms = 0.f;
      e = hipEventElapsedTime(&ms, ev.start, ev.stop);
      if (e != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
      r->total_ms[ev.kernel] += ms;
      r->launches[ev.kernel] += 1;
      r->free_events.push_back(ev);
    }
    r->pending.clear();
    return TDK_OK;
  });
}

tdk_status tdk_timing_read(tdk_round* r, int32_t kernel, double* total_ms, int64_t* launches) {
  if (!r || !total_ms || !launches) return fail(TDK_ERR_INVALID_ARG, "NULL argument");
  if (kernel < 0 || kernel >= TDK_KERNEL_KINDS) return fail(TDK_ERR_INVALID_ARG, "kernel id out of range");
  tdk_status st = drain_events(r);
  if (st != TDK_OK) return st;
  *total_ms = r->total_ms[kernel];
  *launches = r->launches[kernel];
  return TDK_OK;
}

tdk_status tdk_timing_reset(tdk_round* r) {
  if (!r) return fail(TDK_ERR_INVALID_ARG, "round is NULL");
  tdk_status st = drain_events(r);
  if (st != TDK_OK) return st;
  for (int k = 0; k < TDK_KERNEL_KINDS; ++k) { r->total_ms[k] = 0; r->launches[k] = 0; }
  return TDK_OK;
}

double tdk_dense_bytes(const tdk_model* m, int64_t span_tokens) {
  if (!m) return 0.0;
  return (double)span_tokens * 2.0 * m->num_kv_heads * m->head_dim * 2.0;
}

double tdk_diff_bytes(const tdk_model* m, int64_t diff_pages) {
  if (!m) return 0.0;
  const double page = 2.0 * m->page_tokens * m->num_kv_heads * m->head_dim * 2.0;
  return diff_pages * page + diff_pages * 4.0 + 12.0;
}

double tdk_family_cost(int64_t n_agents, double ratio) { return 1.0 + (double)(n_agents - 1) / ratio; }

tdk_status tdk_util_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if ((bytes && (!dst || !src)) || (bytes & 15) || (((uintptr_t)dst | (uintptr_t)src) & 15))
    return fail(TDK_ERR_INVALID_ARG, "copy: NULL, misaligned or size not a multiple of 16");
  hipError_t e = launch_copy(static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), bytes / 16,
                             static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? TDK_OK : hip_fail(e, "copy kernel");
}

tdk_status tdk_util_fill(void* dst, uint32_t word, size_t bytes, void* hip_stream) {
  if ((bytes && !dst) || (bytes & 15) || ((uintptr_t)dst & 15))
    return fail(TDK_ERR_INVALID_ARG, "fill: NULL, misaligned or size not a multiple of 16");
  hipError_t e = launch_fill(static_cast<u32x4*>(dst), word, bytes / 16, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? TDK_OK : hip_fail(e, "fill kernel");
}

tdk_status tdk_util_page_fill(void* dst, const int32_t* page_ids, int32_t n_pages, size_t page_bytes,
                              uint32_t word, void* hip_stream) {
  if (n_pages < 0 || (n_pages && (!dst || !page_ids)) || (page_bytes & 15) || ((uintptr_t)dst & 15) ||
      page_bytes > ((size_t)1 << 30))
    return fail(TDK_ERR_INVALID_ARG, "page_fill: NULL, misaligned or bad size");
  hipError_t e = launch_page_fill(static_cast<u32x4*>(dst), page_ids, n_pages, (int)(page_bytes / 16), word,
                                  static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? TDK_OK : hip_fail(e, "page fill kernel");
}

tdk_status tdk_util_page_read(const void* src, const int32_t* page_ids, int32_t n_pages, size_t page_bytes,
                              void* sink16, void* hip_stream) {
  if (n_pages < 0 || (n_pages && (!src || !page_ids || !sink16)) || (page_bytes & 15) ||
      (((uintptr_t)src | (uintptr_t)sink16) & 15) || page_bytes > ((size_t)1 << 30))
    return fail(TDK_ERR_INVALID_ARG, "page_read: NULL, misaligned or bad size");
  hipError_t e = launch_page_read(static_cast<const u32x4*>(src), page_ids, n_pages, (int)(page_bytes / 16),
                                  static_cast<u32x4*>(sink16), static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? TDK_OK : hip_fail(e, "page read kernel");
}

tdk_status tdk_util_page_fill_product(void* plane_k, void* plane_v, const int32_t* page_ids, int32_t n_pages, int32_t group,
                                      int32_t num_kv_heads, int32_t page_tokens, uint32_t word, void* hip_stream) {
  if (n_pages < 0 || group < 1 || num_kv_heads < 1 || num_kv_heads > 8 || (page_tokens != 16 && page_tokens != 32) ||
      (n_pages && (!plane_k || !plane_v || !page_ids)) || (((uintptr_t)plane_k | (uintptr_t)plane_v) & 15))
    return fail(TDK_ERR_INVALID_ARG, "page_fill_product: NULL, misaligned or bad shape");
  hipError_t e = launch_page_fill_product(static_cast<u32x4*>(plane_k), static_cast<u32x4*>(plane_v), page_ids, n_pages, group,
                                          num_kv_heads, page_tokens, word, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? TDK_OK : hip_fail(e, "page fill kernel (product form)");
}

tdk_status tdk_util_page_read_product(const void* plane_k, const void* plane_v, const int32_t* page_ids, int32_t n_pages,
                                      int32_t group, int32_t num_kv_heads, int32_t page_tokens, void* sink16, void* hip_stream) {
  if (n_pages < 0 || group < 1 || num_kv_heads < 1 || num_kv_heads > 8 || (page_tokens != 16 && page_tokens != 32) ||
      (n_pages && (!plane_k || !plane_v || !page_ids || !sink16)) ||
      (((uintptr_t)plane_k | (uintptr_t)plane_v | (uintptr_t)sink16) & 15))
    return fail(TDK_ERR_INVALID_ARG, "page_read_product: NULL, misaligned or bad shape");
  hipError_t e = launch_page_read_product(static_cast<const u32x4*>(plane_k), static_cast<const u32x4*>(plane_v), page_ids, n_pages,
                                          group, num_kv_heads, page_tokens, static_cast<u32x4*>(sink16),
                                          static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? TDK_OK : hip_fail(e, "page read kernel (product form)");
}

size_t tdk_timeline_bytes(const tdk_round* r) {
  return r ? 32 * ((size_t)r->rd.n_work + 1) : 0;
}

tdk_status tdk_timeline_set(tdk_round* r, void* stamps, size_t bytes) {
  if (!r) return fail(TDK_ERR_INVALID_ARG, "round is NULL");
  if (stamps && (bytes < tdk_timeline_bytes(r) || ((uintptr_t)stamps & 7)))
    return fail(TDK_ERR_INVALID_ARG, "stamp buffer smaller than tdk_timeline_bytes() or misaligned");
  r->rd.stamps = static_cast<unsigned long long*>(stamps);
  return TDK_OK;
}

}  // extern "C"
