// C ABI of the batched dataflow-graph executor: context, index upload, level launch loop.
//
// Runtime pieces of the paper that live here (appendix "Other Details"): arena-style reuse
// of the index/scratch buffers across calls, asynchronous execution on the caller's stream,
// and one batched host-to-device transfer per forward call for all index lists.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "acrobat.h"
#include "cell_kernels.h"
#include "dfg_runtime.h"
#include "persistent_kernels.h"
#include "scheduler.h"
#include "tdc_runtime.h"

using namespace acrobat;

// Scratch of the entry point that allocates nothing (acrobat_treelstm_forward_noalloc): the device copy
// of the index lists, then the partial tiles of k-split levels.  One array per GPU, held until the
// process ends; every call on a GPU shares it.  In host code the array's name is only a handle: the
// device address comes from hipGetSymbolAddress, once per device (static_scratch_for).
constexpr size_t kStaticScratchBytes = (size_t)ACROBAT_NOALLOC_SCRATCH_MIB << 20;
constexpr size_t kStaticIndexBytes = (size_t)1 << 20;  // 3 int32 per node for ACROBAT_NOALLOC_MAX_NODES nodes
constexpr size_t kStaticCounterBytes = (size_t)32 << 10;  // tile counters of evenly split levels, at the end
static_assert(3 * sizeof(int32_t) * (size_t)ACROBAT_NOALLOC_MAX_NODES <= kStaticIndexBytes, "index region too small");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on `device`, which must be the current device.  Looked up once per device.
hipError_t static_scratch_for(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}
}  // namespace

namespace {
// One at a time per GPU for the launches whose workgroups wait for each other (the persistent recurrences, the
// MV-RNN dataflow launches): two of them sharing the compute units could each hold slots the other's missing
// workgroups need, and both would only end by the bound of their waits.  Launches from one stream are ordered
// anyway; when such a launch comes from another stream than the one before it (another context's, say), an event
// recorded on that earlier stream now - behind the earlier launch and whatever followed it - is what the new stream
// waits for first.  Costs nothing while one stream is in use.  Not applied to a launch that is being captured into
// a graph (a graph cannot wait for an event outside it): replays of such graphs must not overlap other launches
// of this kind.
struct WaitingLaunchGate {
  std::mutex m;
  hipEvent_t order = nullptr;
  hipStream_t last = nullptr;
  bool any = false;
};
WaitingLaunchGate g_gate[kMaxDevices];

hipError_t order_waiting_launch(int device, hipStream_t stream) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  WaitingLaunchGate& g = g_gate[device];
  std::lock_guard<std::mutex> lock(g.m);
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &st) != hipSuccess) (void)hipGetLastError();
  if (st != hipStreamCaptureStatusNone) return hipSuccess;
  if (g.any && g.last != stream) {
    if (!g.order) {
      const hipError_t e = hipEventCreateWithFlags(&g.order, hipEventDisableTiming);
      if (e != hipSuccess) return e;
    }
    if (hipEventRecord(g.order, g.last) == hipSuccess) {
      const hipError_t e = hipStreamWaitEvent(stream, g.order, 0);
      if (e != hipSuccess) return e;
    } else {
      (void)hipGetLastError();  // the earlier stream no longer exists: its work was ordered before its destruction returned
    }
  }
  g.last = stream;
  g.any = true;
  return hipSuccess;
}
}  // namespace

struct acrobat_ctx {
  int device = 0;
  std::string err;
  // last schedule (host): level_off / level_nodes, or the tree scheduler's own lists (what `last` names)
  int32_t n_levels = 0;
  std::vector<int32_t> level_off, level_nodes;
  TreeScheduler tree_scheduler;   // keeps its buffers from call to call
  TreeSchedule tree_schedule;
  std::vector<int32_t> leaf_tokens;
  const std::vector<int32_t>* last_off = &level_off;
  const std::vector<int32_t>* last_nodes = &level_nodes;
  // index staging: pinned host buffer -> device buffer, one copy per forward call
  int32_t* h_stage = nullptr;
  int32_t* h_stage_dev = nullptr;  // the staging buffer's address on the device side (kernels may read it in place)
  int32_t* d_idx = nullptr;
  size_t stage_cap = 0, idx_cap = 0;  // in int32 elements
  hipEvent_t stage_done = nullptr;    // the last upload out of h_stage has finished
  bool stage_pending = false;
  // the entry point that allocates nothing: a staging buffer of fixed size (made by acrobat_create) and
  // this device's address of the library's static scratch array
  int32_t* h_fixed_stage = nullptr;   // kStaticIndexBytes of pinned host memory
  hipEvent_t fixed_done = nullptr;    // the last upload out of h_fixed_stage has finished
  bool fixed_pending = false;
  unsigned char* static_scratch = nullptr;
  int32_t n_cu = 0;  // compute units of the device
  // scratch for the hoisted LSTM input transform
  float* d_scratch = nullptr;
  size_t scratch_cap = 0;  // in floats
  // split-k workspace of the cell kernels (allocated at the first forward call)
  SplitKWorkspace splitk;
  bool gather_fusion = true;  // false: explicit gather launches (ablation)
  int mvrnn_variant = 0;  // which MV-RNN level kernel (acrobat_set_tuning): 1 = streaming
  // tree generation: a zero row (previous-sibling state of a first child) and the scores on the host
  float* d_zero_row = nullptr;
  size_t zero_row_cap = 0;  // in floats
  float* h_scores = nullptr;
  size_t scores_cap = 0;  // in floats
  hipStream_t tdc_stream = nullptr;             // second group of instances (the first uses the caller's stream)
  hipEvent_t tdc_order = nullptr;               // orders the second stream behind the caller's at the start of a call
  // persistent kernels: arrival counters + status word on the device, the status word's copy on the host
  bool persistent = true;           // acrobat_set_persistent
  int32_t max_polls = 1 << 18;      // bound of every wait inside a persistent kernel
  unsigned* d_sync = nullptr;       // [kPersistSyncWords]: the probe's flag lines | arrival counters | status
  unsigned* h_status = nullptr;     // pinned host word that a kernel raises when one of its waits runs out
  bool sync_dirty = false;          // the arrival counters in d_sync may be non-zero: clear them before the next persistent recurrence
  unsigned* h_status_dev = nullptr; // the same word's address on the device side
  unsigned* d_node_flags = nullptr; // one word per arena row: the epoch of the call that last finished the node
  size_t node_flags_cap = 0;
  unsigned epoch = 0;               // of the last dataflow launch; never 0
  // profiling
  bool profiling = false;
  std::vector<acrobat_launch_record> records;
  std::vector<hipEvent_t> events;  // pool, two per record
};

struct acrobat_dfg {
  acrobat_ctx* ctx = nullptr;
  std::string err;
  Dfg graph;
  DfgBuckets buckets;
};

namespace {

int fail(acrobat_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->err = msg;
  return code;
}

int fail_hip(acrobat_ctx* ctx, hipError_t e, const char* what) {
  return fail(ctx, e == hipErrorOutOfMemory ? ACROBAT_ENOMEM : ACROBAT_EHIP,
              std::string(what) + ": " + hipGetErrorString(e));
}

#define HIP_TRY(ctx, expr)                                   \
  do {                                                       \
    hipError_t e_ = (expr);                                  \
    if (e_ != hipSuccess) return fail_hip(ctx, e_, #expr);   \
  } while (0)

bool stream_is_capturing(hipStream_t stream) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  return hipStreamIsCapturing(stream, &st) == hipSuccess && st != hipStreamCaptureStatusNone;
}

// Makes room for `n` int32 in the pinned staging buffer and the device index buffer and waits
// until a previous upload no longer reads the staging buffer.  While `stream` is being captured
// into a graph nothing may be allocated or waited for: the buffers must already be large enough
// (one uncaptured call of the same size beforehand does that), and the caller must keep other
// calls away from this context until it has finished with the graph, whose upload node reads the
// staging buffer at every replay.
int reserve_indices(acrobat_ctx* ctx, size_t n, hipStream_t stream) {
  const bool capturing = stream_is_capturing(stream);
  if (capturing) {
    if (n > ctx->stage_cap || n > ctx->idx_cap)
      return fail(ctx, ACROBAT_EINVAL, "stream capture: index buffers too small, run once without capture first");
    return ACROBAT_OK;
  }
  if (ctx->stage_pending) {
    HIP_TRY(ctx, hipEventSynchronize(ctx->stage_done));
    ctx->stage_pending = false;
  }
  if (n > ctx->stage_cap) {
    const size_t cap = n + n / 2 + 1024;
    if (ctx->h_stage) HIP_TRY(ctx, hipHostFree(ctx->h_stage));
    ctx->h_stage = nullptr;
    ctx->stage_cap = 0;
    HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->h_stage), cap * sizeof(int32_t), hipHostMallocDefault));
    ctx->stage_cap = cap;
    HIP_TRY(ctx, hipHostGetDevicePointer(reinterpret_cast<void**>(&ctx->h_stage_dev), ctx->h_stage, 0));
  }
  if (n > ctx->idx_cap) {
    const size_t cap = n + n / 2 + 1024;
    if (ctx->d_idx) HIP_TRY(ctx, hipFree(ctx->d_idx));  // waits for kernels still using it
    ctx->d_idx = nullptr;
    ctx->idx_cap = 0;
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->d_idx), cap * sizeof(int32_t)));
    ctx->idx_cap = cap;
  }
  return ACROBAT_OK;
}

int upload_indices(acrobat_ctx* ctx, size_t n, hipStream_t stream) {
  HIP_TRY(ctx, hipMemcpyAsync(ctx->d_idx, ctx->h_stage, n * sizeof(int32_t), hipMemcpyHostToDevice, stream));
  if (stream_is_capturing(stream)) return ACROBAT_OK;
  HIP_TRY(ctx, hipEventRecord(ctx->stage_done, stream));
  ctx->stage_pending = true;
  return ACROBAT_OK;
}

int reserve_scratch(acrobat_ctx* ctx, size_t n_floats, hipStream_t stream) {
  if (n_floats <= ctx->scratch_cap) return ACROBAT_OK;
  if (stream_is_capturing(stream)) return fail(ctx, ACROBAT_EINVAL, "stream capture: scratch too small, run once without capture first");
  if (ctx->d_scratch) HIP_TRY(ctx, hipFree(ctx->d_scratch));
  ctx->d_scratch = nullptr;
  ctx->scratch_cap = 0;
  HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->d_scratch), n_floats * sizeof(float)));
  ctx->scratch_cap = n_floats;
  return ACROBAT_OK;
}

// Partial-tile workspace of the k-split levels: 128 MiB.
int reserve_splitk(acrobat_ctx* ctx, hipStream_t stream) {
  if (ctx->splitk.partial) return ACROBAT_OK;
  if (stream_is_capturing(stream)) return fail(ctx, ACROBAT_EINVAL, "stream capture: workspace not allocated, run once without capture first");
  constexpr size_t kPartialFloats = (size_t)32 << 20;
  float* p = nullptr;
  HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&p), kPartialFloats * sizeof(float)));
  ctx->splitk.partial = p;
  ctx->splitk.partial_floats = kPartialFloats;
  // tile counters of the levels that are split evenly inside one launch: zero between launches
  constexpr int kCounters = 8192;
  unsigned* c = nullptr;
  HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&c), kCounters * sizeof(unsigned)));
  HIP_TRY(ctx, hipMemset(c, 0, kCounters * sizeof(unsigned)));
  ctx->splitk.counters = c;
  ctx->splitk.n_counters = kCounters;
  int cus = 0;
  HIP_TRY(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device));
  ctx->splitk.n_cu = cus;
  return ACROBAT_OK;
}

constexpr int kSyncWords = kPersistSyncWords;  // the probe's flag lines, arrival counters, then the status word
constexpr int kSyncWordsPadded = (kSyncWords + 3) / 4 * 4;

int reserve_sync(acrobat_ctx* ctx, hipStream_t stream) {
  if (ctx->d_sync) return ACROBAT_OK;
  if (stream_is_capturing(stream)) return fail(ctx, ACROBAT_EINVAL, "stream capture: counters not allocated, run once without capture first");
  HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->d_sync), kSyncWordsPadded * sizeof(unsigned)));
  HIP_TRY(ctx, hipMemset(ctx->d_sync, 0, kSyncWordsPadded * sizeof(unsigned)));
  HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->h_status), sizeof(unsigned), hipHostMallocDefault));
  *ctx->h_status = 0;
  HIP_TRY(ctx, hipHostGetDevicePointer(reinterpret_cast<void**>(&ctx->h_status_dev), ctx->h_status, 0));
  return ACROBAT_OK;
}

// The persistent recurrences count their workgroups in and out in the first words of d_sync and leave them zero
// (leave_block): a clearing launch is only needed after something else has used the words - the probe, or a
// launch whose wait ran out.  (While that condition has not been read with acrobat_device_status, launches give
// up at their first long wait anyway.)
int clean_counters(acrobat_ctx* ctx, hipStream_t stream) {
  if (!ctx->sync_dirty) return ACROBAT_OK;
  HIP_TRY(ctx, launch_fill_u32(ctx->d_sync, 0u, kRnnMaxBlocks * kPersistCounterStride, stream));
  if (!stream_is_capturing(stream)) ctx->sync_dirty = false;  // (a captured clearing launch has not run yet)
  return ACROBAT_OK;
}

// Per-launch timing when profiling is on: every launch gets its own start/stop events, which the
// runtime stamps with the kernel's begin and end (the k-split reduction kernel gets a record of its
// own, kind ACROBAT_K_SPLITK_REDUCE, right behind its level's record).
struct LaunchTimer {
  acrobat_ctx* ctx;
  hipStream_t stream;
  bool allowed = true;  // false: this call never times its launches, whatever the context's setting
  LaunchEvents ev;  // events of the launch that begin() announced (all null when profiling is off)
  bool on() const { return allowed && ctx->profiling; }
  int begin(int32_t kind, int32_t level, int32_t n) {
    ev = LaunchEvents();
    if (!on()) return ACROBAT_OK;
    if (stream_is_capturing(stream)) return fail(ctx, ACROBAT_EINVAL, "profiling cannot be combined with stream capture");
    const size_t first = 2 * ctx->records.size();
    while (ctx->events.size() < first + 4) {
      hipEvent_t e;
      HIP_TRY(ctx, hipEventCreate(&e));
      ctx->events.push_back(e);
    }
    ctx->records.push_back({kind, level, n, 0, 1, 0.0f});
    ev.start = ctx->events[first];
    ev.stop = ctx->events[first + 1];
    ev.reduce_start = ctx->events[first + 2];
    ev.reduce_stop = ctx->events[first + 3];
    return ACROBAT_OK;
  }
  int32_t* tile() { return on() ? &ctx->records.back().tile : nullptr; }
  int32_t* ksplit() { return on() ? &ctx->records.back().ksplit : nullptr; }
  int end() {
    if (!on()) return ACROBAT_OK;
    const acrobat_launch_record r = ctx->records.back();
    if (r.ksplit > 1) ctx->records.push_back({ACROBAT_K_SPLITK_REDUCE, r.level, r.n, r.tile, r.ksplit, 0.0f});
    return ACROBAT_OK;
  }
  int finish() {
    if (!on()) return ACROBAT_OK;
    HIP_TRY(ctx, hipStreamSynchronize(stream));
    for (size_t i = 0; i < ctx->records.size(); ++i)
      HIP_TRY(ctx, hipEventElapsedTime(&ctx->records[i].ms, ctx->events[2 * i], ctx->events[2 * i + 1]));
    return ACROBAT_OK;
  }
};

#define TRY(expr)                        \
  do {                                   \
    int rc_ = (expr);                    \
    if (rc_ != ACROBAT_OK) return rc_;   \
  } while (0)

// Executes the graph nodes `first`, `first + 1`, ... bucket by bucket on the stream.  Buckets of one
// (phase, depth) do not depend on each other; two neighbours with the same shapes share a launch.
int run_graph(acrobat_dfg* g, size_t first, hipStream_t stream);
// The launches of run_graph for nodes that g->buckets already holds.  The index lists are written to
// `st` (pinned host memory, 3 ints per node).  in_place null: st is the context's staging buffer and is
// uploaded to the device copy; else `in_place` is st's address on the device side and the kernels read
// the lists straight out of it - one command less in the chain of a short evaluation, for callers that
// wait for these launches before they write that memory again.
// `ws`: the k-split workspace these launches may use.  Callers that keep several groups of launches in
// flight on different streams hand every group a region of its own.
int launch_buckets(acrobat_dfg* g, hipStream_t stream, int32_t* st, const int32_t* in_place, const SplitKWorkspace& ws);

int begin_call(acrobat_ctx* ctx) {
  if (!ctx) return ACROBAT_EINVAL;
  ctx->err.clear();
  ctx->records.clear();
  ctx->last_off = &ctx->level_off;
  ctx->last_nodes = &ctx->level_nodes;
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  return ACROBAT_OK;
}

int run_graph(acrobat_dfg* g, size_t first, hipStream_t stream) {
  acrobat_ctx* ctx = g->ctx;
  g->graph.bucket(g->buckets, first);
  const size_t n = g->buckets.order.size();
  if (n == 0) return ACROBAT_OK;
  TRY(reserve_splitk(ctx, stream));
  TRY(reserve_indices(ctx, 3 * n, stream));
  TRY(launch_buckets(g, stream, ctx->h_stage, nullptr, ctx->splitk));
  return ACROBAT_OK;
}

int launch_buckets(acrobat_dfg* g, hipStream_t stream, int32_t* st, const int32_t* in_place, const SplitKWorkspace& ws) {
  acrobat_ctx* ctx = g->ctx;
  const std::vector<DfgNode>& nodes = g->graph.nodes();
  const size_t n = g->buckets.order.size();
  if (n == 0) return ACROBAT_OK;
  // by bucket position: row written | first operand row | second operand row
  for (size_t p = 0; p < n; ++p) {
    const DfgNode& x = nodes[g->buckets.order[p]];
    st[p] = x.out_row;
    st[n + p] = x.arg0;
    st[2 * n + p] = x.arg1;
  }
  const int32_t* idx = ctx->d_idx;
  if (in_place) {
    idx = in_place;
  } else {
    TRY(upload_indices(ctx, 3 * n, stream));
  }
  static const CellEpilogue kEpi[] = {EPI_TREE_LEAF, EPI_TREE_INTERNAL, EPI_LSTM_STEP, EPI_STORE_Z,
                                      EPI_RNN_STEP, EPI_RELU_OUT, EPI_STORE_Z1};
  auto level_args = [&](size_t b) {
    const int32_t off = g->buckets.off[b], cnt = g->buckets.off[b + 1] - off;
    const acrobat_op_desc& d = g->graph.ops()[g->buckets.op[b]];
    CellLevelArgs a{};
    a.n = cnt; a.H = d.H; a.nseg = d.nseg; a.kseg = d.kseg;
    a.src0 = d.src0; a.ld0 = d.ld0; a.idx0 = idx + n + off;
    a.src1 = d.src1; a.ld1 = d.ld1; a.idx1 = idx + 2 * n + off;
    a.W = d.W; a.ldw = d.ldw; a.bias = d.bias;
    a.out_rows = idx + off;
    a.h = d.h; a.c = d.c; a.cprev_src = d.cprev_src; a.zadd = d.zadd; a.zout = d.zout;
    a.n_cols = d.n_cols; a.y = d.y; a.ldo = d.ldo;
    return a;
  };
  auto same_batch_shape = [&](size_t b0, size_t b1) {
    const DfgNode& x = nodes[g->buckets.order[g->buckets.off[b0]]];
    const DfgNode& y = nodes[g->buckets.order[g->buckets.off[b1]]];
    if (x.phase != y.phase || x.depth != y.depth) return false;
    const acrobat_op_desc& d0 = g->graph.ops()[g->buckets.op[b0]];
    const acrobat_op_desc& d1 = g->graph.ops()[g->buckets.op[b1]];
    return d0.epilogue == d1.epilogue && d0.H == d1.H && d0.nseg == d1.nseg && d0.kseg == d1.kseg &&
           d0.epilogue != ACROBAT_EPI_RELU_OUT && d0.epilogue != ACROBAT_EPI_MVRNN;
  };
  LaunchTimer timer{ctx, stream};
  const size_t n_buckets = g->buckets.op.size();
  for (size_t b = 0; b < n_buckets; ++b) {
    const acrobat_op_desc& d = g->graph.ops()[g->buckets.op[b]];
    if (d.epilogue == ACROBAT_EPI_MVRNN) {
      const int32_t off = g->buckets.off[b];
      MvrnnLevelArgs m{};
      m.n = g->buckets.off[b + 1] - off;
      m.d = d.H;
      m.variant = ctx->mvrnn_variant;
      m.out_rows = idx + off;
      m.lsrc = idx + n + off;
      m.rsrc = idx + 2 * n + off;
      m.vec_tab = d.src0; m.mat_tab = d.src1;
      m.W = d.W; m.WM = d.W2;
      m.vec = d.h; m.mat = d.c;
      TRY(timer.begin(ACROBAT_K_DFG_BUCKET, (int32_t)b, m.n));
      HIP_TRY(ctx, launch_mvrnn_level(m, stream, timer.tile(), timer.ev));
      TRY(timer.end());
      continue;
    }
    const CellLevelArgs a = level_args(b);
    if (b + 1 < n_buckets && same_batch_shape(b, b + 1)) {
      const CellLevelArgs a1 = level_args(b + 1);
      TRY(timer.begin(ACROBAT_K_DFG_BUCKET, (int32_t)b, a.n + a1.n));
      HIP_TRY(ctx, launch_cell_level_pair(kEpi[d.epilogue], a, a1, stream, ws, timer.tile(), timer.ksplit(), timer.ev));
      TRY(timer.end());
      ++b;
      continue;
    }
    TRY(timer.begin(ACROBAT_K_DFG_BUCKET, (int32_t)b, a.n));
    HIP_TRY(ctx, launch_cell_level(kEpi[d.epilogue], a, stream, ws, timer.tile(), timer.ksplit(), timer.ev));
    TRY(timer.end());
  }
  return timer.finish();
}

}  // namespace

extern "C" {

const char* acrobat_strerror(int code) {
  switch (code) {
    case ACROBAT_OK: return "ok";
    case ACROBAT_EINVAL: return "invalid argument";
    case ACROBAT_ESTRUCT: return "malformed input structure";
    case ACROBAT_ENOMEM: return "out of memory";
    case ACROBAT_EHIP: return "HIP runtime error";
    case ACROBAT_ETIMEOUT: return "a wait inside a persistent kernel ran out";
    default: return "unknown error code";
  }
}

int acrobat_create(acrobat_ctx** out, int device) {
  if (!out) return ACROBAT_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return ACROBAT_EHIP;
  if (hipSetDevice(device) != hipSuccess) return ACROBAT_EHIP;
  acrobat_ctx* ctx = new (std::nothrow) acrobat_ctx();
  if (!ctx) return ACROBAT_ENOMEM;
  ctx->device = device;
  void* scratch_ptr = nullptr;
  if (hipEventCreateWithFlags(&ctx->stage_done, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&ctx->fixed_done, hipEventDisableTiming) != hipSuccess ||
      hipHostMalloc(reinterpret_cast<void**>(&ctx->h_fixed_stage), kStaticIndexBytes, hipHostMallocDefault) != hipSuccess ||
      static_scratch_for(device, &scratch_ptr) != hipSuccess) {
    (void)hipGetLastError();
    acrobat_destroy(ctx);
    return ACROBAT_EHIP;
  }
  ctx->static_scratch = static_cast<unsigned char*>(scratch_ptr);
  if (hipDeviceGetAttribute(&ctx->n_cu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) {
    acrobat_destroy(ctx);
    return ACROBAT_EHIP;
  }
  *out = ctx;
  return ACROBAT_OK;
}

void acrobat_destroy(acrobat_ctx* ctx) {
  if (!ctx) return;
  (void)hipSetDevice(ctx->device);
  if (ctx->stage_pending) (void)hipEventSynchronize(ctx->stage_done);
  if (ctx->fixed_pending) (void)hipEventSynchronize(ctx->fixed_done);
  if (ctx->h_fixed_stage) (void)hipHostFree(ctx->h_fixed_stage);
  if (ctx->fixed_done) (void)hipEventDestroy(ctx->fixed_done);
  if (ctx->d_idx) (void)hipFree(ctx->d_idx);
  if (ctx->d_scratch) (void)hipFree(ctx->d_scratch);
  if (ctx->splitk.partial) (void)hipFree(ctx->splitk.partial);
  if (ctx->splitk.counters) (void)hipFree(ctx->splitk.counters);
  if (ctx->h_stage) (void)hipHostFree(ctx->h_stage);
  if (ctx->d_sync) (void)hipFree(ctx->d_sync);
  if (ctx->d_node_flags) (void)hipFree(ctx->d_node_flags);
  if (ctx->h_status) (void)hipHostFree(ctx->h_status);
  if (ctx->d_zero_row) (void)hipFree(ctx->d_zero_row);
  if (ctx->h_scores) (void)hipHostFree(ctx->h_scores);
  if (ctx->tdc_stream) (void)hipStreamDestroy(ctx->tdc_stream);
  if (ctx->tdc_order) (void)hipEventDestroy(ctx->tdc_order);
  if (ctx->stage_done) (void)hipEventDestroy(ctx->stage_done);
  for (hipEvent_t e : ctx->events) (void)hipEventDestroy(e);
  delete ctx;
}

const char* acrobat_last_error(const acrobat_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int acrobat_schedule_trees(const acrobat_trees* trees, int32_t vocab, int32_t* n_levels,
                           int32_t* level_off, int32_t* level_nodes, int32_t* lrow, int32_t* rrow) {
  if (!trees || !n_levels || !level_off) return ACROBAT_EINVAL;
  try {
    // buffers kept per thread: a call allocates nothing once they have grown to the batch size
    static thread_local TreeScheduler scheduler;
    static thread_local TreeSchedule s;
    std::string err;
    const int rc = scheduler.begin(*trees, vocab, s, nullptr, err);
    if (rc != ACROBAT_OK) return rc;
    scheduler.finish(*trees, s);
    if (s.n_nodes > 0 && !level_nodes) return ACROBAT_EINVAL;
    *n_levels = s.n_levels;
    std::memcpy(level_off, s.level_off.data(), s.level_off.size() * sizeof(int32_t));
    const size_t bytes = (size_t)s.n_nodes * sizeof(int32_t);
    if (s.n_nodes > 0) {
      std::memcpy(level_nodes, s.level_nodes.data(), bytes);
      if (lrow) std::memcpy(lrow, s.lrow.data(), bytes);
      if (rrow) std::memcpy(rrow, s.rrow.data(), bytes);
    }
    return ACROBAT_OK;
  } catch (const std::bad_alloc&) {
    return ACROBAT_ENOMEM;
  } catch (...) {
    return ACROBAT_EINVAL;
  }
}

int acrobat_schedule_seqs(int32_t n_seq, const int32_t* len, int32_t* n_levels, int32_t* level_off,
                          int32_t* level_rows) {
  if (!n_levels || !level_off) return ACROBAT_EINVAL;
  try {
    SeqSchedule s;
    std::string err;
    const int rc = schedule_seqs(n_seq, len, s, err);
    if (rc != ACROBAT_OK) return rc;
    if (s.n_rows > 0 && !level_rows) return ACROBAT_EINVAL;
    *n_levels = s.n_levels;
    std::memcpy(level_off, s.level_off.data(), s.level_off.size() * sizeof(int32_t));
    if (s.n_rows > 0) std::memcpy(level_rows, s.level_rows.data(), (size_t)s.n_rows * sizeof(int32_t));
    return ACROBAT_OK;
  } catch (const std::bad_alloc&) {
    return ACROBAT_ENOMEM;
  } catch (...) {
    return ACROBAT_EINVAL;
  }
}

}  // extern "C"

namespace {

// acrobat_treelstm_forward and its variant that allocates nothing.  `noalloc`: the index lists are staged in
// the context's fixed pinned buffer and uploaded into the library's static device array, which also holds the
// partial tiles of k-split levels; nothing is allocated or freed, no per-launch events are made (profiling is
// ignored) and the unfused-gather ablation, which needs scratch, is not available.
int treelstm_forward(acrobat_ctx* ctx, const acrobat_trees* trees, int32_t H, int32_t D, int32_t V, const float* d_emb,
                     const float* d_Wleaf, const float* d_bleaf, const float* d_U, const float* d_b, float* d_h,
                     float* d_c, void* hip_stream, const bool noalloc) {
  try {
    TRY(begin_call(ctx));
    if (!trees) return fail(ctx, ACROBAT_EINVAL, "trees is null");
    if (H <= 0 || D <= 0 || H % 32 || D % 32) return fail(ctx, ACROBAT_EINVAL, "H and D must be positive multiples of 32");
    if (V <= 0) return fail(ctx, ACROBAT_EINVAL, "V must be positive");
    // Phase 1 of the schedule: the whole structure is validated (nothing is launched for malformed input),
    // depths and level sizes are known and the leaves are listed with their tokens; phase 2 sorts the
    // internal levels.
    TreeSchedule& s = ctx->tree_schedule;
    ctx->n_levels = 0;
    ctx->last_off = &s.level_off;
    ctx->last_nodes = &s.level_nodes;
    {
      const int rc = ctx->tree_scheduler.begin(*trees, V, s, &ctx->leaf_tokens, ctx->err);
      if (rc != ACROBAT_OK) {
        s.level_off.assign(1, 0);
        s.level_nodes.clear();
        return rc;
      }
    }
    ctx->n_levels = s.n_levels;
    const int32_t N = s.n_nodes;
    if (N == 0) return ACROBAT_OK;
    if (!d_emb || !d_Wleaf || !d_U || !d_h || !d_c) {
      ctx->tree_scheduler.finish(*trees, s);
      return fail(ctx, ACROBAT_EINVAL, "a device pointer is null");
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    struct FinishOnExit {  // whatever happens below, acrobat_last_schedule reports the complete schedule
      acrobat_ctx* ctx; const acrobat_trees* trees; bool done = false;
      void now() { if (!done) ctx->tree_scheduler.finish(*trees, ctx->tree_schedule); done = true; }
      ~FinishOnExit() { now(); }
    } finish{ctx, trees};
    if ((double)5 * H * 2 * H >= 2147483648.0 || (double)5 * H * D >= 2147483648.0)
      return fail(ctx, ACROBAT_EINVAL, "weight matrix has 2^31 or more elements");
    if (noalloc && N > ACROBAT_NOALLOC_MAX_NODES)
      return fail(ctx, ACROBAT_EINVAL, "acrobat_treelstm_forward_noalloc: more than ACROBAT_NOALLOC_MAX_NODES (" +
                                           std::to_string(ACROBAT_NOALLOC_MAX_NODES) + ") nodes");
    // index lists by schedule position: out row | first operand row | second operand row
    // (+ 0, 1, 2, ... for the unfused-gather ablation, whose level kernels read gathered copies)
    const int32_t n_leaf = s.level_off[1];
    int32_t n_wide = 0;  // widest internal level
    for (int32_t lv = 1; lv < s.n_levels; ++lv) n_wide = std::max(n_wide, s.level_off[lv + 1] - s.level_off[lv]);
    const bool unfused = !ctx->gather_fusion && !noalloc;
    const size_t n_iota = unfused ? (size_t)std::max(n_leaf, 2 * n_wide) : 0;
    // (Uploading the leaf lists and launching level 0 before the internal levels are sorted was measured and
    // dropped: the second upload sits behind the leaf kernel in stream order, so its three copy commands land
    // between level 0 and level 1 - 0.731 instead of 0.691 ms per forward on 17 134 nodes - while the sort
    // it would hide takes 20 us and is hidden anyway whenever a forward call is already queued.)
    int32_t* st = nullptr;     // pinned staging
    int32_t* d_idx = nullptr;  // its device copy
    SplitKWorkspace ws;
    if (noalloc) {
      if (ctx->fixed_pending) {  // the previous upload out of the fixed staging buffer must be through
        HIP_TRY(ctx, hipEventSynchronize(ctx->fixed_done));
        ctx->fixed_pending = false;
      }
      st = ctx->h_fixed_stage;
      d_idx = reinterpret_cast<int32_t*>(ctx->static_scratch);
      ws = ctx->splitk;  // tuning hook settings
      ws.partial = reinterpret_cast<float*>(ctx->static_scratch + kStaticIndexBytes);
      ws.partial_floats = (kStaticScratchBytes - kStaticIndexBytes - kStaticCounterBytes) / sizeof(float);
      // the tile counters: a region nothing else ever writes, zero when the library is loaded and whenever no
      // launch is in flight
      ws.counters = reinterpret_cast<unsigned*>(ctx->static_scratch + kStaticScratchBytes - kStaticCounterBytes);
      ws.n_counters = (int32_t)(kStaticCounterBytes / sizeof(unsigned));
      ws.n_cu = ctx->n_cu;
    } else {
      TRY(reserve_splitk(ctx, stream));
      TRY(reserve_indices(ctx, 3 * (size_t)N + n_iota, stream));
      st = ctx->h_stage;
      d_idx = ctx->d_idx;
      ws = ctx->splitk;
    }
    // staging layout: out row | first operand row (token at a leaf) | second operand row, N entries each
    const size_t n_int = (size_t)(N - n_leaf);
    auto stage_leaves = [&]() {
      std::memcpy(st, s.level_nodes.data(), (size_t)n_leaf * sizeof(int32_t));
      std::memcpy(st + N, ctx->leaf_tokens.data(), (size_t)n_leaf * sizeof(int32_t));  // leaves gather by token
    };
    auto stage_internal = [&]() {
      std::memcpy(st + n_leaf, s.level_nodes.data() + n_leaf, n_int * sizeof(int32_t));
      std::memcpy(st + N + n_leaf, s.lrow.data() + n_leaf, n_int * sizeof(int32_t));
      std::memcpy(st + 2 * (size_t)N + n_leaf, s.rrow.data() + n_leaf, n_int * sizeof(int32_t));
    };
    auto copy_up = [&](size_t first, size_t count) {
      return hipMemcpyAsync(d_idx + first, st + first, count * sizeof(int32_t), hipMemcpyHostToDevice, stream);
    };
    auto staging_in_flight = [&]() {  // the staging buffer may be rewritten once these uploads are through
      if (stream_is_capturing(stream)) return hipSuccess;
      const hipError_t e = hipEventRecord(noalloc ? ctx->fixed_done : ctx->stage_done, stream);
      (noalloc ? ctx->fixed_pending : ctx->stage_pending) = true;
      return e;
    };
    if (unfused) TRY(reserve_scratch(ctx, std::max((size_t)n_leaf * D, 4 * (size_t)n_wide * H), stream));
    finish.now();
    stage_leaves();
    stage_internal();
    for (size_t i = 0; i < n_iota; ++i) st[3 * (size_t)N + i] = (int32_t)i;
    HIP_TRY(ctx, copy_up(0, 3 * (size_t)N + n_iota));  // one upload (the second operands of level 0 are never read)
    HIP_TRY(ctx, staging_in_flight());
    const int32_t* d_out = d_idx;
    const int32_t* d_ia = d_idx + N;
    const int32_t* d_ib = d_idx + 2 * (size_t)N;
    const int32_t* d_iota = d_idx + 3 * (size_t)N;

    LaunchTimer timer{ctx, stream, !noalloc};
    for (int32_t lv = 0; lv < s.n_levels; ++lv) {
      const int32_t off = s.level_off[lv], n = s.level_off[lv + 1] - off;
      CellLevelArgs a{};
      a.n = n;
      a.H = H;
      a.out_rows = d_out + off;
      a.h = d_h;
      a.c = d_c;
      if (lv == 0) {
        a.nseg = 1; a.kseg = D;
        a.src0 = d_emb; a.idx0 = d_ia + off; a.ld0 = D;
        a.W = d_Wleaf; a.ldw = D; a.bias = d_bleaf;
      } else {
        a.nseg = 2; a.kseg = H;
        a.src0 = d_h; a.idx0 = d_ia + off; a.ld0 = H;
        a.src1 = d_h; a.idx1 = d_ib + off; a.ld1 = H;
        a.W = d_U; a.ldw = 2 * H; a.bias = d_b;
        a.cprev_src = d_c;
      }
      if (unfused) {  // copy the operand rows first, then let the level kernel read the copies in order
        GatherArgs g{};
        g.n = n;
        float* hbuf = ctx->d_scratch;                        // [2n, H]: left rows, right rows
        float* cbuf = ctx->d_scratch + 2 * (size_t)n_wide * H;  // same for c
        if (lv == 0) {
          g.width = D; g.count = 1;
          g.idx[0] = a.idx0; g.src[0] = d_emb; g.dst[0] = ctx->d_scratch;
          a.src0 = ctx->d_scratch; a.idx0 = d_iota;
        } else {
          g.width = H; g.count = 4;
          g.idx[0] = a.idx0; g.src[0] = d_h; g.dst[0] = hbuf;
          g.idx[1] = a.idx1; g.src[1] = d_h; g.dst[1] = hbuf + (size_t)n * H;
          g.idx[2] = a.idx0; g.src[2] = d_c; g.dst[2] = cbuf;
          g.idx[3] = a.idx1; g.src[3] = d_c; g.dst[3] = cbuf + (size_t)n * H;
          a.src0 = hbuf; a.src1 = hbuf; a.idx0 = d_iota; a.idx1 = d_iota + n;
          a.cprev_src = cbuf;
        }
        TRY(timer.begin(ACROBAT_K_GATHER, lv, n));
        HIP_TRY(ctx, launch_gather_rows(g, stream, timer.ev));
        TRY(timer.end());
      }
      TRY(timer.begin(lv == 0 ? ACROBAT_K_TREE_LEAF : ACROBAT_K_TREE_INTERNAL, lv, n));
      HIP_TRY(ctx, launch_cell_level(lv == 0 ? EPI_TREE_LEAF : EPI_TREE_INTERNAL, a, stream, ws,
                                     timer.tile(), timer.ksplit(), timer.ev));
      TRY(timer.end());
    }
    return timer.finish();
  } catch (const std::bad_alloc&) {
    return fail(ctx, ACROBAT_ENOMEM, "host allocation failed");
  } catch (...) {
    return fail(ctx, ACROBAT_EINVAL, "unexpected exception");
  }
}

}  // namespace

extern "C" {

int acrobat_treelstm_forward(acrobat_ctx* ctx, const acrobat_trees* trees, int32_t H, int32_t D,
                             int32_t V, const float* d_emb, const float* d_Wleaf,
                             const float* d_bleaf, const float* d_U, const float* d_b, float* d_h,
                             float* d_c, void* hip_stream) {
  return treelstm_forward(ctx, trees, H, D, V, d_emb, d_Wleaf, d_bleaf, d_U, d_b, d_h, d_c, hip_stream, false);
}

int acrobat_treelstm_forward_noalloc(acrobat_ctx* ctx, const acrobat_trees* trees, int32_t H, int32_t D,
                                     int32_t V, const float* d_emb, const float* d_Wleaf,
                                     const float* d_bleaf, const float* d_U, const float* d_b, float* d_h,
                                     float* d_c, void* hip_stream) {
  return treelstm_forward(ctx, trees, H, D, V, d_emb, d_Wleaf, d_bleaf, d_U, d_b, d_h, d_c, hip_stream, true);
}

int acrobat_mvrnn_forward(acrobat_ctx* ctx, const acrobat_trees* trees, int32_t d, int32_t V,
                          const float* d_vec_tab, const float* d_mat_tab, const float* d_W,
                          const float* d_WM, float* d_vec, float* d_mat, int32_t copy_leaves,
                          void* hip_stream) {
  try {
    TRY(begin_call(ctx));
    if (!trees) return fail(ctx, ACROBAT_EINVAL, "trees is null");
    if (d != 64 && d != 128) return fail(ctx, ACROBAT_EINVAL, "only d == 64 and d == 128 are supported");
    if (V <= 0) return fail(ctx, ACROBAT_EINVAL, "V must be positive");
    TreeSchedule& s = ctx->tree_schedule;
    ctx->n_levels = 0;
    ctx->last_off = &s.level_off;
    ctx->last_nodes = &s.level_nodes;
    {
      const int rc = ctx->tree_scheduler.begin(*trees, V, s, nullptr, ctx->err);
      if (rc != ACROBAT_OK) {
        s.level_off.assign(1, 0);
        s.level_nodes.clear();
        return rc;
      }
      ctx->tree_scheduler.finish(*trees, s);
    }
    ctx->n_levels = s.n_levels;
    const int32_t N = s.n_nodes;
    if (N == 0) return ACROBAT_OK;
    if (!d_vec_tab || !d_mat_tab || !d_W || !d_WM || !d_vec || !d_mat)
      return fail(ctx, ACROBAT_EINVAL, "a device pointer is null");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    // child source codes: arena row of an internal child, -(token + 1) for a leaf child
    TRY(reserve_indices(ctx, 3 * (size_t)N, stream));
    int32_t* st = ctx->h_stage;
    std::memcpy(st, s.level_nodes.data(), (size_t)N * sizeof(int32_t));
    const int32_t n_leaf = s.level_off[1];
    for (int32_t p = 0; p < n_leaf; ++p) {
      st[N + p] = trees->token[s.level_nodes[p]];
      st[2 * (size_t)N + p] = -1;
    }
    auto code = [&](int32_t g) { return trees->left[g] < 0 ? -(trees->token[g] + 1) : g; };
    for (int32_t p = n_leaf; p < N; ++p) {
      st[N + p] = code(s.lrow[p]);
      st[2 * (size_t)N + p] = code(s.rrow[p]);
    }
    TRY(upload_indices(ctx, 3 * (size_t)N, stream));
    const int32_t* d_out = ctx->d_idx;
    const int32_t* d_ia = ctx->d_idx + N;
    const int32_t* d_ib = ctx->d_idx + 2 * (size_t)N;

    LaunchTimer timer{ctx, stream};
    if (copy_leaves) {
      TRY(timer.begin(ACROBAT_K_MVRNN_LEAFCOPY, 0, n_leaf));
      HIP_TRY(ctx, launch_mvrnn_leaf_copy(n_leaf, d, d_out, d_ia, d_vec_tab, d_mat_tab, d_vec, d_mat, stream, timer.ev));
      TRY(timer.end());
    }
    // One launch for all internal levels where the kernel exists (d = 64) and every workgroup is resident at
    // once: a node then waits for its own two children instead of a whole level for the previous one.
    const int32_t n_internal = N - n_leaf;
    // (Batches with very wide levels keep one launch per level: at 1 024 trees the single launch is 10 % slower,
    // 0.54 vs 0.49 ms - its flag checks and write-through stores buy nothing where levels are bandwidth bound.)
    int32_t widest = 0;
    for (int32_t lv = 1; lv < s.n_levels; ++lv) widest = std::max(widest, s.level_off[lv + 1] - s.level_off[lv]);
    const int32_t widest_limit = d == 64 ? 2048 : 512;  // (a d = 128 node is four times the bytes)
    const size_t flag_words = (size_t)N * 4;  // one per workgroup of a node
    // d = 64: four workgroups per node while the levels are narrow enough for a node's latency to be what counts
    // (the configuration of 64 trees, widest level 563: 0.097 against 0.100 ms; 16 trees 0.063 against 0.073;
    // 96 trees, widest level 850: 0.120 against 0.117, 192 trees 0.168 against 0.145 - every workgroup of a node
    // reads both child matrices whole)
    const bool quarters = d == 64 && widest <= 640;
    const int df_wgs = ctx->persistent && ctx->mvrnn_variant == 0 && s.n_levels > 2 && widest <= widest_limit &&
                               !stream_is_capturing(stream)
                           ? mvrnn_dataflow_workgroups(d, n_internal, quarters) : 0;
    if (df_wgs > 0) {
      TRY(reserve_sync(ctx, stream));
      if (flag_words > ctx->node_flags_cap) {
        const size_t cap = flag_words + flag_words / 2 + 1024;
        if (ctx->d_node_flags) HIP_TRY(ctx, hipFree(ctx->d_node_flags));
        ctx->d_node_flags = nullptr;
        ctx->node_flags_cap = 0;
        HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->d_node_flags), cap * sizeof(unsigned)));
        HIP_TRY(ctx, hipMemsetAsync(ctx->d_node_flags, 0, cap * sizeof(unsigned), stream));
        ctx->node_flags_cap = cap;
      }
      if (++ctx->epoch == 0) {  // wrapped: every stale word could pass for a fresh one
        HIP_TRY(ctx, hipMemsetAsync(ctx->d_node_flags, 0, ctx->node_flags_cap * sizeof(unsigned), stream));
        ctx->epoch = 1;
      }
      MvrnnLevelArgs a{};
      a.n = n_internal;
      a.d = d;
      a.out_rows = d_out + n_leaf;
      a.lsrc = d_ia + n_leaf;
      a.rsrc = d_ib + n_leaf;
      a.vec_tab = d_vec_tab; a.mat_tab = d_mat_tab;
      a.W = d_W; a.WM = d_WM;
      a.vec = d_vec; a.mat = d_mat;
      a.flags = ctx->d_node_flags; a.epoch = ctx->epoch;
      a.status = ctx->h_status_dev; a.max_polls = ctx->max_polls;
      TRY(timer.begin(ACROBAT_K_MVRNN_PERSISTENT, 1, n_internal));
      HIP_TRY(ctx, order_waiting_launch(ctx->device, stream));
      HIP_TRY(ctx, launch_mvrnn_dataflow(a, df_wgs, quarters, stream, timer.ev));
      TRY(timer.end());
      return timer.finish();
    }
    for (int32_t lv = 1; lv < s.n_levels; ++lv) {
      const int32_t off = s.level_off[lv], n = s.level_off[lv + 1] - off;
      MvrnnLevelArgs a{};
      a.n = n;
      a.d = d;
      a.variant = ctx->mvrnn_variant;
      a.out_rows = d_out + off;
      a.lsrc = d_ia + off;
      a.rsrc = d_ib + off;
      a.vec_tab = d_vec_tab; a.mat_tab = d_mat_tab;
      a.W = d_W; a.WM = d_WM;
      a.vec = d_vec; a.mat = d_mat;
      TRY(timer.begin(ACROBAT_K_MVRNN_LEVEL, lv, n));
      HIP_TRY(ctx, launch_mvrnn_level(a, stream, timer.tile(), timer.ev));
      TRY(timer.end());
    }
    return timer.finish();
  } catch (const std::bad_alloc&) {
    return fail(ctx, ACROBAT_ENOMEM, "host allocation failed");
  } catch (...) {
    return fail(ctx, ACROBAT_EINVAL, "unexpected exception");
  }
}

int acrobat_varlen_lstm_forward(acrobat_ctx* ctx, int32_t n_seq, const int32_t* len, int32_t H,
                                int32_t D, const float* d_x, const float* d_Wx,
                                const float* d_Wh, const float* d_b, float* d_h, float* d_c,
                                void* hip_stream) {
  try {
    TRY(begin_call(ctx));
    if (H <= 0 || D <= 0 || H % 32 || D % 32) return fail(ctx, ACROBAT_EINVAL, "H and D must be positive multiples of 32");
    SeqSchedule s;
    {
      const int rc = schedule_seqs(n_seq, len, s, ctx->err);
      if (rc != ACROBAT_OK) return rc;
    }
    ctx->n_levels = s.n_levels;
    ctx->level_off = s.level_off;
    ctx->level_nodes = s.level_rows;
    const int32_t R = (int32_t)s.n_rows;
    if (R == 0) return ACROBAT_OK;
    if (!d_x || !d_Wx || !d_Wh || !d_h || !d_c) return fail(ctx, ACROBAT_EINVAL, "a device pointer is null");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    if ((double)4 * H * H >= 2147483648.0 || (double)4 * H * D >= 2147483648.0)
      return fail(ctx, ACROBAT_EINVAL, "weight matrix has 2^31 or more elements");
    TRY(reserve_splitk(ctx, stream));
    TRY(reserve_scratch(ctx, (size_t)R * 4 * (size_t)H, stream));
    auto input_transform = [&](LaunchTimer& timer) {  // hoisted: every step of every sequence in one dense batch
      CellLevelArgs a{};
      a.n = R; a.H = H; a.nseg = 1; a.kseg = D;
      a.src0 = d_x; a.ld0 = D;
      a.W = d_Wx; a.ldw = D; a.bias = d_b;
      a.zout = ctx->d_scratch;
      TRY(timer.begin(ACROBAT_K_LSTM_INPUT, 0, R));
      HIP_TRY(ctx, launch_cell_level(EPI_STORE_Z, a, stream, ctx->splitk, timer.tile(), timer.ksplit(), timer.ev));
      return timer.end();
    };

    // One launch for the whole recurrence where the shape allows it: the steps are the same batches in the
    // same order, executed by workgroups that keep W_h on chip and synchronise among themselves.
    const int32_t n_live = s.level_off[1];  // sequences with at least one step
    const int32_t slots = kLstmSlots;
    const int32_t n_blocks = (n_live + slots - 1) / slots;
    if (ctx->persistent && s.n_levels >= 2 && (double)R * H * sizeof(float) < 4294967296.0 &&
        lstm_persistent_eligible(H, n_blocks, nullptr)) {
      TRY(reserve_sync(ctx, stream));
      const size_t n_slots = (size_t)n_blocks * slots;
      TRY(reserve_indices(ctx, 2 * n_slots, stream));
      int32_t* st = ctx->h_stage;
      // sequences by non-increasing length (ties by id): a counting sort over the lengths; rank r goes to block
      // r / slots, slot r % slots, so a block's live slots are a prefix at every step, its sequences are of
      // similar length (few dead rows in its products) and the blocks of short sequences leave the chip early
      std::vector<int32_t> first(s.n_levels + 2, 0);  // first[l]: count, then rank of the first sequence of length l
      for (int32_t q = 0; q < n_seq; ++q)
        if (len[q] > 0) ++first[len[q]];
      for (int32_t l = s.n_levels, run = 0; l >= 1; --l) {
        const int32_t cnt = first[l];
        first[l] = run;
        run += cnt;
      }
      std::fill(st, st + 2 * n_slots, 0);
      int32_t row0 = 0;
      for (int32_t q = 0; q < n_seq; ++q) {
        if (len[q] > 0) {
          const int32_t r = first[len[q]]++;
          const size_t slot = (size_t)r;  // block r / slots, slot r % slots
          st[slot] = row0;
          st[n_slots + slot] = len[q];
        }
        row0 += len[q];
      }
      TRY(upload_indices(ctx, 2 * n_slots, stream));
      LaunchTimer timer{ctx, stream};
      TRY(clean_counters(ctx, stream));
      TRY(input_transform(timer));
      LstmPersistentArgs pa{};
      pa.n_blocks = n_blocks; pa.H = H;
      pa.slot_row0 = ctx->d_idx; pa.slot_len = ctx->d_idx + n_slots;
      pa.Wh = d_Wh; pa.xp = ctx->d_scratch; pa.h = d_h; pa.c = d_c;
      pa.h_bytes = (uint32_t)((size_t)R * H * sizeof(float));
      pa.counters = ctx->d_sync; pa.status = ctx->h_status_dev;
      pa.max_polls = ctx->max_polls;
      TRY(timer.begin(ACROBAT_K_LSTM_PERSISTENT, 0, R));
      if (timer.tile()) *timer.tile() = 16;
      HIP_TRY(ctx, order_waiting_launch(ctx->device, stream));
      HIP_TRY(ctx, launch_lstm_persistent(pa, stream, timer.ev));
      TRY(timer.end());
      return timer.finish();
    }

    // by schedule position: row written | row of the previous step (unused at t = 0)
    TRY(reserve_indices(ctx, 2 * (size_t)R, stream));
    int32_t* st = ctx->h_stage;
    std::memcpy(st, s.level_rows.data(), (size_t)R * sizeof(int32_t));
    for (int32_t p = 0; p < R; ++p) st[R + p] = s.level_rows[p] - 1;
    for (int32_t p = 0; p < s.level_off[1]; ++p) st[R + p] = s.level_rows[p];  // keep in range
    TRY(upload_indices(ctx, 2 * (size_t)R, stream));
    const int32_t* d_out = ctx->d_idx;
    const int32_t* d_prev = ctx->d_idx + R;

    LaunchTimer timer{ctx, stream};
    TRY(input_transform(timer));
    for (int32_t t = 0; t < s.n_levels; ++t) {
      const int32_t off = s.level_off[t], n = s.level_off[t + 1] - off;
      CellLevelArgs a{};
      a.n = n; a.H = H;
      a.out_rows = d_out + off;
      a.h = d_h; a.c = d_c;
      a.zadd = ctx->d_scratch;
      a.W = d_Wh; a.ldw = H;
      if (t > 0) {
        a.nseg = 1; a.kseg = H;
        a.src0 = d_h; a.idx0 = d_prev + off; a.ld0 = H;
        a.cprev_src = d_c;
      }
      TRY(timer.begin(ACROBAT_K_LSTM_STEP, t, n));
      HIP_TRY(ctx, launch_cell_level(EPI_LSTM_STEP, a, stream, ctx->splitk, timer.tile(), timer.ksplit(), timer.ev));
      TRY(timer.end());
    }
    return timer.finish();
  } catch (const std::bad_alloc&) {
    return fail(ctx, ACROBAT_ENOMEM, "host allocation failed");
  } catch (...) {
    return fail(ctx, ACROBAT_EINVAL, "unexpected exception");
  }
}

int acrobat_schedule_birnn(int32_t n_seq, const int32_t* len, int32_t* n_levels, int32_t* level_off,
                           int32_t* level_codes) {
  if (!n_levels || !level_off) return ACROBAT_EINVAL;
  try {
    BirnnSchedule s;
    std::string err;
    const int rc = schedule_birnn(n_seq, len, s, err);
    if (rc != ACROBAT_OK) return rc;
    if (s.n_rows > 0 && !level_codes) return ACROBAT_EINVAL;
    *n_levels = s.n_levels;
    std::memcpy(level_off, s.level_off.data(), s.level_off.size() * sizeof(int32_t));
    if (s.n_rows > 0) std::memcpy(level_codes, s.level_codes.data(), s.level_codes.size() * sizeof(int32_t));
    return ACROBAT_OK;
  } catch (const std::bad_alloc&) {
    return ACROBAT_ENOMEM;
  } catch (...) {
    return ACROBAT_EINVAL;
  }
}

int acrobat_birnn_forward(acrobat_ctx* ctx, int32_t n_seq, const int32_t* len, int32_t H, int32_t D,
                          int32_t n_out, const float* d_x, const acrobat_rnn_dir* fwd,
                          const acrobat_rnn_dir* bwd, const float* d_C, const float* d_cb,
                          float* d_hf, float* d_hb, float* d_y, void* hip_stream) {
  try {
    TRY(begin_call(ctx));
    if (H <= 0 || D <= 0 || H % 32 || D % 32) return fail(ctx, ACROBAT_EINVAL, "H and D must be positive multiples of 32");
    if (n_out < 1) return fail(ctx, ACROBAT_EINVAL, "n_out must be positive");
    BirnnSchedule s;
    {
      const int rc = schedule_birnn(n_seq, len, s, ctx->err);
      if (rc != ACROBAT_OK) return rc;
    }
    ctx->n_levels = s.n_levels;
    ctx->level_off = s.level_off;
    ctx->level_nodes = s.level_codes;
    const int32_t R = (int32_t)s.n_rows;
    if (R == 0) return ACROBAT_OK;
    if (!fwd || !bwd) return fail(ctx, ACROBAT_EINVAL, "a direction's parameter block is null");
    if (!d_x || !d_C || !d_hf || !d_hb || !d_y || !fwd->Wx || !fwd->Wh || !fwd->h_init || !bwd->Wx || !bwd->Wh ||
        !bwd->h_init)
      return fail(ctx, ACROBAT_EINVAL, "a device pointer is null");
    if ((double)H * H >= 2147483648.0 || (double)H * D >= 2147483648.0 || (double)n_out * 2 * H >= 2147483648.0)
      return fail(ctx, ACROBAT_EINVAL, "weight matrix has 2^31 or more elements");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int32_t T = s.n_levels - 1;  // recurrence steps; level T is the output batch
    TRY(reserve_splitk(ctx, stream));
    // One launch for both recurrences where the shape allows it (see the LSTM forward call): the steps are the
    // same batches, executed by workgroups that keep W_h on chip and synchronise among themselves.
    const int32_t n_live = s.fwd_off[1];  // sequences with at least one token
    const int32_t blocks_per_dir = (n_live + kRnnSlots - 1) / kRnnSlots;
    const bool persistent = ctx->persistent && T >= 2 && (double)R * H * sizeof(float) < 4294967296.0 &&
                            rnn_persistent_eligible(H, 2 * blocks_per_dir, nullptr);
    const size_t n_slots = (size_t)blocks_per_dir * kRnnSlots;
    if (persistent) {
      TRY(reserve_sync(ctx, stream));
      TRY(reserve_indices(ctx, 2 * n_slots, stream));
      int32_t* st = ctx->h_stage;
      // sequences by non-increasing length (ties by id), dealt round-robin to the blocks: every block gets the
      // same mix of lengths and its live slots are a prefix at every step
      std::vector<int32_t> first(T + 2, 0);  // first[l]: count, then rank of the first sequence of length l
      for (int32_t q = 0; q < n_seq; ++q)
        if (len[q] > 0) ++first[len[q]];
      for (int32_t l = T, run = 0; l >= 1; --l) {
        const int32_t cnt = first[l];
        first[l] = run;
        run += cnt;
      }
      std::fill(st, st + 2 * n_slots, 0);
      int32_t row0 = 0;
      for (int32_t q = 0; q < n_seq; ++q) {
        if (len[q] > 0) {
          const int32_t r = first[len[q]]++;
          const size_t slot = (size_t)(r % blocks_per_dir) * kRnnSlots + r / blocks_per_dir;
          st[slot] = row0;
          st[n_slots + slot] = len[q];
        }
        row0 += len[q];
      }
      TRY(upload_indices(ctx, 2 * n_slots, stream));
      TRY(clean_counters(ctx, stream));
    } else {
      // per direction, by position in the direction's step lists: row written | row of the previous
      // step of that direction (step 0 gathers row 0 of the initial-state vector)
      TRY(reserve_indices(ctx, 4 * (size_t)R, stream));
      int32_t* st = ctx->h_stage;
      for (int32_t k = 0; k < T; ++k) {
        const int32_t f0 = s.fwd_off[k], nf = s.fwd_off[k + 1] - f0;
        const int32_t* codes = s.level_codes.data() + s.level_off[k];
        for (int32_t p = 0; p < nf; ++p) {
          const int32_t rf = codes[p], rb = codes[nf + p] - R;
          st[f0 + p] = rf;
          st[(size_t)R + f0 + p] = k == 0 ? 0 : rf - 1;
          st[2 * (size_t)R + f0 + p] = rb;
          st[3 * (size_t)R + f0 + p] = k == 0 ? 0 : rb + 1;
        }
      }
      TRY(upload_indices(ctx, 4 * (size_t)R, stream));
    }
    TRY(reserve_scratch(ctx, 2 * (size_t)R * (size_t)H, stream));

    // The two recurrences share nothing but x and never wait for each other: step k of both
    // directions goes out as ONE launch (workgroups of the forward batch, then of the backward
    // batch), and so do the two hoisted input transforms.
    const acrobat_rnn_dir* par[2] = {fwd, bwd};
    float* hdir[2] = {d_hf, d_hb};
    float* xp[2] = {ctx->d_scratch, ctx->d_scratch + (size_t)R * H};

    LaunchTimer timer{ctx, stream};
    {  // hoisted input transforms: one dense batch per direction
      CellLevelArgs a[2] = {};
      for (int dir = 0; dir < 2; ++dir) {
        a[dir].n = R; a[dir].H = H; a[dir].nseg = 1; a[dir].kseg = D;
        a[dir].src0 = d_x; a[dir].ld0 = D;
        a[dir].W = par[dir]->Wx; a[dir].ldw = D; a[dir].bias = par[dir]->b;
        a[dir].zout = xp[dir];
      }
      TRY(timer.begin(ACROBAT_K_RNN_INPUT, 0, 2 * R));
      HIP_TRY(ctx, launch_cell_level_pair(EPI_STORE_Z1, a[0], a[1], stream, ctx->splitk, timer.tile(), timer.ksplit(),
                                          timer.ev));
      TRY(timer.end());
    }
    if (persistent) {
      RnnPersistentArgs pa{};
      pa.n_blocks = 2 * blocks_per_dir; pa.H = H;
      pa.slot_row0 = ctx->d_idx; pa.slot_len = ctx->d_idx + n_slots;
      for (int dir = 0; dir < 2; ++dir) {
        pa.Wh[dir] = par[dir]->Wh; pa.xp[dir] = xp[dir]; pa.h_init[dir] = par[dir]->h_init; pa.h[dir] = hdir[dir];
      }
      pa.h_bytes = (uint32_t)((size_t)R * H * sizeof(float));
      pa.counters = ctx->d_sync; pa.status = ctx->h_status_dev; pa.max_polls = ctx->max_polls;
      TRY(timer.begin(ACROBAT_K_RNN_PERSISTENT, 0, 2 * R));
      if (timer.tile()) *timer.tile() = 16;
      HIP_TRY(ctx, order_waiting_launch(ctx->device, stream));
      HIP_TRY(ctx, launch_rnn_persistent(pa, stream, timer.ev));
      TRY(timer.end());
    }
    for (int32_t k = 0; k < (persistent ? 0 : T); ++k) {
      const int32_t off = s.fwd_off[k], n = s.fwd_off[k + 1] - off;
      CellLevelArgs a[2] = {};
      for (int dir = 0; dir < 2; ++dir) {
        a[dir].n = n; a[dir].H = H; a[dir].nseg = 1; a[dir].kseg = H;
        a[dir].out_rows = ctx->d_idx + 2 * (size_t)dir * R + off;
        a[dir].idx0 = ctx->d_idx + (2 * (size_t)dir + 1) * R + off;
        a[dir].src0 = k == 0 ? par[dir]->h_init : hdir[dir];
        a[dir].ld0 = H;
        a[dir].W = par[dir]->Wh; a[dir].ldw = H;
        a[dir].zadd = xp[dir];
        a[dir].h = hdir[dir];
      }
      TRY(timer.begin(ACROBAT_K_RNN_STEP, k, 2 * n));
      HIP_TRY(ctx, launch_cell_level_pair(EPI_RNN_STEP, a[0], a[1], stream, ctx->splitk, timer.tile(), timer.ksplit(),
                                          timer.ev));
      TRY(timer.end());
    }
    {  // phase 1: every token's output operator in one batch; [hf_t ; hb_t] is read in place
      CellLevelArgs a{};
      a.n = R; a.H = (n_out + 31) / 32 * 32; a.n_cols = n_out;
      a.nseg = 2; a.kseg = H;
      a.src0 = d_hf; a.ld0 = H;
      a.src1 = d_hb; a.ld1 = H;
      a.W = d_C; a.ldw = 2 * H; a.bias = d_cb;
      a.y = d_y; a.ldo = n_out;
      TRY(timer.begin(ACROBAT_K_RNN_OUTPUT, T, R));
      HIP_TRY(ctx, launch_cell_level(EPI_RELU_OUT, a, stream, ctx->splitk, timer.tile(), timer.ksplit(), timer.ev));
      TRY(timer.end());
    }
    return timer.finish();
  } catch (const std::bad_alloc&) {
    return fail(ctx, ACROBAT_ENOMEM, "host allocation failed");
  } catch (...) {
    return fail(ctx, ACROBAT_EINVAL, "unexpected exception");
  }
}

int acrobat_dfg_create(acrobat_ctx* ctx, acrobat_dfg** out) {
  if (!out) return ACROBAT_EINVAL;
  *out = new (std::nothrow) acrobat_dfg();
  if (!*out) return ACROBAT_ENOMEM;
  (*out)->ctx = ctx;
  return ACROBAT_OK;
}

void acrobat_dfg_destroy(acrobat_dfg* g) { delete g; }

const char* acrobat_dfg_last_error(const acrobat_dfg* g) { return g ? g->err.c_str() : "null graph"; }

int acrobat_dfg_register_op(acrobat_dfg* g, const acrobat_op_desc* desc, int32_t* op_id) {
  if (!g || !desc || !op_id) return ACROBAT_EINVAL;
  try {
    g->err.clear();
    return g->graph.register_op(*desc, op_id, g->err);
  } catch (...) {
    g->err = "host allocation failed";
    return ACROBAT_ENOMEM;
  }
}

int acrobat_dfg_clear(acrobat_dfg* g) {
  if (!g) return ACROBAT_EINVAL;
  g->graph.clear();
  return ACROBAT_OK;
}

int acrobat_dfg_invoke(acrobat_dfg* g, int32_t op, int32_t phase, int32_t depth, int32_t out_row,
                       int32_t arg0, int32_t arg1, int32_t prod0, int32_t prod1, int32_t* node) {
  if (!g) return ACROBAT_EINVAL;
  try {
    return g->graph.invoke(op, phase, depth, out_row, arg0, arg1, prod0, prod1, node, g->err);
  } catch (...) {
    g->err = "host allocation failed";
    return ACROBAT_ENOMEM;
  }
}

int acrobat_dfg_build_treelstm(acrobat_dfg* g, const acrobat_trees* trees, int32_t vocab,
                               int32_t op_leaf, int32_t op_internal) {
  if (!g || !trees) return ACROBAT_EINVAL;
  try {
    g->err.clear();
    return dfg_build_treelstm(g->graph, *trees, vocab, op_leaf, op_internal, g->err);
  } catch (...) {
    g->err = "host allocation failed";
    return ACROBAT_ENOMEM;
  }
}

int acrobat_dfg_schedule(acrobat_dfg* g, int32_t* n_buckets, const int32_t** bucket_off,
                         const int32_t** order, const int32_t** bucket_op) {
  if (!g || !n_buckets || !bucket_off || !order || !bucket_op) return ACROBAT_EINVAL;
  try {
    g->graph.bucket(g->buckets);
  } catch (...) {
    g->err = "host allocation failed";
    return ACROBAT_ENOMEM;
  }
  *n_buckets = (int32_t)g->buckets.op.size();
  *bucket_off = g->buckets.off.data();
  *order = g->buckets.order.data();
  *bucket_op = g->buckets.op.data();
  return ACROBAT_OK;
}

int acrobat_dfg_ghost(acrobat_dfg* g, int32_t phase, int32_t depth, int32_t prod, int32_t* node) {
  if (!g) return ACROBAT_EINVAL;
  try {
    return g->graph.ghost(phase, depth, prod, node, g->err);
  } catch (...) {
    g->err = "host allocation failed";
    return ACROBAT_ENOMEM;
  }
}

int acrobat_dfg_run(acrobat_dfg* g, void* hip_stream) {
  if (!g) return ACROBAT_EINVAL;
  acrobat_ctx* ctx = g->ctx;
  if (!ctx) {
    g->err = "graph was created without a context";
    return ACROBAT_EINVAL;
  }
  try {
    TRY(begin_call(ctx));
    return run_graph(g, 0, static_cast<hipStream_t>(hip_stream));
  } catch (const std::bad_alloc&) {
    return fail(ctx, ACROBAT_ENOMEM, "host allocation failed");
  } catch (...) {
    return fail(ctx, ACROBAT_EINVAL, "unexpected exception");
  }
}

namespace {

const float kNoTensor[1] = {0.0f};  // stands in for tensors that a schedule-only run never touches

// registers the six operators of the tree-generation program
int drnn_register_ops(Dfg& graph, const acrobat_drnn_params& p, int32_t n_inst, int32_t max_nodes, const float* d_x0,
                      const float* d_zero, float* d_a, float* d_f, float* d_g, float* d_y, DrnnOps& ops, std::string& err) {
  const int32_t rows = max_nodes > 0 ? max_nodes : 1;
  acrobat_op_desc cell{};
  cell.epilogue = ACROBAT_EPI_RNN_STEP;
  cell.H = p.H; cell.nseg = 2; cell.kseg = p.H;
  cell.ld0 = p.H; cell.ld1 = p.H; cell.ldw = 2 * p.H;
  cell.out_rows = rows;
  auto reg = [&](const float* src0, int32_t rows0, const float* src1, int32_t rows1, const float* W, const float* b,
                 float* h, int32_t* id) {
    acrobat_op_desc d = cell;
    d.src0 = src0; d.src0_rows = rows0; d.src1 = src1; d.src1_rows = rows1; d.W = W; d.bias = b; d.h = h;
    return graph.register_op(d, id, err);
  };
  TRY(reg(d_x0, n_inst > 0 ? n_inst : 1, p.emb, p.n_labels, p.Wa, p.ba, d_a, &ops.a_root));
  TRY(reg(d_a, rows, p.emb, p.n_labels, p.Wa, p.ba, d_a, &ops.a));
  TRY(reg(d_zero, 1, p.emb, p.n_labels, p.Wf, p.bf, d_f, &ops.f_first));
  TRY(reg(d_f, rows, p.emb, p.n_labels, p.Wf, p.bf, d_f, &ops.f));
  TRY(reg(d_a, rows, d_f, rows, p.Wp, p.bp, d_g, &ops.p));
  acrobat_op_desc o{};
  o.epilogue = ACROBAT_EPI_STORE_Z1;
  o.H = p.n_out; o.nseg = 1; o.kseg = p.H;
  o.src0 = d_g; o.ld0 = p.H; o.src0_rows = rows;
  o.W = p.Wo; o.ldw = p.H; o.bias = p.bo; o.zout = d_y; o.out_rows = rows;
  return graph.register_op(o, &ops.o, err);
}

void drnn_copy_out(const DrnnTrees& t, const DrnnStats& st, acrobat_drnn_trees* out, acrobat_drnn_stats* stats) {
  const size_t n = t.inst.size();
  if (out) {
    auto cp = [n](int32_t* dst, const std::vector<int32_t>& src) {
      if (dst && n) std::memcpy(dst, src.data(), n * sizeof(int32_t));
    };
    cp(out->inst, t.inst); cp(out->parent, t.parent); cp(out->prev, t.prev); cp(out->sib_index, t.sib_index);
    cp(out->depth, t.depth); cp(out->label, t.label); cp(out->round, t.round);
  }
  if (stats) *stats = {(int32_t)n, st.n_rounds, st.n_buckets, st.n_fibers, st.n_ghosts};
}

}  // namespace

int acrobat_drnn_schedule(int32_t n_inst, int32_t n_labels, const acrobat_drnn_decisions* decisions, int32_t mode,
                          int32_t use_ghosts, int32_t max_nodes, acrobat_drnn_trees* trees, acrobat_drnn_stats* stats) {
  if (!decisions || n_inst < 0 || max_nodes < 0 || n_labels < 1) return ACROBAT_EINVAL;
  try {
    Dfg graph[kMaxTdcGroups];
    Dfg* graphs[kMaxTdcGroups] = {&graph[0], &graph[1]};
    DfgBuckets buckets;
    std::string err;
    acrobat_drnn_params p{};
    p.H = 32; p.n_labels = n_labels; p.n_out = 32;
    p.emb = p.Wa = p.Wf = p.Wp = p.Wo = kNoTensor;
    float* none = const_cast<float*>(kNoTensor);
    DrnnOps ops;
    for (Dfg& g : graph) TRY(drnn_register_ops(g, p, n_inst, max_nodes, kNoTensor, kNoTensor, none, none, none, none, ops, err));
    DrnnTrees t;
    DrnnStats st;
    const DrnnEvaluate evaluate = [&](int32_t group, size_t first, int32_t* n_buckets) {
      graph[group].bucket(buckets, first);
      *n_buckets = (int32_t)buckets.op.size();
      return ACROBAT_OK;
    };
    const DrnnWait wait = [](int32_t) { return ACROBAT_OK; };
    const DrnnScores scores = [](int32_t) { return (const float*)nullptr; };
    if (decisions->from_scores) return ACROBAT_EINVAL;  // nothing is computed here: there are no scores to decide from
    const int rc = drnn_generate(graphs, drnn_default_groups(n_inst, mode), ops, n_inst, n_labels, 32, *decisions, mode, use_ghosts != 0, max_nodes,
                                 evaluate, wait, scores, t, st, err);
    drnn_copy_out(t, st, trees, stats);
    return rc;
  } catch (...) {
    return ACROBAT_ENOMEM;
  }
}

int acrobat_drnn_forward(acrobat_ctx* ctx, int32_t n_inst, const float* d_x0, const acrobat_drnn_params* params,
                         const acrobat_drnn_decisions* decisions, int32_t mode, int32_t use_ghosts, int32_t max_nodes,
                         acrobat_drnn_trees* trees, float* d_a, float* d_f, float* d_g, float* d_y,
                         acrobat_drnn_stats* stats, void* hip_stream) {
  if (!ctx) return ACROBAT_EINVAL;
  try {
    TRY(begin_call(ctx));
    if (stats) *stats = acrobat_drnn_stats{};
    if (!params || !decisions || n_inst < 0 || max_nodes < 0) return fail(ctx, ACROBAT_EINVAL, "null argument or negative size");
    const acrobat_drnn_params& p = *params;
    if (p.H <= 0 || p.H % 32 || p.n_out <= 0 || p.n_out % 32 || p.n_labels < 1)
      return fail(ctx, ACROBAT_EINVAL, "H and n_out must be positive multiples of 32, n_labels >= 1");
    if (!p.emb || !p.Wa || !p.Wf || !p.Wp || !p.Wo) return fail(ctx, ACROBAT_EINVAL, "null parameter pointer");
    if (n_inst == 0) return ACROBAT_OK;
    if (!d_x0 || !d_a || !d_f || !d_g || !d_y) return fail(ctx, ACROBAT_EINVAL, "null tensor pointer");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (stream_is_capturing(stream)) return fail(ctx, ACROBAT_EINVAL, "a call that waits for tensor values cannot be captured");
    if ((size_t)p.H > ctx->zero_row_cap) {
      if (ctx->d_zero_row) HIP_TRY(ctx, hipFree(ctx->d_zero_row));
      ctx->d_zero_row = nullptr;
      ctx->zero_row_cap = 0;
      HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->d_zero_row), (size_t)p.H * sizeof(float)));
      ctx->zero_row_cap = (size_t)p.H;
      HIP_TRY(ctx, hipMemset(ctx->d_zero_row, 0, (size_t)p.H * sizeof(float)));
    }
    const size_t need = (size_t)(max_nodes > 0 ? max_nodes : 1) * (size_t)p.n_out;
    if (need > ctx->scores_cap) {
      if (ctx->h_scores) HIP_TRY(ctx, hipHostFree(ctx->h_scores));
      ctx->h_scores = nullptr;
      ctx->scores_cap = 0;
      HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->h_scores), need * sizeof(float), hipHostMallocDefault));
      ctx->scores_cap = need;
    }
    // The score layer writes straight into pinned host memory: the program waits for these values
    // at every evaluation, and a store over the bus is cheaper than a copy command in the chain of
    // dependent launches.  d_y receives them all in one copy at the end.
    float* scores_dev = nullptr;  // device-side address of the pinned buffer
    HIP_TRY(ctx, hipHostGetDevicePointer(reinterpret_cast<void**>(&scores_dev), ctx->h_scores, 0));
    // Two groups of instances, each with a graph and a stream of its own (the
    // second stream is the library's, default priority): the host runs one group's program while the
    // other group's kernels execute.  With per-launch timing on there is one group: its records are
    // read after every evaluation.
    const int32_t n_groups = ctx->profiling ? 1 : drnn_default_groups(n_inst, mode);
    if (!ctx->tdc_stream) HIP_TRY(ctx, hipStreamCreateWithFlags(&ctx->tdc_stream, hipStreamNonBlocking));
    if (!ctx->tdc_order) HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->tdc_order, hipEventDisableTiming));
    hipStream_t streams[kMaxTdcGroups] = {stream, ctx->tdc_stream};
    if (n_groups > 1) {  // what the caller has enqueued so far comes first on the second stream too
      HIP_TRY(ctx, hipEventRecord(ctx->tdc_order, stream));
      HIP_TRY(ctx, hipStreamWaitEvent(ctx->tdc_stream, ctx->tdc_order, 0));
    }
    acrobat_dfg g[kMaxTdcGroups];
    Dfg* graphs[kMaxTdcGroups] = {&g[0].graph, &g[1].graph};
    DrnnOps ops;
    for (acrobat_dfg& x : g) {
      x.ctx = ctx;
      const int rc = drnn_register_ops(x.graph, p, n_inst, max_nodes, d_x0, ctx->d_zero_row, d_a, d_f, d_g, scores_dev, ops, x.err);
      if (rc != ACROBAT_OK) return fail(ctx, rc, x.err);
    }
    TRY(reserve_splitk(ctx, stream));
    // The groups' launches overlap on their streams, and a k-split level parks its partial tiles in the
    // workspace between its two launches: every group gets a region of its own.
    SplitKWorkspace group_ws[kMaxTdcGroups];
    for (int32_t q = 0; q < n_groups; ++q) {
      group_ws[q] = ctx->splitk;
      group_ws[q].partial_floats = ctx->splitk.partial_floats / (size_t)n_groups;
      group_ws[q].partial = ctx->splitk.partial + (size_t)q * group_ws[q].partial_floats;
      group_ws[q].n_counters = ctx->splitk.n_counters / n_groups;
      group_ws[q].counters = ctx->splitk.counters + (size_t)q * group_ws[q].n_counters;
    }
    // Index lists: every group stages its lists in a region of its own of the pinned buffer and its
    // kernels read them there.  A region is rewritten only after the group's previous evaluation has
    // been waited for; it grows (both streams idle first) when an evaluation needs more.
    size_t region = 4096 + 16 * (size_t)n_inst;  // int32 per group
    TRY(reserve_indices(ctx, (size_t)n_groups * region, stream));
    const size_t n_out = (size_t)p.n_out;
    const DrnnEvaluate evaluate = [&](int32_t k, size_t first, int32_t* n_buckets) {
      g[k].graph.bucket(g[k].buckets, first);
      *n_buckets = (int32_t)g[k].buckets.op.size();
      const size_t need = 3 * g[k].buckets.order.size();
      if (need > region) {
        for (int32_t q = 0; q < n_groups; ++q) HIP_TRY(ctx, hipStreamSynchronize(streams[q]));
        region = 2 * need;
        TRY(reserve_indices(ctx, (size_t)n_groups * region, stream));
      }
      TRY(launch_buckets(&g[k], streams[k], ctx->h_stage + (size_t)k * region, ctx->h_stage_dev + (size_t)k * region,
                         group_ws[k]));
      return ACROBAT_OK;
    };
    // (each group has a stream to itself; waiting for the stream measured faster than waiting for an event on it)
    const DrnnWait wait = [&](int32_t k) {
      HIP_TRY(ctx, hipStreamSynchronize(streams[k]));
      return ACROBAT_OK;
    };
    const DrnnScores scores = [&](int32_t node) { return (const float*)(ctx->h_scores + (size_t)node * n_out); };
    DrnnTrees t;
    DrnnStats st;
    std::string err;
    const int rc = drnn_generate(graphs, n_groups, ops, n_inst, p.n_labels, p.n_out, *decisions, mode, use_ghosts != 0, max_nodes,
                                 evaluate, wait, scores, t, st, err);
    drnn_copy_out(t, st, trees, stats);
    for (int32_t q = 0; q < n_groups; ++q) HIP_TRY(ctx, hipStreamSynchronize(streams[q]));
    if (!t.inst.empty()) {
      HIP_TRY(ctx, hipMemcpyAsync(d_y, ctx->h_scores, t.inst.size() * n_out * sizeof(float), hipMemcpyHostToDevice, stream));
      HIP_TRY(ctx, hipStreamSynchronize(stream));
    }
    if (rc != ACROBAT_OK) return ctx->err.empty() ? fail(ctx, rc, err) : rc;
    return ACROBAT_OK;
  } catch (const std::bad_alloc&) {
    return fail(ctx, ACROBAT_ENOMEM, "host allocation failed");
  } catch (...) {
    return fail(ctx, ACROBAT_EINVAL, "unexpected exception");
  }
}

int acrobat_last_schedule(const acrobat_ctx* ctx, int32_t* n_levels, const int32_t** level_off,
                          const int32_t** level_nodes) {
  if (!ctx || !n_levels || !level_off || !level_nodes) return ACROBAT_EINVAL;
  *n_levels = ctx->n_levels;
  *level_off = ctx->last_off->data();
  *level_nodes = ctx->last_nodes->data();
  return ACROBAT_OK;
}

int acrobat_set_profiling(acrobat_ctx* ctx, int32_t enabled) {
  if (!ctx) return ACROBAT_EINVAL;
  ctx->profiling = enabled != 0;
  return ACROBAT_OK;
}

int acrobat_set_persistent(acrobat_ctx* ctx, int32_t enabled, int32_t max_polls) {
  if (!ctx) return ACROBAT_EINVAL;
  ctx->persistent = enabled != 0;
  ctx->max_polls = max_polls < 0 ? (1 << 18) : max_polls;
  return ACROBAT_OK;
}

int acrobat_device_status(acrobat_ctx* ctx) {
  if (!ctx) return ACROBAT_EINVAL;
  if (!ctx->h_status || *ctx->h_status == 0) return ACROBAT_OK;
  *ctx->h_status = 0;
  ctx->sync_dirty = true;  // a launch that gave up leaves its counters as they were
  return fail(ctx, ACROBAT_ETIMEOUT, "a workgroup of a persistent launch gave up waiting; the launch's outputs are incomplete");
}

int acrobat_sync_probe(acrobat_ctx* ctx, int32_t groups, int32_t group_size, int32_t rounds, int32_t same_xcd,
                       int32_t style, int32_t write_through, int32_t store_floats, int32_t load_floats,
                       double* us_per_round, double* phase_us, void* hip_stream) {
  try {
    TRY(begin_call(ctx));
    if (!us_per_round || !phase_us) return fail(ctx, ACROBAT_EINVAL, "null output pointer");
    if (groups < 1 || groups > kPersistMaxBlocks || group_size < 1 || groups * group_size > 256 || rounds < 1 || rounds > 100000)
      return fail(ctx, ACROBAT_EINVAL, "groups in 1..8, at most 256 workgroups, rounds in 1..100000");
    if (style < 0 || style > 3 || (style == 2 && group_size > kPersistMaxColBlocks))
      return fail(ctx, ACROBAT_EINVAL, "style in 0..3; flag lines (style 2) hold at most 32 members");
    if (store_floats < 0 || store_floats > 16384 || store_floats % 256 || load_floats < 0 || load_floats % 1024 ||
        load_floats > group_size * store_floats)
      return fail(ctx, ACROBAT_EINVAL, "payload sizes: store multiple of 256 up to 16384, load multiple of 1024 within the group's stores");
    if (style == 3 && (store_floats & (store_floats - 1)))
      return fail(ctx, ACROBAT_EINVAL, "style 3 checks what it reads: store_floats must be a power of two");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (stream_is_capturing(stream)) return fail(ctx, ACROBAT_EINVAL, "the probe synchronises: it cannot be captured");
    int cus = 0;
    HIP_TRY(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device));
    if (groups * group_size > cus) return fail(ctx, ACROBAT_EINVAL, "more workgroups than compute units: they would not all be resident");
    TRY(reserve_sync(ctx, stream));
    const int n_wg = groups * group_size;
    // two generations of payload, used in turn; style 3: one per round
    const size_t payload_floats = (style == 3 ? (size_t)rounds : 2) * (size_t)n_wg * (size_t)std::max(store_floats, 1);
    if (payload_floats * sizeof(float) > ((size_t)1 << 30))
      return fail(ctx, ACROBAT_EINVAL, "style 3 keeps every round's payload: rounds x workgroups x store_floats x 4 bytes must not exceed 1 GiB");
    float* payload = nullptr;
    unsigned long long* ticks = nullptr;
    unsigned* stale = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = ACROBAT_OK;
    auto cleanup = [&]() {
      if (payload) (void)hipFree(payload);
      if (ticks) (void)hipFree(ticks);
      if (stale) (void)hipFree(stale);
      if (e0) (void)hipEventDestroy(e0);
      if (e1) (void)hipEventDestroy(e1);
    };
#define PROBE_TRY(expr)                                     \
  do {                                                      \
    hipError_t e_ = (expr);                                 \
    if (e_ != hipSuccess) { rc = fail_hip(ctx, e_, #expr); cleanup(); return rc; } \
  } while (0)
    PROBE_TRY(hipMalloc(reinterpret_cast<void**>(&payload), payload_floats * sizeof(float)));
    PROBE_TRY(hipMalloc(reinterpret_cast<void**>(&ticks), (size_t)n_wg * 5 * sizeof(unsigned long long)));
    PROBE_TRY(hipMalloc(reinterpret_cast<void**>(&stale), sizeof(unsigned)));
    PROBE_TRY(hipMemsetAsync(stale, 0, sizeof(unsigned), stream));
    PROBE_TRY(hipEventCreate(&e0));
    PROBE_TRY(hipEventCreate(&e1));
    SyncProbeArgs a{};
    a.groups = groups; a.group_size = group_size; a.rounds = rounds; a.same_xcd = same_xcd != 0; a.style = style;
    a.write_through = write_through != 0;
    a.store_floats = store_floats; a.load_floats = load_floats;
    a.payload = payload; a.flags = ctx->d_sync; a.counters = ctx->d_sync + kPersistFlagWords;
    a.status = ctx->h_status_dev; a.max_polls = ctx->max_polls;
    a.ticks = ticks;
    a.stale = stale;
    LaunchEvents ev;
    ev.start = e0; ev.stop = e1;
    ctx->sync_dirty = true;  // the probe's counters end wherever its rounds took them
    PROBE_TRY(launch_fill_u32(ctx->d_sync, 0u, kSyncWords, stream));
    PROBE_TRY(launch_sync_probe(a, stream, ev));
    PROBE_TRY(hipStreamSynchronize(stream));
    float ms = 0.0f;
    PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
    std::vector<unsigned long long> host((size_t)n_wg * 5);
    PROBE_TRY(hipMemcpy(host.data(), ticks, host.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
    unsigned n_stale = 0;
    PROBE_TRY(hipMemcpy(&n_stale, stale, sizeof(unsigned), hipMemcpyDeviceToHost));
#undef PROBE_TRY
    cleanup();
    *us_per_round = (double)ms * 1e3 / rounds;
    for (int i = 0; i < 5; ++i) {  // mean over the workgroups; the clock runs at 100 MHz
      double sum = 0.0;
      for (int w = 0; w < n_wg; ++w) sum += (double)host[(size_t)w * 5 + i];
      phase_us[i] = sum / n_wg / rounds * 0.01;
    }
    phase_us[5] = (double)n_stale;
    return acrobat_device_status(ctx);
  } catch (const std::bad_alloc&) {
    return fail(ctx, ACROBAT_ENOMEM, "host allocation failed");
  } catch (...) {
    return fail(ctx, ACROBAT_EINVAL, "unexpected exception");
  }
}

int acrobat_set_tuning(acrobat_ctx* ctx, int32_t force_tile, int32_t force_ksplit, int32_t mvrnn_variant) {
  if (!ctx) return ACROBAT_EINVAL;
  if (force_tile != 0 && force_tile != 6 && force_tile != 16 && force_tile != 32 && force_tile != 64 && force_tile != 33 &&
      force_tile != 65)
    return fail(ctx, ACROBAT_EINVAL, "force_tile must be 0, 6, 16, 32, 64, 33 or 65");
  if (force_ksplit < 0 || force_ksplit > 32 || (force_ksplit & (force_ksplit - 1)))
    return fail(ctx, ACROBAT_EINVAL, "force_ksplit must be 0 or a power of two up to 32");
  if (mvrnn_variant != 0 && mvrnn_variant != 1) return fail(ctx, ACROBAT_EINVAL, "mvrnn_variant must be 0 or 1");
  ctx->splitk.force_bm = force_tile;
  ctx->splitk.force_ksplit = force_ksplit;
  ctx->mvrnn_variant = mvrnn_variant;
  return ACROBAT_OK;
}

int acrobat_set_gather_fusion(acrobat_ctx* ctx, int32_t enabled) {
  if (!ctx) return ACROBAT_EINVAL;
  ctx->gather_fusion = enabled != 0;
  return ACROBAT_OK;
}

int acrobat_last_profile(const acrobat_ctx* ctx, int32_t* n_records, const acrobat_launch_record** records) {
  if (!ctx || !n_records || !records) return ACROBAT_EINVAL;
  *n_records = (int32_t)ctx->records.size();
  *records = ctx->records.data();
  return ACROBAT_OK;
}

}  // extern "C"
