// C ABI of libheddle: context, argument validation, plan upload, kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "heddle_debug.h"
#include "heddle_internal.h"
#include "kernels.h"

using namespace heddle;

namespace {

constexpr int kStagingSlots = 8;
constexpr int kUploadsPerGuard = 4;    // an event is recorded after every 4th plan upload only: a record
                                       // costs about 3 us of stream time
constexpr int kGuards = kStagingSlots / kUploadsPerGuard;
constexpr int kTimedKernels = 8;       // split-K decode, combine, append, kv write, pack, unpack, shared prefix,
                                       // narrow append
constexpr int kEventPairs = 2048;      // per timed kernel; older records are overwritten

// Scratch of heddle_attn_decode_static: device memory that is part of the library's code object
// instead of the heap.  Layout: plan image [kStaticPlanWords] | partial sums | partial (max, sum)
// records, each region starting at a multiple of 256 bytes.
constexpr size_t kStaticPlanWords = 16384;                       // 64 KiB
constexpr size_t kStaticPartBytes = size_t{16} << 20;            // 16 MiB for both partial arrays
constexpr size_t kStaticBytes = kStaticPlanWords * sizeof(int32_t) + kStaticPartBytes + 256;
constexpr int kMaxDevices = 64;

struct StagingSlot {
  int32_t* host = nullptr;             // pinned
  void* host_dev = nullptr;            // the same memory as the device addresses it
  size_t cap_words = 0;
  uint64_t used_at = 0;                // number of the upload that last read `host`; 0: none pending
};

// Recorded on the stream after upload number `seq`: once it has completed, the copy kernels of
// that upload and of all earlier ones have read their staging buffers.
struct UploadGuard {
  hipEvent_t done = nullptr;
  uint64_t seq = 0;
  bool pending = false;
};

struct KernelTimer {
  std::vector<hipEvent_t> start, stop;
  int64_t recorded = 0;                // launches recorded since enable
  int64_t seen = 0;                    // launches since enable
};

}  // namespace

// One copy per GPU that loads the library, held until the process ends.  Host code never uses this
// name as an address: static_scratch_of() asks the runtime where the current device keeps it.
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

struct heddle_ctx {
  heddle_config cfg{};
  PlanParams plan{};
  float scale = 0.f;
  bool has_device = false;
  bool enqueued = false;
  std::unique_ptr<BlockManager> blocks;

  StagingSlot staging[kStagingSlots];
  int next_slot = 0;
  UploadGuard guards[kGuards];
  int next_guard = 0;
  uint64_t uploads = 0;
  int32_t* dev_plan = nullptr;
  size_t dev_plan_words = 0;
  float* dev_part_acc = nullptr;
  size_t dev_part_acc_elems = 0;
  float* dev_part_ml = nullptr;
  size_t dev_part_ml_elems = 0;
  unsigned char* static_scratch = nullptr;   // this device's copy of `scratch` (nullptr: lookup failed)
  // The scratch above serves one call after the other in stream order.  A call on another stream
  // than the one before first waits (on the device) for that stream's work of this context.
  hipStream_t last_stream = nullptr;
  hipEvent_t handoff = nullptr;

  int32_t timing_every = 0;             // 0 = off; N = record every N-th launch of each kernel
  KernelTimer timers[kTimedKernels];

  // host scratch reused between calls
  std::vector<AppendTile> tiles;
  SharedPlan shared;                    // the plan of the last decode step (without groups in plain decode)
  int32_t min_share_blk = 4, group_wg_per_cu = 1;
  AppendSplit split;
  int32_t append_wg_per_cu = 2, append_min_steps = 4;
};

namespace {

thread_local char g_detail[256] = "";

int hip_failed(hipError_t e, const char* what, int line) {
  std::snprintf(g_detail, sizeof(g_detail), "%s -> %s (line %d)", what, hipGetErrorString(e), line);
  return HEDDLE_E_HIP;
}

#define HEDDLE_HIP(expr)                                                \
  do {                                                                  \
    const hipError_t heddle_hip_e = (expr);                             \
    if (heddle_hip_e != hipSuccess) return hip_failed(heddle_hip_e, #expr, __LINE__); \
  } while (0)

class DeviceGuard {
 public:
  explicit DeviceGuard(int dev) {
    ok_ = hipGetDevice(&prev_) == hipSuccess;
    if (ok_ && prev_ != dev) ok_ = hipSetDevice(dev) == hipSuccess;
    switched_ = ok_ && prev_ != dev;
  }
  ~DeviceGuard() {
    if (switched_) (void)hipSetDevice(prev_);
  }
  bool ok() const { return ok_; }

 private:
  int prev_ = 0;
  bool ok_ = false, switched_ = false;
};

int grow_device(void** ptr, size_t* have, size_t want, size_t elem_bytes) {
  if (want <= *have) return HEDDLE_OK;
  // grow-only scratch: the old buffer may still be read by enqueued work
  HEDDLE_HIP(hipDeviceSynchronize());
  if (*ptr != nullptr) HEDDLE_HIP(hipFree(*ptr));
  *ptr = nullptr;
  *have = 0;
  const size_t cap = want + want / 4;
  void* p = nullptr;
  if (hipMalloc(&p, cap * elem_bytes) != hipSuccess) return HEDDLE_E_NOMEM;
  *ptr = p;
  *have = cap;
  return HEDDLE_OK;
}

// Takes the next pinned staging slot, waiting for the copy that last read it: for the oldest
// guard recorded at or after that upload (with 8 slots and a guard every 4th upload there is
// one unless calls failed in between; then the device is synchronised).
int acquire_slot(heddle_ctx* ctx, size_t words, StagingSlot** out, bool may_allocate = true) {
  if (!may_allocate && words > ctx->staging[ctx->next_slot].cap_words) return HEDDLE_E_NOMEM;
  StagingSlot& s = ctx->staging[ctx->next_slot];
  ctx->next_slot = (ctx->next_slot + 1) % kStagingSlots;
  if (s.used_at != 0) {
    UploadGuard* cover = nullptr;
    for (UploadGuard& g : ctx->guards)
      if (g.seq >= s.used_at && (cover == nullptr || g.seq < cover->seq)) cover = &g;
    if (cover == nullptr) {
      HEDDLE_HIP(hipDeviceSynchronize());
    } else if (cover->pending) {
      HEDDLE_HIP(hipEventSynchronize(cover->done));
      for (UploadGuard& g : ctx->guards)
        if (g.seq <= cover->seq) g.pending = false;      // stream order: older guards have completed too
    }
    s.used_at = 0;
  }
  if (words > s.cap_words) {
    if (s.host != nullptr) HEDDLE_HIP(hipHostFree(s.host));
    s.host = nullptr;
    s.cap_words = 0;
    const size_t cap = (words + words / 2 + 1024 + 3) & ~static_cast<size_t>(3);   // whole 16-byte pieces
    void* p = nullptr;
    if (hipHostMalloc(&p, cap * sizeof(int32_t), hipHostMallocDefault) != hipSuccess) return HEDDLE_E_NOMEM;
    s.host = static_cast<int32_t*>(p);
    s.cap_words = cap;
    s.host_dev = nullptr;
    HEDDLE_HIP(hipHostGetDevicePointer(&s.host_dev, p, 0));
  }
  *out = &s;
  return HEDDLE_OK;
}

// The image is copied by a kernel that reads the pinned buffer (see plan_copy_kernel), in whole
// 16-byte pieces: both buffers are sized in multiples of four words.
// With `rows` the same launch stores the new K/V row of every trajectory of a decode step.
int upload_to(heddle_ctx* ctx, StagingSlot* s, size_t words, int32_t* dst, hipStream_t stream,
              const KvWriteLaunch* rows = nullptr) {
  const size_t padded = (words + 3) & ~static_cast<size_t>(3);
  HEDDLE_HIP(launch_plan_copy(s->host_dev, dst, padded / 4, rows, stream));
  s->used_at = ++ctx->uploads;
  if (ctx->uploads % kUploadsPerGuard == 0) {
    UploadGuard& g = ctx->guards[ctx->next_guard];
    ctx->next_guard = (ctx->next_guard + 1) % kGuards;
    HEDDLE_HIP(hipEventRecord(g.done, stream));
    g.seq = ctx->uploads;
    g.pending = true;
  }
  return HEDDLE_OK;
}

// Upload into the context's own plan buffer, grown first if the image does not fit.
int upload(heddle_ctx* ctx, StagingSlot* s, size_t words, hipStream_t stream, const KvWriteLaunch* rows = nullptr) {
  const size_t padded = (words + 3) & ~static_cast<size_t>(3);
  const int rc = grow_device(reinterpret_cast<void**>(&ctx->dev_plan), &ctx->dev_plan_words, padded, sizeof(int32_t));
  if (rc != HEDDLE_OK) return rc;
  return upload_to(ctx, s, words, ctx->dev_plan, stream, rows);
}

// Every stream-taking call passes here before it touches the staging ring or the scratch: work of
// this context already enqueued on another stream is ordered in front of what the call enqueues.
int enter_stream(heddle_ctx* ctx, hipStream_t stream) {
  if (ctx->enqueued && stream != ctx->last_stream) {
    HEDDLE_HIP(hipEventRecord(ctx->handoff, ctx->last_stream));
    HEDDLE_HIP(hipStreamWaitEvent(stream, ctx->handoff, 0));
  }
  ctx->last_stream = stream;
  return HEDDLE_OK;
}

// The kernels move K/V, queries and outputs in 16-byte pieces.
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Address of `scratch` on the current device, asked once per device and kept.
std::mutex g_static_mutex;
unsigned char* g_static_ptr[kMaxDevices] = {};
bool g_static_asked[kMaxDevices] = {};

unsigned char* static_scratch_of(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_static_asked[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) {
      (void)hip_failed(e, "hipGetSymbolAddress(scratch)", __LINE__);
      p = nullptr;
    }
    g_static_ptr[device] = static_cast<unsigned char*>(p);
    g_static_asked[device] = true;
  }
  return g_static_ptr[device];
}

struct TimedScope {
  heddle_ctx* ctx;
  int which;
  hipStream_t stream;
  int idx = -1;
  TimedScope(heddle_ctx* c, int w, hipStream_t s) : ctx(c), which(w), stream(s) {
    if (ctx->timing_every > 0) {
      KernelTimer& t = ctx->timers[which];
      if (t.seen++ % ctx->timing_every == 0) {
        idx = static_cast<int>(t.recorded % kEventPairs);
        (void)hipEventRecord(t.start[idx], stream);
      }
    }
  }
  ~TimedScope() {
    if (idx >= 0) {
      KernelTimer& t = ctx->timers[which];
      (void)hipEventRecord(t.stop[idx], stream);
      ++t.recorded;
    }
  }
};

// Frees what the context holds on its device (the device must be current).
void release_device_objects(heddle_ctx* ctx) {
  for (StagingSlot& s : ctx->staging)
    if (s.host) (void)hipHostFree(s.host);
  for (UploadGuard& g : ctx->guards)
    if (g.done) (void)hipEventDestroy(g.done);
  if (ctx->handoff) (void)hipEventDestroy(ctx->handoff);
  if (ctx->dev_plan) (void)hipFree(ctx->dev_plan);
  if (ctx->dev_part_acc) (void)hipFree(ctx->dev_part_acc);
  if (ctx->dev_part_ml) (void)hipFree(ctx->dev_part_ml);
  for (KernelTimer& t : ctx->timers) {
    for (hipEvent_t e : t.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : t.stop) (void)hipEventDestroy(e);
  }
}

bool table_covers(const int32_t* row_off_host, int32_t b, int64_t tokens) {
  const int64_t have = static_cast<int64_t>(row_off_host[b + 1]) - row_off_host[b];
  return have >= (tokens + HEDDLE_BLOCK_TOKENS - 1) / HEDDLE_BLOCK_TOKENS;
}

}  // namespace

extern "C" {

int heddle_ctx_create(const heddle_config* cfg, heddle_ctx** out) {
  if (cfg == nullptr || out == nullptr) return HEDDLE_E_INVAL;
  if (cfg->n_q_heads < 1 || cfg->n_kv_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads != 0) return HEDDLE_E_INVAL;
  if (cfg->block_tokens != HEDDLE_BLOCK_TOKENS || cfg->n_blocks < 1) return HEDDLE_E_INVAL;
  if (cfg->head_dim < 8 || cfg->head_dim % 8 != 0) return HEDDLE_E_INVAL;
  if (cfg->n_cu < 0 || cfg->wg_per_cu < 0 || cfg->min_chunk_blk < 0 || cfg->tile_blk < 0 || cfg->max_split < 0 ||
      cfg->min_share_blk < 0 || cfg->group_wg_per_cu < 0 || cfg->append_wg_per_cu < 0 || cfg->append_min_steps < 0)
    return HEDDLE_E_INVAL;
  if (cfg->device < -1 || (cfg->device >= 0 && cfg->kv_pool == nullptr)) return HEDDLE_E_INVAL;
  if (!(cfg->scale >= 0.f) || !std::isfinite(cfg->scale)) return HEDDLE_E_INVAL;
  // Head shapes the packed-dot decode kernel is not built for (3, 5, 6, 7 ... query heads per kv
  // head) decode on the matrix-core kernel, which cuts keys at multiples of 64: the plan's parts
  // must then start there.
  if (cfg->device >= 0) {
    const int32_t group = cfg->n_q_heads / cfg->n_kv_heads;
    const int32_t tile_blk = cfg->tile_blk ? cfg->tile_blk : 4;
    const bool on_mfma_only = narrow_shape_supported(group, cfg->head_dim) &&
                              tile_blk % (kAppendStepKeys / HEDDLE_BLOCK_TOKENS) == 0;
    if (!decode_shape_supported(group, cfg->head_dim) && !on_mfma_only) return HEDDLE_E_UNSUPPORTED;
  }

  std::unique_ptr<heddle_ctx> ctx(new (std::nothrow) heddle_ctx);
  if (!ctx) return HEDDLE_E_NOMEM;
  ctx->cfg = *cfg;
  ctx->scale = cfg->scale > 0.f ? cfg->scale : 1.0f / std::sqrt(static_cast<float>(cfg->head_dim));
  ctx->blocks.reset(new (std::nothrow) BlockManager(cfg->n_blocks));
  if (!ctx->blocks) return HEDDLE_E_NOMEM;

  int n_cu = cfg->n_cu;
  if (cfg->device >= 0) {
    int count = 0;
    HEDDLE_HIP(hipGetDeviceCount(&count));
    if (cfg->device >= count) return HEDDLE_E_INVAL;
    DeviceGuard guard(cfg->device);
    if (!guard.ok()) return HEDDLE_E_HIP;
    if (n_cu == 0) HEDDLE_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, cfg->device));
    for (UploadGuard& g : ctx->guards) {
      const hipError_t e = hipEventCreateWithFlags(&g.done, hipEventDisableTiming);
      if (e != hipSuccess) {
        g.done = nullptr;
        release_device_objects(ctx.get());
        return hip_failed(e, "hipEventCreateWithFlags", __LINE__);
      }
    }
    {
      const hipError_t e = hipEventCreateWithFlags(&ctx->handoff, hipEventDisableTiming);
      if (e != hipSuccess) {
        ctx->handoff = nullptr;
        release_device_objects(ctx.get());
        return hip_failed(e, "hipEventCreateWithFlags", __LINE__);
      }
    }
    // every staging slot starts large enough for the biggest plan image the static-scratch entry
    // point accepts, which then never meets a slot it would have to enlarge
    for (StagingSlot& sl : ctx->staging) {
      void* p = nullptr;
      hipError_t e = hipHostMalloc(&p, kStaticPlanWords * sizeof(int32_t), hipHostMallocDefault);
      if (e == hipSuccess) {
        sl.host = static_cast<int32_t*>(p);
        sl.cap_words = kStaticPlanWords;
        e = hipHostGetDevicePointer(&sl.host_dev, p, 0);
      }
      if (e != hipSuccess) {
        release_device_objects(ctx.get());
        return hip_failed(e, "hipHostMalloc (staging ring)", __LINE__);
      }
    }
    ctx->static_scratch = static_scratch_of(cfg->device);
    ctx->shared.items.reserve(kStaticPlanWords / 8);
    ctx->shared.nsplit.reserve(kStaticPlanWords / 4);
    ctx->shared.part_off.reserve(kStaticPlanWords / 4 + 1);
    ctx->has_device = true;
  } else if (n_cu == 0) {
    n_cu = 256;
  }
  ctx->plan.n_kv_heads = cfg->n_kv_heads;
  ctx->plan.n_cu = n_cu;
  ctx->plan.wg_per_cu = cfg->wg_per_cu ? cfg->wg_per_cu : 4;
  ctx->plan.min_chunk_blk = cfg->min_chunk_blk ? cfg->min_chunk_blk : 16;
  ctx->plan.tile_blk = cfg->tile_blk ? cfg->tile_blk : 4;
  ctx->plan.max_split = cfg->max_split ? cfg->max_split : 64;
  ctx->min_share_blk = cfg->min_share_blk ? cfg->min_share_blk : 4;
  ctx->group_wg_per_cu = cfg->group_wg_per_cu ? cfg->group_wg_per_cu : 1;
  ctx->append_wg_per_cu = cfg->append_wg_per_cu ? cfg->append_wg_per_cu : 2;
  ctx->append_min_steps = cfg->append_min_steps ? cfg->append_min_steps : 4;
  *out = ctx.release();
  return HEDDLE_OK;
}

int heddle_ctx_destroy(heddle_ctx* ctx) {
  if (ctx == nullptr) return HEDDLE_E_INVAL;
  int rc = HEDDLE_OK;
  if (ctx->has_device) {
    DeviceGuard guard(ctx->cfg.device);
    if (ctx->enqueued && hipDeviceSynchronize() != hipSuccess) rc = HEDDLE_E_HIP;
    release_device_objects(ctx);
  }
  delete ctx;
  return rc;
}

int heddle_ctx_reserve(heddle_ctx* ctx, int32_t max_trajectories, int32_t max_chunk_rows, int32_t with_shared_prefix) {
  if (ctx == nullptr || max_trajectories < 1 || max_chunk_rows < 0) return HEDDLE_E_INVAL;
  if (!ctx->has_device) return HEDDLE_E_UNSUPPORTED;
  DeviceGuard guard(ctx->cfg.device);
  if (!guard.ok()) return HEDDLE_E_HIP;
  // Upper bounds that follow from the plan rules: a trajectory (tile) of n blocks (steps) is cut
  // into at most n/chunk + 1 parts and chunk >= total/target, so a batch has at most
  // target + (number of trajectories or tiles) work items.
  const size_t B = static_cast<size_t>(max_trajectories);
  const size_t n_kv = static_cast<size_t>(ctx->cfg.n_kv_heads);
  const size_t Hq = static_cast<size_t>(ctx->cfg.n_q_heads), D = static_cast<size_t>(ctx->cfg.head_dim);
  const size_t n_cu = static_cast<size_t>(ctx->plan.n_cu);
  const size_t target = std::max<size_t>(1, n_cu * ctx->plan.wg_per_cu / n_kv);
  size_t items = target + B, parts = target + B;
  size_t words = 8 * items + 4 * B + 1;
  if (with_shared_prefix) {
    const size_t target_g = std::max<size_t>(1, n_cu * ctx->group_wg_per_cu / n_kv);
    const size_t prefix_parts = std::min<size_t>(static_cast<size_t>(ctx->plan.max_split), target_g + 1);
    parts += B * prefix_parts;                          // every member owns a slot per part of its group's prefix
    words = 8 * items + 8 * (target_g + B) + 5 * B + 1 + B;
  }
  if (max_chunk_rows > 0) {
    const size_t G = Hq / n_kv;
    const size_t tile_rows = static_cast<size_t>(std::max(1, append_tile_rows(static_cast<int32_t>(G))));
    const size_t target_a = std::max<size_t>(1, n_cu * ctx->append_wg_per_cu / n_kv);
    const size_t tiles = static_cast<size_t>(max_chunk_rows) / tile_rows + B;
    const size_t a_items = target_a + tiles;
    const size_t a_slots = tile_rows * 2 * target_a;    // at most target_a tiles are cut, into at most 2 target_a parts
    const size_t a_split_rows = tile_rows * target_a;
    parts = std::max(parts, a_slots);
    words = std::max(words, 8 * a_items + 3 * B + 2 + 3 * a_split_rows);
  }
  int rc = grow_device(reinterpret_cast<void**>(&ctx->dev_part_acc), &ctx->dev_part_acc_elems, parts * Hq * D,
                       sizeof(float));
  if (rc != HEDDLE_OK) return rc;
  rc = grow_device(reinterpret_cast<void**>(&ctx->dev_part_ml), &ctx->dev_part_ml_elems, parts * Hq * 4, sizeof(float));
  if (rc != HEDDLE_OK) return rc;
  const size_t padded = (words + 3) & ~size_t{3};
  rc = grow_device(reinterpret_cast<void**>(&ctx->dev_plan), &ctx->dev_plan_words, padded, sizeof(int32_t));
  if (rc != HEDDLE_OK) return rc;
  bool synced = false;
  for (StagingSlot& sl : ctx->staging) {
    if (sl.cap_words >= padded) continue;
    if (!synced) {                                      // a pending copy may still read the old buffers
      HEDDLE_HIP(hipDeviceSynchronize());
      synced = true;
    }
    if (sl.host != nullptr) HEDDLE_HIP(hipHostFree(sl.host));
    sl.host = nullptr;
    sl.host_dev = nullptr;
    sl.cap_words = 0;
    sl.used_at = 0;
    void* p = nullptr;
    if (hipHostMalloc(&p, padded * sizeof(int32_t), hipHostMallocDefault) != hipSuccess) return HEDDLE_E_NOMEM;
    sl.host = static_cast<int32_t*>(p);
    sl.cap_words = padded;
    HEDDLE_HIP(hipHostGetDevicePointer(&sl.host_dev, p, 0));
  }
  ctx->shared.items.reserve(items);
  ctx->shared.nsplit.reserve(B);
  ctx->shared.part_off.reserve(B + 1);
  return HEDDLE_OK;
}

int heddle_kv_alloc(heddle_ctx* ctx, int32_t n, int32_t* out_block_ids) {
  if (ctx == nullptr) return HEDDLE_E_INVAL;
  return ctx->blocks->alloc(n, out_block_ids);
}

int heddle_kv_retain(heddle_ctx* ctx, int32_t n, const int32_t* block_ids) {
  if (ctx == nullptr) return HEDDLE_E_INVAL;
  return ctx->blocks->retain(n, block_ids);
}

int heddle_kv_free(heddle_ctx* ctx, int32_t n, const int32_t* block_ids) {
  if (ctx == nullptr) return HEDDLE_E_INVAL;
  return ctx->blocks->release(n, block_ids);
}

int heddle_ctx_set_kv_pool(heddle_ctx* ctx, void* kv_pool) {
  if (ctx == nullptr || kv_pool == nullptr || ctx->cfg.device < 0) return HEDDLE_E_INVAL;
  ctx->cfg.kv_pool = kv_pool;
  return HEDDLE_OK;
}

int heddle_kv_num_free(const heddle_ctx* ctx, int32_t* out) {
  if (ctx == nullptr || out == nullptr) return HEDDLE_E_INVAL;
  *out = ctx->blocks->num_free();
  return HEDDLE_OK;
}

int heddle_plan_decode(const heddle_ctx* ctx, int32_t B, const int32_t* len_host, heddle_plan* plan) {
  if (ctx == nullptr || plan == nullptr || len_host == nullptr || B < 1) return HEDDLE_E_INVAL;
  if (!plan->item_b || !plan->item_s || !plan->item_blk_begin || !plan->item_blk_end || !plan->nsplit ||
      !plan->part_off)
    return HEDDLE_E_INVAL;
  for (int32_t b = 0; b < B; ++b)
    if (len_host[b] < 1 || len_host[b] > HEDDLE_MAX_CONTEXT) return HEDDLE_E_INVAL;
  std::vector<DecodeItem> items;
  std::vector<int32_t> nsplit, part_off;
  int32_t chunk = 0;
  plan_decode(ctx->plan, B, len_host, items, nsplit, part_off, chunk);
  if (static_cast<int64_t>(items.size()) > plan->cap_items) return HEDDLE_E_NOMEM;
  plan->n_items = static_cast<int32_t>(items.size());
  plan->chunk = chunk;
  for (size_t i = 0; i < items.size(); ++i) {
    plan->item_b[i] = items[i].b;
    plan->item_s[i] = items[i].s;
    plan->item_blk_begin[i] = items[i].blk_begin;
    plan->item_blk_end[i] = items[i].blk_end;
  }
  std::memcpy(plan->nsplit, nsplit.data(), sizeof(int32_t) * B);
  std::memcpy(plan->part_off, part_off.data(), sizeof(int32_t) * (static_cast<size_t>(B) + 1));
  return HEDDLE_OK;
}

int heddle_plan_append(const heddle_ctx* ctx, int32_t B, const int32_t* ctx_len_host,
                       const int32_t* cu_chunk_host, int32_t tile_rows, heddle_append_plan* plan) {
  if (ctx == nullptr || plan == nullptr || ctx_len_host == nullptr || cu_chunk_host == nullptr || B < 1)
    return HEDDLE_E_INVAL;
  if (!plan->tile_b || !plan->tile_row0 || !plan->tile_rows_n || !plan->tile_extent) return HEDDLE_E_INVAL;
  if (cu_chunk_host[0] != 0) return HEDDLE_E_INVAL;
  for (int32_t b = 0; b < B; ++b) {
    const int64_t C = static_cast<int64_t>(cu_chunk_host[b + 1]) - cu_chunk_host[b];
    if (C < 1 || ctx_len_host[b] < 0 || ctx_len_host[b] + C > HEDDLE_MAX_CONTEXT) return HEDDLE_E_INVAL;
  }
  if (tile_rows <= 0) tile_rows = append_tile_rows(ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads);
  if (tile_rows < 1) tile_rows = 1;
  std::vector<AppendTile> tiles;
  plan_append(B, ctx_len_host, cu_chunk_host, tile_rows, tiles);
  if (static_cast<int64_t>(tiles.size()) > plan->cap_tiles) return HEDDLE_E_NOMEM;
  plan->n_tiles = static_cast<int32_t>(tiles.size());
  plan->tile_rows = tile_rows;
  for (size_t i = 0; i < tiles.size(); ++i) {
    plan->tile_b[i] = tiles[i].b;
    plan->tile_row0[i] = tiles[i].row0;
    plan->tile_rows_n[i] = tiles[i].rows;
    plan->tile_extent[i] = tiles[i].extent;
  }
  return HEDDLE_OK;
}

namespace {

int check_decode_args(const heddle_ctx* ctx, const heddle_decode_args* args) {
  if (ctx == nullptr || args == nullptr) return HEDDLE_E_INVAL;
  if (!ctx->has_device) return HEDDLE_E_UNSUPPORTED;
  const int32_t B = args->B;
  if (B < 1 || !args->len_host || !args->row_off_host || !args->row_off || !args->block_ids || !args->q ||
      !args->out)
    return HEDDLE_E_INVAL;
  if ((args->k_new == nullptr) != (args->v_new == nullptr)) return HEDDLE_E_INVAL;
  if (misaligned(args->q) || misaligned(args->out) || misaligned(args->k_new) || misaligned(args->v_new) ||
      misaligned(ctx->cfg.kv_pool))
    return HEDDLE_E_INVAL;
  if (args->row_off_host[0] < 0) return HEDDLE_E_INVAL;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t n = args->len_host[b];
    if (n < 1 || n > HEDDLE_MAX_CONTEXT) return HEDDLE_E_INVAL;
    if (args->row_off_host[b + 1] < args->row_off_host[b] || !table_covers(args->row_off_host, b, n))
      return HEDDLE_E_INVAL;
  }
  return HEDDLE_OK;
}

// Which kernel reads the blocks of a decode step (all of them in heddle_attn_decode, the private
// ones in heddle_attn_decode_shared): true = the matrix-core kernel for short-row tiles, fed the plan
// as an append of one token per trajectory; false = the packed-dot split-K kernel.
// With 8 query heads per kv head the packed-dot kernel is bound by its arithmetic and the matrix-core
// kernel is not; head shapes the packed-dot kernel has no lane layout for (3, 5, 6, 7 ... query heads
// per kv head) have no other choice.  The matrix-core kernel cuts keys at multiples of 64, so the
// plan's parts must start at multiples of 4 blocks (tile_blk % 4 == 0); a context whose shape needs
// that kernel is only created with such a tile_blk.
bool decode_on_matrix_cores(const heddle_ctx* ctx) {
  const int32_t G = ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads;
  const bool aligned = ctx->plan.tile_blk % (kAppendStepKeys / HEDDLE_BLOCK_TOKENS) == 0;
  const bool splitk_built = decode_shape_supported(G, ctx->cfg.head_dim);
  return narrow_shape_supported(G, ctx->cfg.head_dim) && aligned && (G == 8 || !splitk_built);
}

// Group formation of the shared-prefix plan with this context's parameters; on shapes the
// matrix-core kernel is not built for nobody is grouped.  Where the private blocks are read by
// the matrix-core kernel, which starts at multiples of 64 keys, shared prefixes end at
// multiples of 4 blocks.
void plan_shared_for(const heddle_ctx* ctx, int32_t B, const int32_t* len, const int32_t* row_off,
                     const int32_t* block_ids, SharedPlan& out) {
  const int32_t G = ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads;
  const int32_t step_blk = kAppendStepKeys / HEDDLE_BLOCK_TOKENS;
  const bool mfma_private = decode_on_matrix_cores(ctx);
  // a shape that needs the matrix-core kernel with a plan off its 64-key grid cannot be created
  const bool can_group = append_shape_supported(G, ctx->cfg.head_dim) &&
                         (mfma_private || decode_shape_supported(G, ctx->cfg.head_dim));
  const int32_t tile_members = can_group ? append_tile_rows(G) : 1;
  plan_decode_shared(ctx->plan, can_group ? ctx->min_share_blk : INT32_MAX, ctx->group_wg_per_cu, tile_members,
                     mfma_private ? step_blk : 1, B, len, row_off, block_ids, out);
}

}  // namespace

int heddle_plan_decode_shared(const heddle_ctx* ctx, int32_t B, const int32_t* len_host,
                              const int32_t* row_off_host, const int32_t* block_ids_host,
                              heddle_shared_plan* plan) {
  if (ctx == nullptr || plan == nullptr || !len_host || !row_off_host || !block_ids_host || B < 1)
    return HEDDLE_E_INVAL;
  if (!plan->item_b || !plan->item_s || !plan->item_blk_begin || !plan->item_blk_end || !plan->gitem_g ||
      !plan->gitem_k || !plan->gitem_blk_begin || !plan->gitem_blk_end || !plan->gitem_m0 || !plan->gitem_mn ||
      !plan->group_leader || !plan->group_prefix || !plan->group_parts || !plan->member_off || !plan->members ||
      !plan->traj_group || !plan->traj_prefix || !plan->nsplit || !plan->part_off)
    return HEDDLE_E_INVAL;
  if (row_off_host[0] < 0) return HEDDLE_E_INVAL;
  for (int32_t b = 0; b < B; ++b) {
    if (len_host[b] < 1 || len_host[b] > HEDDLE_MAX_CONTEXT) return HEDDLE_E_INVAL;
    if (row_off_host[b + 1] < row_off_host[b] || !table_covers(row_off_host, b, len_host[b])) return HEDDLE_E_INVAL;
  }
  SharedPlan sp;
  plan_shared_for(ctx, B, len_host, row_off_host, block_ids_host, sp);
  const size_t n_groups = sp.group_leader.size();
  if (static_cast<int64_t>(sp.items.size()) > plan->cap_items ||
      static_cast<int64_t>(sp.gitems.size()) > plan->cap_gitems || static_cast<int64_t>(n_groups) > plan->cap_groups)
    return HEDDLE_E_NOMEM;
  plan->n_items = static_cast<int32_t>(sp.items.size());
  plan->n_gitems = static_cast<int32_t>(sp.gitems.size());
  plan->n_groups = static_cast<int32_t>(n_groups);
  plan->chunk = sp.chunk;
  plan->chunk_g = sp.chunk_g;
  for (size_t i = 0; i < sp.items.size(); ++i) {
    plan->item_b[i] = sp.items[i].b;
    plan->item_s[i] = sp.items[i].s;
    plan->item_blk_begin[i] = sp.items[i].blk_begin;
    plan->item_blk_end[i] = sp.items[i].blk_end;
  }
  for (size_t i = 0; i < sp.gitems.size(); ++i) {
    plan->gitem_g[i] = sp.gitems[i].g;
    plan->gitem_k[i] = sp.gitems[i].k;
    plan->gitem_blk_begin[i] = sp.gitems[i].blk_begin;
    plan->gitem_blk_end[i] = sp.gitems[i].blk_end;
    plan->gitem_m0[i] = sp.gitems[i].m0;
    plan->gitem_mn[i] = sp.gitems[i].mn;
  }
  auto copy = [](int32_t* dst, const std::vector<int32_t>& v) {
    if (!v.empty()) std::memcpy(dst, v.data(), sizeof(int32_t) * v.size());
  };
  copy(plan->group_leader, sp.group_leader);
  copy(plan->group_prefix, sp.group_prefix);
  copy(plan->group_parts, sp.group_parts);
  copy(plan->member_off, sp.member_off);
  copy(plan->members, sp.members);
  copy(plan->traj_group, sp.traj_group);
  copy(plan->traj_prefix, sp.traj_prefix);
  copy(plan->nsplit, sp.nsplit);
  copy(plan->part_off, sp.part_off);
  return HEDDLE_OK;
}

namespace {

// One decode step: heddle_attn_decode (block_ids_host == nullptr: no group search, the plan of
// heddle_plan_decode), heddle_attn_decode_shared (groups from the host copy of the table) and
// heddle_attn_decode_static (static_scratch: plan image and partials in the library's static device
// array, nothing allocated).  Without groups the plan image and the launches of the shared-prefix
// form reduce to those of the plain one.
int decode_call(heddle_ctx* ctx, const heddle_decode_args* args, const int32_t* block_ids_host, void* hip_stream,
                bool static_scratch) {
  int rc = check_decode_args(ctx, args);
  if (rc != HEDDLE_OK) return rc;
  const int32_t B = args->B;
  if (block_ids_host != nullptr) {
    // the host copy of the table is at hand here: ids of the needed blocks must name pool blocks
    for (int32_t b = 0; b < B; ++b) {
      const int32_t* row = block_ids_host + args->row_off_host[b];
      const int32_t need = (args->len_host[b] + HEDDLE_BLOCK_TOKENS - 1) / HEDDLE_BLOCK_TOKENS;
      for (int32_t i = 0; i < need; ++i)
        if (row[i] < 0 || row[i] >= ctx->cfg.n_blocks) return HEDDLE_E_INVAL;
    }
  }
  const int32_t Hq = ctx->cfg.n_q_heads, D = ctx->cfg.head_dim;
  const bool mfma_private = decode_on_matrix_cores(ctx);
  if (!mfma_private && !decode_shape_supported(Hq / ctx->cfg.n_kv_heads, D)) return HEDDLE_E_UNSUPPORTED;

  DeviceGuard guard(ctx->cfg.device);
  if (!guard.ok()) return HEDDLE_E_HIP;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  SharedPlan& sp = ctx->shared;
  if (block_ids_host != nullptr) {
    plan_shared_for(ctx, B, args->len_host, args->row_off_host, block_ids_host, sp);
  } else {
    sp.gitems.clear();
    sp.members.clear();
    plan_decode(ctx->plan, B, args->len_host, sp.items, sp.nsplit, sp.part_off, sp.chunk);
  }
  const size_t n_items = sp.items.size(), n_gitems = sp.gitems.size(), n_members = sp.members.size();
  const size_t n_parts = static_cast<size_t>(sp.part_off[B]);

  // plan image: item records | group item records | trajectory records | first_pos[B] | cu_rows[B+1] | members
  const size_t nB = static_cast<size_t>(B);
  const size_t words = 8 * n_items + 8 * n_gitems + 2 * nB + nB + nB + 1 + n_members;
  const size_t padded = (words + 3) & ~size_t{3};
  const size_t acc_elems = n_parts * Hq * D, ml_elems = n_parts * Hq * 4;
  int32_t* dev_plan = nullptr;
  float *part_acc = nullptr, *part_ml = nullptr;
  if (static_scratch) {
    if (ctx->static_scratch == nullptr) {
      std::snprintf(g_detail, sizeof(g_detail), "hipGetSymbolAddress(scratch) failed when the context was created");
      return HEDDLE_E_HIP;
    }
    const size_t acc_bytes = (acc_elems * sizeof(float) + 255) & ~size_t{255};
    if (padded > kStaticPlanWords || acc_bytes + ml_elems * sizeof(float) > kStaticPartBytes) {
      std::snprintf(g_detail, sizeof(g_detail),
                    "static scratch too small: plan image %zu words (limit %zu), partials %zu bytes (limit %zu)",
                    words, kStaticPlanWords, acc_bytes + ml_elems * sizeof(float), kStaticPartBytes);
      return HEDDLE_E_NOMEM;
    }
    dev_plan = reinterpret_cast<int32_t*>(ctx->static_scratch);
    part_acc = reinterpret_cast<float*>(ctx->static_scratch + kStaticPlanWords * sizeof(int32_t));
    part_ml = reinterpret_cast<float*>(ctx->static_scratch + kStaticPlanWords * sizeof(int32_t) + acc_bytes);
  } else {
    rc = grow_device(reinterpret_cast<void**>(&ctx->dev_part_acc), &ctx->dev_part_acc_elems, acc_elems, sizeof(float));
    if (rc != HEDDLE_OK) return rc;
    rc = grow_device(reinterpret_cast<void**>(&ctx->dev_part_ml), &ctx->dev_part_ml_elems, ml_elems, sizeof(float));
    if (rc != HEDDLE_OK) return rc;
    rc = grow_device(reinterpret_cast<void**>(&ctx->dev_plan), &ctx->dev_plan_words, padded, sizeof(int32_t));
    if (rc != HEDDLE_OK) return rc;
    dev_plan = ctx->dev_plan;
    part_acc = ctx->dev_part_acc;
    part_ml = ctx->dev_part_ml;
  }
  rc = enter_stream(ctx, stream);
  if (rc != HEDDLE_OK) return rc;
  StagingSlot* slot = nullptr;
  rc = acquire_slot(ctx, words, &slot, !static_scratch);
  if (rc != HEDDLE_OK) return rc;
  int32_t* w = slot->host;
  DecodeItemRec* h_items = reinterpret_cast<DecodeItemRec*>(w);
  GroupItemRec* h_gitems = reinterpret_cast<GroupItemRec*>(w + 8 * n_items);
  DecodeTrajRec* h_trajs = reinterpret_cast<DecodeTrajRec*>(w + 8 * (n_items + n_gitems));
  int32_t* h_first = w + 8 * (n_items + n_gitems) + 2 * nB;
  int32_t* h_cu = h_first + B;
  int32_t* h_members = h_cu + B + 1;
  for (size_t i = 0; i < n_items; ++i) {
    const DecodeItem& it = sp.items[i];
    if (mfma_private) {       // the item as the matrix-core kernel reads it: one new token of trajectory b
      AppendItemRec& r = reinterpret_cast<AppendItemRec*>(w)[i];
      r.b = it.b;
      r.row0 = 0;
      r.rows_n = 1;
      r.key_end = std::min(args->len_host[it.b], it.blk_end * HEDDLE_BLOCK_TOKENS);
      r.step_begin = it.blk_begin / (kAppendStepKeys / HEDDLE_BLOCK_TOKENS);
      r.slot0 = sp.part_off[it.b] + it.s;
      r.nsplit = sp.nsplit[it.b];
      r.pad = 0;
      continue;
    }
    DecodeItemRec& r = h_items[i];
    r.b = it.b;
    r.slot = sp.part_off[it.b] + it.s;
    r.blk_begin = it.blk_begin;
    r.blk_end = it.blk_end;
    r.len = args->len_host[it.b];
    r.table_off = args->row_off_host[it.b];
    r.nsplit = sp.nsplit[it.b];
    r.pad = 0;
  }
  for (size_t i = 0; i < n_gitems; ++i) {
    const GroupItem& it = sp.gitems[i];
    GroupItemRec& r = h_gitems[i];
    r.table_off = args->row_off_host[sp.group_leader[it.g]];
    r.blk_begin = it.blk_begin;
    r.blk_end = it.blk_end;
    r.part = it.k;
    r.member_off = sp.member_off[it.g] + it.m0;
    r.n_members = it.mn;
    r.pad[0] = r.pad[1] = 0;
  }
  for (int32_t b = 0; b < B; ++b) {
    h_trajs[b].part_off = sp.part_off[b];
    h_trajs[b].nsplit = sp.nsplit[b];
    h_first[b] = args->len_host[b] - 1;
    h_cu[b] = b;
  }
  h_cu[B] = B;
  if (n_members > 0) std::memcpy(h_members, sp.members.data(), sizeof(int32_t) * n_members);
  // the step's new K/V rows are stored by the launch that copies the plan image; its row writers
  // read first_pos from the pinned image
  KvWriteLaunch kw{};
  if (args->k_new != nullptr) {
    kw.pool = static_cast<uint16_t*>(ctx->cfg.kv_pool);
    kw.row_off = args->row_off;
    kw.block_ids = args->block_ids;
    kw.first_pos = static_cast<const int32_t*>(slot->host_dev) + (h_first - w);
    kw.k = static_cast<const uint16_t*>(args->k_new);
    kw.v = static_cast<const uint16_t*>(args->v_new);
    kw.B = B;
    kw.n_rows = B;
    kw.n_wblk = B;
    kw.n_kv_heads = ctx->cfg.n_kv_heads;
    kw.head_dim = D;
    kw.one_row_each = 1;
  }
  rc = upload_to(ctx, slot, words, dev_plan, stream, args->k_new != nullptr ? &kw : nullptr);
  if (rc != HEDDLE_OK) return rc;
  const int32_t* d = dev_plan;
  ctx->enqueued = true;

  const float scale_log2 = ctx->scale * 1.4426950408889634f;
  const DecodeTrajRec* d_trajs = reinterpret_cast<const DecodeTrajRec*>(d + 8 * (n_items + n_gitems));
  if (n_gitems > 0) {
    GroupLaunch gl{};
    gl.pool = static_cast<const uint16_t*>(ctx->cfg.kv_pool);
    gl.block_ids = args->block_ids;
    gl.items = reinterpret_cast<const GroupItemRec*>(d + 8 * n_items);
    gl.members = d + (h_members - w);
    gl.trajs = d_trajs;
    gl.q = static_cast<const uint16_t*>(args->q);
    gl.part_acc = part_acc;
    gl.part_ml = part_ml;
    gl.n_items = static_cast<int32_t>(n_gitems);
    gl.n_q_heads = Hq;
    gl.n_kv_heads = ctx->cfg.n_kv_heads;
    gl.head_dim = D;
    gl.scale_log2 = scale_log2;
    TimedScope t(ctx, 6, stream);
    HEDDLE_HIP(launch_group_attn(gl, stream));
  }

  DecodeLaunch dl{};
  dl.pool = static_cast<const uint16_t*>(ctx->cfg.kv_pool);
  dl.block_ids = args->block_ids;
  dl.items = reinterpret_cast<const DecodeItemRec*>(d);
  dl.trajs = d_trajs;
  dl.q = static_cast<const uint16_t*>(args->q);
  dl.part_acc = part_acc;
  dl.part_ml = part_ml;
  dl.out = static_cast<uint16_t*>(args->out);
  dl.lse = args->lse;
  dl.B = B;
  dl.n_items = static_cast<int32_t>(n_items);
  dl.n_q_heads = Hq;
  dl.n_kv_heads = ctx->cfg.n_kv_heads;
  dl.head_dim = D;
  dl.scale_log2 = scale_log2;
  if (mfma_private) {
    AppendLaunch al{};                         // the private blocks seen as an append: L = len - 1, one new row each
    al.pool = dl.pool;
    al.row_off = args->row_off;
    al.block_ids = args->block_ids;
    al.ctx_len = d + (h_first - w);
    al.cu_chunk = d + (h_cu - w);
    al.items = reinterpret_cast<const AppendItemRec*>(d);
    al.q = dl.q;
    al.out = dl.out;
    al.lse = dl.lse;
    al.part_acc = dl.part_acc;
    al.part_ml = dl.part_ml;
    al.n_items = dl.n_items;
    al.n_q_heads = Hq;
    al.n_kv_heads = dl.n_kv_heads;
    al.head_dim = D;
    al.scale_log2 = scale_log2;
    TimedScope t(ctx, 7, stream);
    HEDDLE_HIP(launch_narrow_attn(al, stream));
  } else {
    TimedScope t(ctx, 0, stream);
    HEDDLE_HIP(launch_decode_splitk(dl, stream));
  }
  if (n_parts > nB) {
    TimedScope t(ctx, 1, stream);
    HEDDLE_HIP(launch_decode_combine(dl, stream));
  }
  return HEDDLE_OK;
}

}  // namespace

int heddle_attn_decode_shared(heddle_ctx* ctx, const heddle_decode_args* args, const int32_t* block_ids_host,
                              void* hip_stream) {
  if (block_ids_host == nullptr) return HEDDLE_E_INVAL;
  return decode_call(ctx, args, block_ids_host, hip_stream, false);
}

int heddle_plan_append_split(const heddle_ctx* ctx, int32_t B, const int32_t* ctx_len_host,
                             const int32_t* cu_chunk_host, int32_t tile_rows, heddle_append_split_plan* plan) {
  if (ctx == nullptr || plan == nullptr || ctx_len_host == nullptr || cu_chunk_host == nullptr || B < 1)
    return HEDDLE_E_INVAL;
  if (!plan->tile_b || !plan->tile_row0 || !plan->tile_rows_n || !plan->tile_extent || !plan->tile_nsplit ||
      !plan->tile_part_base || !plan->item_tile || !plan->item_k || !plan->item_step_begin || !plan->item_step_end)
    return HEDDLE_E_INVAL;
  if (cu_chunk_host[0] != 0) return HEDDLE_E_INVAL;
  for (int32_t b = 0; b < B; ++b) {
    const int64_t C = static_cast<int64_t>(cu_chunk_host[b + 1]) - cu_chunk_host[b];
    if (C < 1 || ctx_len_host[b] < 0 || ctx_len_host[b] + C > HEDDLE_MAX_CONTEXT) return HEDDLE_E_INVAL;
  }
  if (tile_rows <= 0) tile_rows = append_tile_rows(ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads);
  if (tile_rows < 1) tile_rows = 1;
  std::vector<AppendTile> tiles;
  plan_append(B, ctx_len_host, cu_chunk_host, tile_rows, tiles);
  AppendSplit sp;
  split_append_tiles(ctx->plan, ctx->append_wg_per_cu, ctx->append_min_steps, tiles, ctx_len_host, sp);
  if (static_cast<int64_t>(tiles.size()) > plan->cap_tiles || static_cast<int64_t>(sp.items.size()) > plan->cap_items)
    return HEDDLE_E_NOMEM;
  plan->n_tiles = static_cast<int32_t>(tiles.size());
  plan->n_items = static_cast<int32_t>(sp.items.size());
  plan->n_slots = sp.n_slots;
  plan->tile_rows = tile_rows;
  for (size_t t = 0; t < tiles.size(); ++t) {
    plan->tile_b[t] = tiles[t].b;
    plan->tile_row0[t] = tiles[t].row0;
    plan->tile_rows_n[t] = tiles[t].rows;
    plan->tile_extent[t] = tiles[t].extent;
    plan->tile_nsplit[t] = sp.nsplit[t];
    plan->tile_part_base[t] = sp.part_base[t];
  }
  for (size_t i = 0; i < sp.items.size(); ++i) {
    plan->item_tile[i] = sp.items[i].tile;
    plan->item_k[i] = sp.items[i].k;
    plan->item_step_begin[i] = sp.items[i].step_begin;
    plan->item_step_end[i] = sp.items[i].step_end;
  }
  return HEDDLE_OK;
}

int heddle_attn_decode(heddle_ctx* ctx, const heddle_decode_args* args, void* hip_stream) {
  return decode_call(ctx, args, nullptr, hip_stream, false);
}

int heddle_attn_decode_static(heddle_ctx* ctx, const heddle_decode_args* args, void* hip_stream) {
  return decode_call(ctx, args, nullptr, hip_stream, true);
}

int heddle_attn_append(heddle_ctx* ctx, const heddle_append_args* args, void* hip_stream) {
  if (ctx == nullptr || args == nullptr) return HEDDLE_E_INVAL;
  if (!ctx->has_device) return HEDDLE_E_UNSUPPORTED;
  const int32_t B = args->B;
  if (B < 1 || !args->ctx_len_host || !args->cu_chunk_host || !args->row_off_host || !args->row_off ||
      !args->block_ids || !args->q || !args->out)
    return HEDDLE_E_INVAL;
  if ((args->k == nullptr) != (args->v == nullptr)) return HEDDLE_E_INVAL;
  if (misaligned(args->q) || misaligned(args->out) || misaligned(args->k) || misaligned(args->v) ||
      misaligned(ctx->cfg.kv_pool))
    return HEDDLE_E_INVAL;
  if (args->cu_chunk_host[0] != 0 || args->row_off_host[0] < 0) return HEDDLE_E_INVAL;
  for (int32_t b = 0; b < B; ++b) {
    const int64_t C = static_cast<int64_t>(args->cu_chunk_host[b + 1]) - args->cu_chunk_host[b];
    const int64_t L = args->ctx_len_host[b];
    if (C < 1 || L < 0 || L + C > HEDDLE_MAX_CONTEXT) return HEDDLE_E_INVAL;
    if (args->row_off_host[b + 1] < args->row_off_host[b] || !table_covers(args->row_off_host, b, L + C))
      return HEDDLE_E_INVAL;
  }
  const int32_t G = ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads;
  if (!append_shape_supported(G, ctx->cfg.head_dim)) return HEDDLE_E_UNSUPPORTED;

  DeviceGuard guard(ctx->cfg.device);
  if (!guard.ok()) return HEDDLE_E_HIP;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  plan_append(B, args->ctx_len_host, args->cu_chunk_host, append_tile_rows(G), ctx->tiles);
  AppendSplit& sp = ctx->split;
  split_append_tiles(ctx->plan, ctx->append_wg_per_cu, ctx->append_min_steps, ctx->tiles, args->ctx_len_host, sp);
  const size_t n_items = sp.items.size();
  const int32_t n_rows = args->cu_chunk_host[B];
  const bool any_split = sp.n_slots > 0;
  const int32_t Hq = ctx->cfg.n_q_heads, D = ctx->cfg.head_dim;

  int rc = HEDDLE_OK;
  if (any_split) {
    rc = grow_device(reinterpret_cast<void**>(&ctx->dev_part_acc), &ctx->dev_part_acc_elems,
                     static_cast<size_t>(sp.n_slots) * Hq * D, sizeof(float));
    if (rc != HEDDLE_OK) return rc;
    rc = grow_device(reinterpret_cast<void**>(&ctx->dev_part_ml), &ctx->dev_part_ml_elems,
                     static_cast<size_t>(sp.n_slots) * Hq * 4, sizeof(float));
    if (rc != HEDDLE_OK) return rc;
  }

  // rows of split tiles: the combine pass runs over these only
  size_t n_split_rows = 0;
  for (size_t t = 0; t < ctx->tiles.size(); ++t)
    if (sp.nsplit[t] > 1) n_split_rows += static_cast<size_t>(ctx->tiles[t].rows);

  // plan image: item records | ctx_len[B] | cu_chunk[B+1] | cu_wblk[B+1] | records of the split rows | their row numbers
  const size_t words = 8 * n_items + 3 * static_cast<size_t>(B) + 2 + 3 * n_split_rows;
  rc = enter_stream(ctx, stream);
  if (rc != HEDDLE_OK) return rc;
  StagingSlot* slot = nullptr;
  rc = acquire_slot(ctx, words, &slot);
  if (rc != HEDDLE_OK) return rc;
  int32_t* w = slot->host;
  AppendItemRec* h_items = reinterpret_cast<AppendItemRec*>(w);
  int32_t* h_len = w + 8 * n_items;
  int32_t* h_cu = h_len + B;
  int32_t* h_wblk = h_cu + B + 1;
  DecodeTrajRec* h_rows = reinterpret_cast<DecodeTrajRec*>(h_wblk + B + 1);
  h_wblk[0] = 0;
  for (int32_t b = 0; b < B; ++b) {          // pool blocks that receive the chunk's rows
    const int32_t L = args->ctx_len_host[b], C = args->cu_chunk_host[b + 1] - args->cu_chunk_host[b];
    h_wblk[b + 1] = h_wblk[b] + ((L + C - 1) / HEDDLE_BLOCK_TOKENS - L / HEDDLE_BLOCK_TOKENS + 1);
  }
  std::memcpy(h_len, args->ctx_len_host, sizeof(int32_t) * B);
  std::memcpy(h_cu, args->cu_chunk_host, sizeof(int32_t) * (static_cast<size_t>(B) + 1));
  // items of tiles with few rows go to the kernel that splits the keys over its waves; both lists
  // keep the planner's longest-first order: [0, n_wide) wide, [n_wide, n_items) narrow
  // -- unless they are the smaller part of the batch: a few short-row tiles next to a large append
  // would make a second launch that runs alone on a handful of compute units, while inside the
  // large launch they cost next to nothing
  int32_t narrow_rows = narrow_shape_supported(G, D) ? narrow_tile_rows(G) : 0;
  size_t n_wide = 0;
  int64_t steps_wide = 0, steps_narrow = 0;
  for (const AppendItem& it : sp.items) {
    const bool wide = ctx->tiles[static_cast<size_t>(it.tile)].rows > narrow_rows;
    (wide ? steps_wide : steps_narrow) += it.step_end - it.step_begin;
    n_wide += wide ? 1 : 0;
  }
  if (steps_narrow < steps_wide) {
    narrow_rows = 0;
    n_wide = n_items;
  }
  size_t next_wide = 0, next_narrow = n_wide;
  for (size_t i = 0; i < n_items; ++i) {
    const AppendItem& it = sp.items[i];
    const AppendTile& tl = ctx->tiles[static_cast<size_t>(it.tile)];
    AppendItemRec& r = h_items[tl.rows > narrow_rows ? next_wide++ : next_narrow++];
    r.b = tl.b;
    r.row0 = tl.row0;
    r.rows_n = tl.rows;
    r.key_end = std::min(tl.extent, it.step_end * kAppendStepKeys);
    r.step_begin = it.step_begin;
    r.nsplit = sp.nsplit[static_cast<size_t>(it.tile)];
    r.slot0 = sp.part_base[static_cast<size_t>(it.tile)] + it.k;
    r.pad = 0;
  }
  int32_t* h_row_no = reinterpret_cast<int32_t*>(h_rows + n_split_rows);
  {
    size_t i = 0;
    for (size_t t = 0; t < ctx->tiles.size(); ++t) {
      if (sp.nsplit[t] == 1) continue;
      const AppendTile& tl = ctx->tiles[t];
      const int32_t first_row = args->cu_chunk_host[tl.b] + tl.row0;
      for (int32_t r = 0; r < tl.rows; ++r, ++i) {
        h_rows[i].part_off = sp.part_base[t] + r * sp.nsplit[t];
        h_rows[i].nsplit = sp.nsplit[t];
        h_row_no[i] = first_row + r;
      }
    }
  }
  rc = upload(ctx, slot, words, stream);
  if (rc != HEDDLE_OK) return rc;
  ctx->enqueued = true;
  const int32_t* d = ctx->dev_plan;

  if (args->k != nullptr) {
    KvWriteLaunch kw{};
    kw.pool = static_cast<uint16_t*>(ctx->cfg.kv_pool);
    kw.row_off = args->row_off;
    kw.block_ids = args->block_ids;
    kw.first_pos = d + (h_len - w);
    kw.cu_rows = d + (h_cu - w);
    kw.cu_wblk = d + (h_wblk - w);
    kw.k = static_cast<const uint16_t*>(args->k);
    kw.v = static_cast<const uint16_t*>(args->v);
    kw.B = B;
    kw.n_rows = n_rows;
    kw.n_wblk = h_wblk[B];
    kw.n_kv_heads = ctx->cfg.n_kv_heads;
    kw.head_dim = ctx->cfg.head_dim;
    TimedScope t(ctx, 3, stream);
    HEDDLE_HIP(launch_kv_write(kw, stream));
  }

  AppendLaunch al{};
  al.pool = static_cast<const uint16_t*>(ctx->cfg.kv_pool);
  al.row_off = args->row_off;
  al.block_ids = args->block_ids;
  al.ctx_len = d + (h_len - w);
  al.cu_chunk = d + (h_cu - w);
  al.items = reinterpret_cast<const AppendItemRec*>(d);
  al.part_acc = ctx->dev_part_acc;
  al.part_ml = ctx->dev_part_ml;
  al.q = static_cast<const uint16_t*>(args->q);
  al.out = static_cast<uint16_t*>(args->out);
  al.lse = args->lse;
  al.n_items = static_cast<int32_t>(n_wide);
  al.n_q_heads = ctx->cfg.n_q_heads;
  al.n_kv_heads = ctx->cfg.n_kv_heads;
  al.head_dim = ctx->cfg.head_dim;
  al.scale_log2 = ctx->scale * 1.4426950408889634f;
  if (n_wide > 0) {
    TimedScope t(ctx, 2, stream);
    HEDDLE_HIP(launch_append_attn(al, stream));
  }
  if (n_items > n_wide) {
    al.items += n_wide;
    al.n_items = static_cast<int32_t>(n_items - n_wide);
    TimedScope t(ctx, 7, stream);
    HEDDLE_HIP(launch_narrow_attn(al, stream));
  }
  if (any_split) {          // merge the parts of every row of a split tile; rows of other tiles are final
    DecodeLaunch dl{};
    dl.trajs = reinterpret_cast<const DecodeTrajRec*>(d + (reinterpret_cast<int32_t*>(h_rows) - w));
    dl.out_row = d + (h_row_no - w);
    dl.part_acc = ctx->dev_part_acc;
    dl.part_ml = ctx->dev_part_ml;
    dl.out = static_cast<uint16_t*>(args->out);
    dl.lse = args->lse;
    dl.B = static_cast<int32_t>(n_split_rows);
    dl.n_q_heads = Hq;
    dl.n_kv_heads = ctx->cfg.n_kv_heads;
    dl.head_dim = D;
    TimedScope t(ctx, 1, stream);
    HEDDLE_HIP(launch_decode_combine(dl, stream));
  }
  return HEDDLE_OK;
}

static int kv_move(heddle_ctx* ctx, bool pack, int32_t n, const int32_t* block_ids_host, void* staging,
                   void* hip_stream) {
  if (ctx == nullptr || n < 0 || (n > 0 && (block_ids_host == nullptr || staging == nullptr))) return HEDDLE_E_INVAL;
  if (misaligned(staging) || misaligned(ctx->cfg.kv_pool)) return HEDDLE_E_INVAL;
  const int64_t block_bytes =
      static_cast<int64_t>(ctx->cfg.n_kv_heads) * 2 * HEDDLE_BLOCK_TOKENS * ctx->cfg.head_dim * 2;
  for (int32_t i = 0; i < n; ++i)
    if (block_ids_host[i] < 0 || block_ids_host[i] >= ctx->cfg.n_blocks) return HEDDLE_E_INVAL;
  if (!pack) {   // two staged blocks must not land in the same pool block
    std::vector<int32_t> sorted(block_ids_host, block_ids_host + n);
    std::sort(sorted.begin(), sorted.end());
    if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return HEDDLE_E_INVAL;
  }
  if (!ctx->has_device || block_bytes % 4096 != 0) return HEDDLE_E_UNSUPPORTED;
  if (n == 0) return HEDDLE_OK;
  DeviceGuard guard(ctx->cfg.device);
  if (!guard.ok()) return HEDDLE_E_HIP;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int rc = enter_stream(ctx, stream);
  if (rc != HEDDLE_OK) return rc;
  StagingSlot* slot = nullptr;
  rc = acquire_slot(ctx, static_cast<size_t>(n), &slot);
  if (rc != HEDDLE_OK) return rc;
  std::memcpy(slot->host, block_ids_host, sizeof(int32_t) * static_cast<size_t>(n));
  rc = upload(ctx, slot, static_cast<size_t>(n), stream);
  if (rc != HEDDLE_OK) return rc;
  ctx->enqueued = true;
  TimedScope t(ctx, pack ? 4 : 5, stream);
  HEDDLE_HIP(launch_kv_move(pack, ctx->cfg.kv_pool, staging, ctx->dev_plan, n, block_bytes, stream));
  return HEDDLE_OK;
}

int heddle_kv_pack(heddle_ctx* ctx, int32_t n, const int32_t* block_ids_host, void* staging, void* hip_stream) {
  return kv_move(ctx, true, n, block_ids_host, staging, hip_stream);
}

int heddle_kv_unpack(heddle_ctx* ctx, int32_t n, const int32_t* block_ids_host, const void* staging,
                     void* hip_stream) {
  return kv_move(ctx, false, n, block_ids_host, const_cast<void*>(staging), hip_stream);
}

int heddle_kv_copy(heddle_ctx* ctx, int32_t n, const int32_t* src_block_ids_host, const int32_t* dst_block_ids_host,
                   void* hip_stream) {
  if (ctx == nullptr || n < 0 || (n > 0 && (src_block_ids_host == nullptr || dst_block_ids_host == nullptr)))
    return HEDDLE_E_INVAL;
  const int64_t block_bytes =
      static_cast<int64_t>(ctx->cfg.n_kv_heads) * 2 * HEDDLE_BLOCK_TOKENS * ctx->cfg.head_dim * 2;
  for (int32_t i = 0; i < n; ++i)
    if (src_block_ids_host[i] < 0 || src_block_ids_host[i] >= ctx->cfg.n_blocks || dst_block_ids_host[i] < 0 ||
        dst_block_ids_host[i] >= ctx->cfg.n_blocks)
      return HEDDLE_E_INVAL;
  {   // every destination is written once and read by nobody in this call
    std::vector<int32_t> dst(dst_block_ids_host, dst_block_ids_host + n);
    std::sort(dst.begin(), dst.end());
    if (std::adjacent_find(dst.begin(), dst.end()) != dst.end()) return HEDDLE_E_INVAL;
    for (int32_t i = 0; i < n; ++i)
      if (std::binary_search(dst.begin(), dst.end(), src_block_ids_host[i])) return HEDDLE_E_INVAL;
  }
  if (!ctx->has_device || block_bytes % 4096 != 0) return HEDDLE_E_UNSUPPORTED;
  if (n == 0) return HEDDLE_OK;
  DeviceGuard guard(ctx->cfg.device);
  if (!guard.ok()) return HEDDLE_E_HIP;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int rc = enter_stream(ctx, stream);
  if (rc != HEDDLE_OK) return rc;
  StagingSlot* slot = nullptr;
  rc = acquire_slot(ctx, 2 * static_cast<size_t>(n), &slot);
  if (rc != HEDDLE_OK) return rc;
  std::memcpy(slot->host, src_block_ids_host, sizeof(int32_t) * static_cast<size_t>(n));
  std::memcpy(slot->host + n, dst_block_ids_host, sizeof(int32_t) * static_cast<size_t>(n));
  rc = upload(ctx, slot, 2 * static_cast<size_t>(n), stream);
  if (rc != HEDDLE_OK) return rc;
  ctx->enqueued = true;
  HEDDLE_HIP(launch_kv_copy(ctx->cfg.kv_pool, ctx->dev_plan, n, block_bytes, stream));
  return HEDDLE_OK;
}

int heddle_timing_enable(heddle_ctx* ctx, int32_t on) {
  if (ctx == nullptr) return HEDDLE_E_INVAL;
  if (!ctx->has_device) return HEDDLE_E_UNSUPPORTED;
  DeviceGuard guard(ctx->cfg.device);
  if (!guard.ok()) return HEDDLE_E_HIP;
  if (on) {
    HEDDLE_HIP(hipDeviceSynchronize());
    for (KernelTimer& t : ctx->timers) {
      while (t.start.size() < static_cast<size_t>(kEventPairs)) {
        hipEvent_t a = nullptr, b = nullptr;          // a pair or nothing: the two lists stay the same length
        HEDDLE_HIP(hipEventCreate(&a));
        const hipError_t e = hipEventCreate(&b);
        if (e != hipSuccess) {
          (void)hipEventDestroy(a);
          return hip_failed(e, "hipEventCreate", __LINE__);
        }
        t.start.push_back(a);
        t.stop.push_back(b);
      }
      t.recorded = 0;
      t.seen = 0;
    }
  }
  ctx->timing_every = on > 0 ? on : 0;
  return HEDDLE_OK;
}

int heddle_timing_read(heddle_ctx* ctx, int32_t which, double* avg_us, int64_t* n_launches) {
  if (ctx == nullptr || which < 0 || which >= kTimedKernels || avg_us == nullptr) return HEDDLE_E_INVAL;
  if (!ctx->has_device) return HEDDLE_E_UNSUPPORTED;
  DeviceGuard guard(ctx->cfg.device);
  if (!guard.ok()) return HEDDLE_E_HIP;
  KernelTimer& t = ctx->timers[which];
  const int64_t n = t.recorded < kEventPairs ? t.recorded : kEventPairs;
  double total_ms = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    HEDDLE_HIP(hipEventSynchronize(t.stop[i]));
    float ms = 0.f;
    HEDDLE_HIP(hipEventElapsedTime(&ms, t.start[i], t.stop[i]));
    total_ms += ms;
  }
  *avg_us = n > 0 ? total_ms * 1000.0 / static_cast<double>(n) : 0.0;
  if (n_launches) *n_launches = n;
  return HEDDLE_OK;
}

int heddle_timing_samples(heddle_ctx* ctx, int32_t which, int64_t cap, float* us_out, int64_t* n_out) {
  if (ctx == nullptr || which < 0 || which >= kTimedKernels || n_out == nullptr || cap < 0 ||
      (cap > 0 && us_out == nullptr))
    return HEDDLE_E_INVAL;
  if (!ctx->has_device) return HEDDLE_E_UNSUPPORTED;
  DeviceGuard guard(ctx->cfg.device);
  if (!guard.ok()) return HEDDLE_E_HIP;
  KernelTimer& t = ctx->timers[which];
  const int64_t have = t.recorded < kEventPairs ? t.recorded : kEventPairs;
  const int64_t n = have < cap ? have : cap;
  for (int64_t i = 0; i < n; ++i) {
    HEDDLE_HIP(hipEventSynchronize(t.stop[i]));
    float ms = 0.f;
    HEDDLE_HIP(hipEventElapsedTime(&ms, t.start[i], t.stop[i]));
    us_out[i] = ms * 1000.0f;
  }
  *n_out = have;
  return HEDDLE_OK;
}

int heddle_ctx_scratch_bytes(const heddle_ctx* ctx, uint64_t* out3) {
  if (ctx == nullptr || out3 == nullptr) return HEDDLE_E_INVAL;
  out3[0] = ctx->dev_plan_words * sizeof(int32_t);
  out3[1] = (ctx->dev_part_acc_elems + ctx->dev_part_ml_elems) * sizeof(float);
  uint64_t staging = 0;
  for (const StagingSlot& sl : ctx->staging) staging += sl.cap_words * sizeof(int32_t);
  out3[2] = staging;
  return HEDDLE_OK;
}

int heddle_stream_read(const void* src, uint64_t bytes, uint32_t* sink, void* hip_stream) {
  if (src == nullptr || sink == nullptr || bytes < 16) return HEDDLE_E_INVAL;
  HEDDLE_HIP(launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(hip_stream)));
  return HEDDLE_OK;
}

const char* heddle_strerror(int code) {
  switch (code) {
    case HEDDLE_OK: return "ok";
    case HEDDLE_E_INVAL: return "invalid argument";
    case HEDDLE_E_NOMEM: return "out of blocks or memory";
    case HEDDLE_E_HIP: return "HIP runtime error";
    case HEDDLE_E_UNSUPPORTED: return "unsupported shape or context";
    default: return "unknown error";
  }
}

const char* heddle_last_error_detail(void) { return g_detail; }

int heddle_version(void) { return 1; }

}  // extern "C"
