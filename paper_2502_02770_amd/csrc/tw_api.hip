// Host-side pieces shared by the entry points: argument checks, workspace
// sizes, error strings, and the optional per-kernel event timing.
#include <atomic>
#include <mutex>
#include "topp_common.h"

int tw_decode_chunk(bool dense);
long long tw_decode_max_items(const TwDims& d, bool dense, int union_stride);

int tw_check_kv(const twilight_kv_t* kv, TwDims* d) {
  if (!kv) return TW_EINVAL;
  if (kv->head_dim != TW_HEAD_DIM || kv->page_size != TW_PAGE || kv->quant_group != TW_QGROUP) return TW_EINVAL;
  if (kv->batch <= 0 || kv->num_q_heads <= 0 || kv->num_kv_heads <= 0) return TW_EINVAL;
  if (kv->num_q_heads % kv->num_kv_heads) return TW_EINVAL;
  const int G = kv->num_q_heads / kv->num_kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return TW_EINVAL;
  if (kv->max_pages_per_seq <= 0 || kv->max_pages_per_seq > (1 << 27)) return TW_EINVAL;
  if (kv->num_pool_pages <= 0 || kv->num_pool_pages * kv->num_kv_heads * TW_PAGE > 0x7FFFFFFFll) return TW_EINVAL;
  if ((long long)kv->batch * kv->num_q_heads > 65535ll) return TW_EINVAL;   // grid.y limit
  if (!kv->page_table || !kv->seq_lens) return TW_EINVAL;
  if (kv->quant_bits != 0 && kv->quant_bits != 2 && kv->quant_bits != 4 && kv->quant_bits != 8) return TW_EINVAL;
  d->bits = kv->quant_bits ? kv->quant_bits : 4;
  d->batch = kv->batch; d->Hq = kv->num_q_heads; d->Hkv = kv->num_kv_heads; d->G = G;
  d->max_pages = kv->max_pages_per_seq; d->pool_pages = kv->num_pool_pages;
  return TW_OK;
}

int tw_num_cus() {
  static std::atomic<int> cus[TW_MAX_DEVICES];    // read-only device property, cached per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= TW_MAX_DEVICES) return 256;
  int n = cus[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cus[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

extern "C" int twilight_pinned_device_pointer(void* host_ptr, void** device_ptr) {
  if (!host_ptr || !device_ptr) return TW_EINVAL;
  void* dp = nullptr;
  if (hipHostGetDevicePointer(&dp, host_ptr, 0) != hipSuccess || !dp) {
    (void)hipGetLastError();                       // not pinned / not mapped: leave no sticky error behind
    return TW_EINVAL;
  }
  *device_ptr = dp;
  return TW_OK;
}

extern "C" size_t twilight_workspace_bytes(int which, const twilight_kv_t* kv, int32_t max_sel, int32_t union_stride) {
  TwDims d;
  // the pointers are not needed for sizing: check the shape fields only
  twilight_kv_t tmp;
  if (!kv) return 0;
  tmp = *kv;
  int dummy = 0;
  tmp.page_table = &dummy; tmp.seq_lens = &dummy;
  if (tw_check_kv(&tmp, &d)) return 0;
  const size_t bh = (size_t)d.batch * d.Hq;
  switch (which) {
    case TW_WS_SELECT:
      return align256(bh * d.max_pages * 4);
    case TW_WS_DS_SELECT:
      return align256(bh * d.max_pages * TW_PAGE * 4);
    case TW_WS_PRUNE: {
      const int bound = max_sel > 0 ? max_sel : d.max_pages;
      return tw_prune_layout(d, bound, max_sel <= 0).total;
    }
    case TW_WS_SELECT_PRUNE: {
      if (max_sel <= 0) return 0;
      return align256(bh * d.max_pages * 4) + tw_prune_layout(d, max_sel, false).total;
    }
    case TW_WS_PRUNE_TOKENS:
      if (max_sel <= 0 || (max_sel & 15) || max_sel > 8192) return 0;
      return tw_prune_layout_tokens(d, max_sel).total;
    case TW_WS_DECODE: {
      const bool dense = union_stride <= 0;
      const size_t items = (size_t)tw_decode_max_items(d, dense, union_stride);
      return align256((size_t)(d.batch * d.Hkv + 1) * 4) + align256(items * d.G * 8) + align256(items * d.G * 128 * 4);
    }
    case TW_WS_DECODE_PER_HEAD: {
      if (union_stride <= 0) return 0;
      const size_t items = (size_t)tw_decode_max_items(d, false, union_stride) / d.Hkv * d.Hq;
      return align256((size_t)(d.batch * d.Hq + 1) * 4) + align256(items * 8) + align256(items * 128 * 4);
    }
    default:
      return 0;
  }
}

extern "C" const char* twilight_strerror(int code) {
  switch (code) {
    case TW_OK: return "ok";
    case TW_EINVAL: return "invalid argument (NULL pointer, unsupported shape or parameter)";
    case TW_EWORKSPACE: return "workspace missing or smaller than twilight_workspace_bytes";
    case TW_ELAUNCH: return "HIP reported an error (kernel launch, device or symbol query)";
    case TW_ELIMIT: return "problem exceeds the fixed scratch array of the entry point that allocates nothing";
    default: return "unknown error code";
  }
}

extern "C" int twilight_abi_version(void) { return TW_ABI_VERSION; }

extern "C" const char* twilight_kernel_name(int id) {
  static const char* names[TW_K_COUNT] = {"kquant_append", "page_score", "page_select", "int4_score",
                                          "topp", "union", "sparse_decode", "combine", "score_topp", "select_score_topp"};
  return (id >= 0 && id < TW_K_COUNT) ? names[id] : "?";
}

// ---------------------------------------------------------------- profiling
// The record list is the library's only process-global mutable state.  g_lock serialises every access;
// it is held from tw_prof_before to tw_prof_after of a timed launch (an open record), so launches of other
// threads wait for that one launch while timing is on.  With timing off no lock is taken.
namespace {
struct ProfRec { int id; hipEvent_t e0, e1; };
std::mutex g_lock;
std::atomic<int> g_on{0};   // == g_mode != 0, readable without the lock
int g_mode = 0;
int g_n = 0;
ProfRec g_rec[TW_PROF_MAX_RECORDS];
int g_created = 0;   // events exist for records [0, g_created)
int g_only = -1;     // mode 2: the one kernel id that is timed ...
int g_every = 1;     // ... at every g_every-th of its launches
long long g_seen = 0;
int g_last = -1;     // id of the latest launch of any kernel
int g_pred = -1;     // mode 3: the kernel id that was launched just before g_only's latest launch
}  // namespace

extern "C" int twilight_prof_select(int kernel_id, int every) {
  std::lock_guard<std::mutex> lk(g_lock);
  g_only = kernel_id;
  g_every = every > 0 ? every : 1;
  g_seen = 0;
  g_last = g_pred = -1;
  return TW_OK;
}

extern "C" int twilight_prof_enable(int mode) {
  std::lock_guard<std::mutex> lk(g_lock);
  g_mode = mode < 0 || mode > 3 ? 1 : mode;
  g_on.store(g_mode != 0, std::memory_order_release);
  g_n = 0;
  return TW_OK;
}

// the calling thread's open record (the lock is held while it is open)
static thread_local bool t_open = false;

void tw_prof_before(int kernel_id, hipStream_t s) {
  (void)s;
  t_open = false;
  if (!g_on.load(std::memory_order_acquire)) return;
  g_lock.lock();
  bool take = g_mode != 0 && g_n < TW_PROF_MAX_RECORDS;
  if (g_mode >= 2) {
    // mode 3 also times the launch that comes just before a timed launch of the chosen kernel (the kernel id seen
    // there last time), so that the chosen kernel's start stamp does not wait for an untimed predecessor to drain
    const bool sampled = g_seen % g_every == g_every - 1;   // (the last of every g_every launches: never the first after a start)
    if (kernel_id == g_only) { g_pred = g_last; ++g_seen; }
    else if (!(g_mode == 3 && kernel_id == g_pred)) take = false;
    if (!sampled) take = false;
    g_last = kernel_id;
  }
  if (take && g_n >= g_created) {
    if (hipEventCreate(&g_rec[g_n].e0) != hipSuccess) take = false;
    else if (hipEventCreate(&g_rec[g_n].e1) != hipSuccess) { (void)hipEventDestroy(g_rec[g_n].e0); take = false; }
    else g_created = g_n + 1;
  }
  if (!take) { g_lock.unlock(); return; }
  g_rec[g_n].id = kernel_id;
  t_open = true;                                  // g_lock stays held until tw_prof_after
}

bool tw_prof_events(hipEvent_t* start, hipEvent_t* stop) {
  if (!t_open) return false;
  *start = g_rec[g_n].e0;
  *stop = g_rec[g_n].e1;
  return true;
}

int tw_prof_after(hipStream_t s) {
  (void)s;
  if (t_open) {
    ++g_n;
    t_open = false;
    g_lock.unlock();
  }
  return hipGetLastError() == hipSuccess ? TW_OK : TW_ELAUNCH;
}

extern "C" int twilight_prof_collect(int32_t* kernel_ids, float* ms, int32_t cap) {
  std::lock_guard<std::mutex> lk(g_lock);
  int w = 0;
  for (int i = 0; i < g_n; ++i) {
    if (hipEventSynchronize(g_rec[i].e1) != hipSuccess) break;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_rec[i].e0, g_rec[i].e1) != hipSuccess) break;
    if (w < cap && kernel_ids && ms) { kernel_ids[w] = g_rec[i].id; ms[w] = t; ++w; }
  }
  g_n = 0;
  return w;
}
