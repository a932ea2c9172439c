// C ABI of the sparse MLA decode library (see include/omniattn.h).
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>

#include "kernels.h"
#include "plan.h"

using namespace omniattn;

struct omniattn_plan_s {
  HostPlan hp;
  bool on_device = false;
  int device = -1;
  int num_cus = 0;
  int xcds = 1;        // work group i runs on XCD i % xcds (measured once per device)
  // Device copy of the plan metadata (owned): one allocation holding the unit headers, the
  // segments and the combine items, filled by one asynchronous copy from one of two pinned
  // host buffers of the same layout (used in turn; an event per buffer says when its last
  // copy has been read).  omniattn_plan_update reuses all of it when the new plan fits.
  uint8_t* d_meta = nullptr;
  size_t meta_cap = 0;
  uint8_t* h_meta[2] = {nullptr, nullptr};
  hipEvent_t h_done[2] = {nullptr, nullptr};
  bool h_busy[2] = {false, false};
  int h_next = 0;
  size_t off_segs = 0, off_combine = 0;
};

static __device__ __align__(256) unsigned char scratch[OMNIATTN_STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_hip_error;

int hip_fail(hipError_t e, const char* what) {
  g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  (void)hipGetLastError();  // clear the sticky "last error" so later calls are not blamed
  return OMNIATTN_EHIP;
}

#define OA_HIP(call)                                  \
  do {                                                \
    hipError_t e_ = (call);                           \
    if (e_ != hipSuccess) return hip_fail(e_, #call); \
  } while (0)

// The kernels' dynamic-LDS limit is a per-device function attribute: set once per device.
constexpr int kMaxDevices = 64;
std::mutex g_init_mutex;
bool g_init_done[kMaxDevices] = {};

// Workspace of omniattn_decode_static: partial rows of split sequences and their lse.
// Every device the library runs on holds its own copy of this array until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// address kernels and copies use is the per-device pointer taken once in init_device.
constexpr size_t kStaticScratchBytes = OMNIATTN_STATIC_SCRATCH_BYTES;
void* g_scratch_ptr[kMaxDevices] = {};
int g_xcds[kMaxDevices] = {};

int init_device(int dev) {
  if (dev < 0 || dev >= kMaxDevices) return OMNIATTN_EINVAL;
  std::lock_guard<std::mutex> lock(g_init_mutex);
  if (g_init_done[dev]) return OMNIATTN_OK;
  hipError_t e = init_kernels();
  if (e == hipSuccess) e = init_fp8_kernel();
  if (e != hipSuccess) return hip_fail(e, "kernel attribute setup");
  // (the caller made `dev` current: the address is that of this device's copy)
  void* sp = nullptr;
  e = hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !sp) return hip_fail(e != hipSuccess ? e : hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
  g_scratch_ptr[dev] = sp;
  int xcds = 1;
  e = probe_xcds(&xcds);
  if (e != hipSuccess) return hip_fail(e, "XCD probe");
  g_xcds[dev] = xcds;
  g_init_done[dev] = true;
  return OMNIATTN_OK;
}

void free_device(omniattn_plan_s* pl) {
  if (pl->d_meta) (void)hipFree(pl->d_meta);
  for (int i = 0; i < 2; ++i) {
    if (pl->h_meta[i]) (void)hipHostFree(pl->h_meta[i]);
    if (pl->h_done[i]) (void)hipEventDestroy(pl->h_done[i]);
    pl->h_meta[i] = nullptr;
    pl->h_done[i] = nullptr;
    pl->h_busy[i] = false;
  }
  pl->d_meta = nullptr;
  pl->meta_cap = 0;
}

int build_plan(HostPlan& hp, const omniattn_problem_t& prob, const int32_t* seq_lens, int num_cus) {
  try {
    return build_host_plan(hp, prob, seq_lens, num_cus);
  } catch (const std::bad_alloc&) {
    return OMNIATTN_ENOMEM;
  } catch (...) {
    return OMNIATTN_EINVAL;
  }
}

int make_plan(omniattn_plan_t** plan_out, const omniattn_problem_t* prob, const int32_t* seq_lens,
              int num_cus) {
  omniattn_plan_s* pl = new (std::nothrow) omniattn_plan_s();
  if (!pl) return OMNIATTN_ENOMEM;
  const int rc = build_plan(pl->hp, *prob, seq_lens, num_cus);
  if (rc != OMNIATTN_OK) {
    delete pl;
    return rc;
  }
  pl->num_cus = num_cus;
  *plan_out = pl;
  return OMNIATTN_OK;
}

size_t align16(size_t n) { return (n + 15) & ~(size_t)15; }

// Copies the host plan's metadata to the device on `stream` without synchronising.  Device
// and pinned buffers are allocated on the first call and again only when a plan outgrows them.
int upload_plan(omniattn_plan_s* pl, hipStream_t stream) {
  const HostPlan& hp = pl->hp;
  const size_t n_units = hp.unit_seg.size() - 1, n_segs = hp.segs.size(), n_items = hp.combine.size();
  pl->off_segs = align16(n_units * sizeof(UnitHeader));
  pl->off_combine = pl->off_segs + align16(n_segs * sizeof(DevSegment));
  const size_t bytes = pl->off_combine + align16(n_items * sizeof(CombineItem));
  if (bytes > pl->meta_cap) {
    // (rare: a plan larger than any before it; freeing waits for the device)
    const size_t cap = bytes + bytes / 2 + 4096;
    if (pl->d_meta) (void)hipFree(pl->d_meta);
    pl->d_meta = nullptr;
    pl->meta_cap = 0;
    for (int i = 0; i < 2; ++i) {
      if (pl->h_meta[i]) (void)hipHostFree(pl->h_meta[i]);
      pl->h_meta[i] = nullptr;
      pl->h_busy[i] = false;
      OA_HIP(hipHostMalloc((void**)&pl->h_meta[i], cap, hipHostMallocDefault));
      if (!pl->h_done[i]) OA_HIP(hipEventCreateWithFlags(&pl->h_done[i], hipEventDisableTiming));
    }
    OA_HIP(hipMalloc((void**)&pl->d_meta, cap));
    pl->meta_cap = cap;
  }
  const int hi = pl->h_next;
  pl->h_next ^= 1;
  if (pl->h_busy[hi]) OA_HIP(hipEventSynchronize(pl->h_done[hi]));  // its previous copy has been read
  uint8_t* h = pl->h_meta[hi];
  // The kernels read a segment's partial slots where the planner's record has the unit and tile count.
  std::vector<int32_t> item_of_slot((size_t)hp.n_slots, -1);
  for (size_t i = 0; i < n_items; ++i)
    for (int k = 0; k < hp.combine[i].nslots; ++k) item_of_slot[hp.combine[i].slot0 + k] = (int32_t)i;
  auto dev_seg = [&](size_t i) {
    const Segment& g = hp.segs[i];
    DevSegment d{g.b, g.hb, g.tile_lo, g.tile_hi, g.slot, 0, g.L, 0};
    if (g.slot >= 0) {
      const CombineItem& it = hp.combine[item_of_slot[g.slot]];
      d.slot0 = it.slot0;
      d.nslots = it.nslots;
    }
    return d;
  };
  UnitHeader* hu = (UnitHeader*)h;
  DevSegment* hs = (DevSegment*)(h + pl->off_segs);
  for (size_t i = 0; i < n_segs; ++i) hs[i] = dev_seg(i);
  for (size_t u = 0; u < n_units; ++u) {
    hu[u] = UnitHeader{hp.unit_seg[u], hp.unit_seg[u + 1], 0, 0, DevSegment{}};
    if (hu[u].seg_lo < hu[u].seg_hi) hu[u].first = hs[hu[u].seg_lo];
  }
  if (n_items) std::memcpy(h + pl->off_combine, hp.combine.data(), n_items * sizeof(CombineItem));
  OA_HIP(launch_copy16(pl->d_meta, h, bytes, stream));
  OA_HIP(hipEventRecord(pl->h_done[hi], stream));
  pl->h_busy[hi] = true;
  return OMNIATTN_OK;
}

}  // namespace

extern "C" {

int omniattn_plan_host(omniattn_plan_t** plan_out, const omniattn_problem_t* prob,
                       const int32_t* seq_lens_host, int32_t num_cus) {
  if (!plan_out) return OMNIATTN_EINVAL;
  *plan_out = nullptr;
  if (!prob || !seq_lens_host) return OMNIATTN_EINVAL;
  return make_plan(plan_out, prob, seq_lens_host, num_cus);
}

int omniattn_plan(omniattn_plan_t** plan_out, const omniattn_problem_t* prob,
                  const int32_t* seq_lens_host, void* hip_stream) {
  if (!plan_out) return OMNIATTN_EINVAL;
  *plan_out = nullptr;
  if (!prob || !seq_lens_host) return OMNIATTN_EINVAL;
  int dev = 0;
  OA_HIP(hipGetDevice(&dev));
  int cus = 0;
  OA_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  int rc = init_device(dev);
  if (rc != OMNIATTN_OK) return rc;

  omniattn_plan_s* pl = nullptr;
  rc = make_plan(&pl, prob, seq_lens_host, cus > 0 ? cus : 256);
  if (rc != OMNIATTN_OK) return rc;
  pl->device = dev;
  pl->xcds = g_xcds[dev] > 0 ? g_xcds[dev] : 1;
  try {
    rc = upload_plan(pl, (hipStream_t)hip_stream);
  } catch (const std::bad_alloc&) {
    rc = OMNIATTN_ENOMEM;
  }
  if (rc != OMNIATTN_OK) {
    free_device(pl);
    delete pl;
    return rc;
  }
  pl->on_device = true;
  *plan_out = pl;
  return OMNIATTN_OK;
}

int omniattn_plan_update(omniattn_plan_t* plan, const int32_t* seq_lens_host, void* hip_stream) {
  if (!plan || !seq_lens_host) return OMNIATTN_EINVAL;
  const bool host_only = plan->device < 0;  // made by omniattn_plan_host: nothing to copy
  if (!host_only) {
    if (!plan->on_device) return OMNIATTN_EINVAL;
    int dev = -1;
    OA_HIP(hipGetDevice(&dev));
    if (dev != plan->device) return OMNIATTN_EINVAL;
  }
  // Planned into a scratch object first: a rejected length leaves the plan as it was.
  HostPlan next;
  const omniattn_problem_t prob = plan->hp.prob;
  int rc = build_plan(next, prob, seq_lens_host, plan->num_cus);
  if (rc != OMNIATTN_OK) return rc;
  plan->hp = std::move(next);
  if (host_only) return OMNIATTN_OK;
  try {
    rc = upload_plan(plan, (hipStream_t)hip_stream);
  } catch (const std::bad_alloc&) {
    rc = OMNIATTN_ENOMEM;
  }
  if (rc != OMNIATTN_OK) plan->on_device = false;  // its device copy is no longer whole
  return rc;
}

void omniattn_plan_destroy(omniattn_plan_t* plan) {
  if (!plan) return;
  free_device(plan);
  delete plan;
}

size_t omniattn_plan_workspace_bytes(const omniattn_plan_t* plan) {
  return plan ? plan->hp.workspace_bytes : 0;
}
int64_t omniattn_plan_retained_tokens(const omniattn_plan_t* plan) {
  return plan ? plan->hp.retained_tokens : 0;
}
int32_t omniattn_plan_num_units(const omniattn_plan_t* plan) {
  return plan ? (int32_t)plan->hp.unit_seg.size() - 1 : 0;
}
int32_t omniattn_plan_num_segments(const omniattn_plan_t* plan) {
  return plan ? (int32_t)plan->hp.segs.size() : 0;
}
int32_t omniattn_plan_num_partials(const omniattn_plan_t* plan) { return plan ? plan->hp.n_slots : 0; }
int32_t omniattn_plan_max_splits(const omniattn_plan_t* plan) { return plan ? plan->hp.max_splits : 0; }
int32_t omniattn_plan_num_splits(const omniattn_plan_t* plan) { return omniattn_plan_max_splits(plan); }
int32_t omniattn_plan_tile_tokens(const omniattn_plan_t* plan) { return plan ? plan->hp.tile : 0; }
int32_t omniattn_plan_head_block(const omniattn_plan_t* plan) { return plan ? plan->hp.head_block : 0; }

int32_t omniattn_plan_get_segments(const omniattn_plan_t* plan, int32_t* buf, int32_t cap) {
  if (!plan || (!buf && cap > 0) || cap < 0) return OMNIATTN_EINVAL;
  int32_t n = (int32_t)plan->hp.segs.size();
  if (n > cap) n = cap;
  static_assert(sizeof(Segment) == 8 * sizeof(int32_t), "segment layout is part of the ABI");
  if (n > 0) std::memcpy(buf, plan->hp.segs.data(), (size_t)n * sizeof(Segment));
  return n;
}

int omniattn_plan_tile_range(const omniattn_plan_t* plan, int32_t b, int32_t tile, int32_t* lo,
                             int32_t* hi) {
  if (!plan || !lo || !hi || b < 0 || b >= plan->hp.prob.batch) return OMNIATTN_EINVAL;
  TileLayout tl = tile_layout(plan->hp.seq_lens[b], plan->hp.prob.sink, plan->hp.window_union, plan->hp.tile);
  if (tile < 0 || tile >= tl.count()) return OMNIATTN_EINVAL;
  *lo = tl.logical(tile) * plan->hp.tile;
  *hi = *lo + plan->hp.tile;
  return OMNIATTN_OK;
}

int omniattn_decode(const omniattn_plan_t* plan, const void* q, const void* kv_cache,
                    const float* kv_scales, const int32_t* page_table, void* out, float* lse,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  return omniattn_decode_timed(plan, q, kv_cache, kv_scales, page_table, out, lse, workspace,
                               workspace_bytes, hip_stream, nullptr, nullptr, nullptr);
}

int omniattn_decode_timed(const omniattn_plan_t* plan, const void* q, const void* kv_cache,
                          const float* kv_scales, const int32_t* page_table, void* out,
                          float* lse, void* workspace, size_t workspace_bytes, void* hip_stream,
                          void* ev_begin, void* ev_main_end, void* ev_end) {
  if (!plan || !q || !kv_cache || !page_table || !out || !lse) return OMNIATTN_EINVAL;
  if (!plan->on_device) return OMNIATTN_EINVAL;
  int dev = -1;
  OA_HIP(hipGetDevice(&dev));
  if (dev != plan->device) return OMNIATTN_EINVAL;  // the plan's metadata lives on another device
  const HostPlan& hp = plan->hp;
  const bool fp8 = hp.prob.kv_dtype == OMNIATTN_FP8_E4M3;
  if (fp8 && !kv_scales) return OMNIATTN_EINVAL;
  if (hp.workspace_bytes > 0) {
    if (!workspace || workspace_bytes < hp.workspace_bytes) return OMNIATTN_EWORKSPACE;
    if (((uintptr_t)workspace & 255) != 0) return OMNIATTN_EWORKSPACE;
  }
  if ((((uintptr_t)q | (uintptr_t)kv_cache | (uintptr_t)out) & 15) != 0) return OMNIATTN_EINVAL;
  hipStream_t stream = (hipStream_t)hip_stream;

  DecodeParams dp;
  dp.q = (const uint16_t*)q;
  dp.kv = (const uint8_t*)kv_cache;
  dp.kv_scales = kv_scales;
  dp.page_table = page_table;
  dp.out = out;
  dp.lse = lse;
  dp.part_lse = (float*)workspace;
  dp.part_o = workspace ? (char*)workspace + hp.part_rows_offset : nullptr;
  dp.units = (const UnitHeader*)plan->d_meta;
  dp.segs = (const DevSegment*)(plan->d_meta + plan->off_segs);
  dp.xcds = plan->xcds;
  dp.H = hp.heads_total;
  dp.Hq = hp.prob.num_heads;
  dp.T = hp.q_len;
  dp.Wu = hp.window_union;
  dp.max_pages = hp.prob.max_pages_per_seq;
  dp.S = hp.prob.sink;
  dp.W = hp.prob.window;
  dp.head_block = hp.head_block;
  dp.out_fp32 = hp.prob.out_dtype == OMNIATTN_FP32;
  dp.n_units = (int)hp.unit_seg.size() - 1;
  // A zero scale (uniform attention) is replaced by one too small to matter: the kernel
  // marks masked positions with an infinity that must survive the multiplication.
  dp.scale_log2 = hp.prob.softmax_scale * 1.4426950408889634f;
  if (dp.scale_log2 == 0.f) dp.scale_log2 = 1e-30f;
  if (ev_begin) OA_HIP(hipEventRecord((hipEvent_t)ev_begin, stream));
  if (fp8) OA_HIP(launch_decode_fp8(dp, (int)hp.unit_seg.size() - 1, stream));
  else OA_HIP(launch_decode(dp, hp.waves, (int)hp.unit_seg.size() - 1, stream));
  if (ev_main_end) OA_HIP(hipEventRecord((hipEvent_t)ev_main_end, stream));

  if (!hp.combine.empty()) {
    CombineParams cp;
    cp.items = (const CombineItem*)(plan->d_meta + plan->off_combine);
    cp.part_o = dp.part_o;
    cp.part_lse = dp.part_lse;
    cp.out = out;
    cp.lse = lse;
    cp.H = dp.H;
    cp.head_block = hp.head_block;
    cp.out_fp32 = dp.out_fp32;
    cp.n_items = (int)hp.combine.size();
    OA_HIP(launch_combine(cp, (int)hp.combine.size(), stream));
  }
  if (ev_end) OA_HIP(hipEventRecord((hipEvent_t)ev_end, stream));
  return OMNIATTN_OK;
}

size_t omniattn_static_scratch_bytes(void) { return kStaticScratchBytes; }

int omniattn_decode_static(const omniattn_plan_t* plan, const void* q, const void* kv_cache,
                           const float* kv_scales, const int32_t* page_table, void* out, float* lse,
                           void* hip_stream) {
  if (!plan || !plan->on_device) return OMNIATTN_EINVAL;
  if (plan->hp.workspace_bytes > kStaticScratchBytes) return OMNIATTN_ESCRATCH;
  // the plan was made on plan->device, so that device's scratch address is known
  void* sp = plan->device >= 0 && plan->device < kMaxDevices ? g_scratch_ptr[plan->device] : nullptr;
  if (!sp) return OMNIATTN_EINVAL;
  return omniattn_decode_timed(plan, q, kv_cache, kv_scales, page_table, out, lse, sp, kStaticScratchBytes,
                               hip_stream, nullptr, nullptr, nullptr);
}

int32_t omniattn_ring_pages(int32_t sink, int32_t window) {
  if (sink < 0 || window < 0) return -1;
  return ring_pinned_pages(sink) + ring_ring_pages(window);
}

int32_t omniattn_ring_slot(int32_t sink, int32_t window, int32_t logical_page) {
  if (sink < 0 || window < 0 || logical_page < 0) return -1;
  return ring_slot(sink, window, logical_page);
}

int omniattn_ring_append(const omniattn_problem_t* prob, int32_t* seq_lens, const void* new_rows,
                         const float* new_scales, const int32_t* seq_pages, void* kv_cache,
                         float* kv_scales, int32_t* page_table, void* hip_stream) {
  if (!prob || !seq_lens || !new_rows || !seq_pages || !kv_cache || !page_table) return OMNIATTN_EINVAL;
  if (prob->batch < 1 || prob->max_pages_per_seq < 1 || prob->sink < 0 || prob->window < 0)
    return OMNIATTN_EINVAL;
  if (prob->qk_dim != kQK || prob->page_size != kPage) return OMNIATTN_EUNSUPPORTED;
  const bool fp8 = prob->kv_dtype == OMNIATTN_FP8_E4M3;
  if (!fp8 && prob->kv_dtype != OMNIATTN_BF16) return OMNIATTN_EUNSUPPORTED;
  if (fp8 && (!new_scales || !kv_scales)) return OMNIATTN_EINVAL;
  if ((((uintptr_t)new_rows | (uintptr_t)kv_cache) & 15) != 0) return OMNIATTN_EINVAL;
  AppendParams ap;
  ap.seq_lens = seq_lens;
  ap.new_rows = (const uint8_t*)new_rows;
  ap.new_scales = fp8 ? new_scales : nullptr;
  ap.seq_pages = seq_pages;
  ap.kv = (uint8_t*)kv_cache;
  ap.kv_scales = kv_scales;
  ap.page_table = page_table;
  ap.max_pages = prob->max_pages_per_seq;
  // With several queries per sequence the earliest query's window reaches q_len - 1 tokens
  // further back: the ring is laid out for the union of the queries' windows.
  if (prob->q_len < 0 || prob->q_len > 64) return OMNIATTN_EINVAL;
  const int64_t w_eff = prob->window > 0 ? (int64_t)prob->window + (prob->q_len > 1 ? prob->q_len - 1 : 0) : 0;
  if (w_eff > INT32_MAX) return OMNIATTN_EINVAL;
  ap.S = prob->sink;
  ap.W = (int)w_eff;
  ap.ring_pages = ring_pinned_pages(prob->sink) + ring_ring_pages((int)w_eff);
  ap.row_bytes = fp8 ? kQK : kQK * 2;
  OA_HIP(launch_append(ap, prob->batch, (hipStream_t)hip_stream));
  return OMNIATTN_OK;
}

const char* omniattn_strerror(int code) {
  switch (code) {
    case OMNIATTN_OK: return "ok";
    case OMNIATTN_EINVAL: return "invalid argument";
    case OMNIATTN_EUNSUPPORTED: return "unsupported dtype, head count or dimension";
    case OMNIATTN_EWORKSPACE: return "workspace missing, misaligned or too small";
    case OMNIATTN_EHIP: return "HIP call failed (see omniattn_last_hip_error)";
    case OMNIATTN_ENOMEM: return "out of host memory";
    case OMNIATTN_ESCRATCH:
      return "the plan's workspace exceeds the built-in scratch buffer of omniattn_decode_static "
             "(see omniattn_static_scratch_bytes); use omniattn_decode with a caller-owned workspace";
    default: return "unknown error code";
  }
}

const char* omniattn_last_hip_error(void) { return g_hip_error.c_str(); }

}  // extern "C"
