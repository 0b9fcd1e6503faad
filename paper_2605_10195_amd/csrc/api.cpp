// C ABI of the tree decode-attention library: argument checking, the host page table and
// planner, device workspace management and kernel launches.  See include/spex_tree.h.
#include "../../include/spex_sched.h"
#include "../../include/spex_tree.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "kernels.hpp"
#include "page_table.hpp"
#include "planner.hpp"

namespace {

thread_local std::string g_last_error;

bool hip_failed(hipError_t e, const char *what) {
  if (e == hipSuccess) return false;
  g_last_error = std::string(what) + ": " + hipGetErrorString(e);
  return true;
}

#define HIP_TRY(expr)                                      \
  do {                                                     \
    if (hip_failed((expr), #expr)) return SPEX_ERR_DEVICE; \
  } while (0)

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool is_pow2(int32_t x) { return x > 0 && (x & (x - 1)) == 0; }

// Device copy of a Plan: one blob, arrays at 256-byte aligned offsets.
struct DevicePlan {
  const int32_t *prefix_items = nullptr, *suffix_items = nullptr, *pg_rec = nullptr, *qt_rec = nullptr;
  const int32_t *part_indptr = nullptr, *part_base = nullptr, *part_hstride = nullptr;
  const int32_t *merge_qt = nullptr;
  const int32_t *coop_items[3] = {nullptr, nullptr, nullptr};
  const int32_t *walk_items = nullptr, *walk_blocks = nullptr, *walk_qt = nullptr, *qt_mask = nullptr;
};

}  // namespace

struct spex_tree {
  spex_config_t cfg{};
  spex::Shape shape{};
  spex::PageTable *pt = nullptr;
  spex::Planner planner;
  spex::Plan plan;
  bool plan_on_device = false, device_has_split = false, device_has_walk = false;
  bool plan_patched_by_append = false;  // the cached plan was brought up to date by an append call
  DevicePlan dplan;
  size_t blob_off[15] = {}, blob_ints[15] = {};  // byte offset and length of each list in the blob
  std::vector<int32_t> pending_patches;          // {array, index, value} not yet on the device
  void *d_patch = nullptr;
  size_t d_patch_cap = 0;

  void *d_plan = nullptr;
  size_t d_plan_cap = 0;
  // Pinned staging for host -> device copies (plans, patches, append destinations).  Two slots
  // used in turn: the host may fill one while the copy out of the other is still queued behind
  // earlier kernels, so it can prepare the next call while the GPU runs the current one.
  struct Stage {
    void *h = nullptr;
    size_t cap = 0;
    hipEvent_t event = nullptr;
    bool pending = false;
  } stage[2];
  int stage_cur = 0;
  void *h_stage = nullptr;  // the slot reserved last (stage[stage_cur].h)

  float *d_part_o = nullptr, *d_part_ml = nullptr;
  int64_t part_cap_rows = 0;
  std::vector<char> static_stage;  // host image of the lists for the entry point that allocates nothing

  int32_t prefix_chunk = 0, suffix_chunk = 0, kernel_mode = 0, walk_row_tiles = 0, walk_waves = 0;
  // Profiling: a ring of event sets, one per decode_attention call since it was enabled.
  static constexpr int kProfSlots = 256;
  struct ProfSlot {
    hipEvent_t ev[8] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    bool valid[4] = {false, false, false, false};
  };
  bool profiling = false;
  std::vector<ProfSlot> prof;
  int64_t prof_calls = 0;  // calls recorded since profiling was enabled / last read
  int64_t info[8] = {0, 0, 0, 0, 0, 0, 0, 0};
};

namespace {

spex_status_t check_config(const spex_config_t *c) {
  if (!c) return SPEX_ERR_INVALID_ARG;
  if (c->num_q_heads <= 0 || c->num_kv_heads <= 0 || c->num_kv_heads > 255 ||
      c->num_q_heads % c->num_kv_heads != 0)
    return SPEX_ERR_INVALID_ARG;
  if (c->head_dim < 1 || c->head_dim > 256) return SPEX_ERR_INVALID_ARG;
  if (!is_pow2(c->page_size) || c->page_size > 64) return SPEX_ERR_INVALID_ARG;
  if (c->num_pages < 0 || c->num_pages > INT32_MAX) return SPEX_ERR_INVALID_ARG;
  if (c->prefix_chunk_pages < 0 || c->suffix_chunk_pages < 0) return SPEX_ERR_INVALID_ARG;
  if (c->page_stride_tiles != 0 && c->page_stride_tiles < c->num_kv_heads) return SPEX_ERR_INVALID_ARG;
  if (c->kernel_mode < 0 || c->kernel_mode > 3) return SPEX_ERR_INVALID_ARG;
  if (c->walk_row_tiles != 0 && c->walk_row_tiles != 1 && c->walk_row_tiles != 2 && c->walk_row_tiles != 4)
    return SPEX_ERR_INVALID_ARG;
  if (c->walk_waves != 0 && c->walk_waves != 2 && c->walk_waves != 4 && c->walk_waves != 8) return SPEX_ERR_INVALID_ARG;
  const bool ok = (c->q_dtype == SPEX_F32 && c->kv_dtype == SPEX_F32) ||
                  (c->q_dtype == SPEX_BF16 && c->kv_dtype == SPEX_BF16) ||
                  (c->q_dtype == SPEX_BF16 && c->kv_dtype == SPEX_FP8_E4M3);
  if (!ok) return SPEX_ERR_UNSUPPORTED;
  if ((c->k_pool == nullptr) != (c->v_pool == nullptr)) return SPEX_ERR_INVALID_ARG;
  if (c->kv_dtype == SPEX_FP8_E4M3 && c->k_pool && (!c->k_scale || !c->v_scale))
    return SPEX_ERR_INVALID_ARG;
  return SPEX_OK;
}

size_t elem_size(int32_t dt) { return dt == SPEX_F32 ? 4 : (dt == SPEX_BF16 ? 2 : 1); }

spex::Shape make_shape(const spex_config_t &c) {
  spex::Shape s{};
  s.Hq = c.num_q_heads;
  s.Hkv = c.num_kv_heads;
  s.G = c.num_q_heads / c.num_kv_heads;
  s.D = c.head_dim;
  s.P = c.page_size;
  s.q_dtype = c.q_dtype;
  s.kv_dtype = c.kv_dtype;
  const bool tiled = c.kv_dtype != SPEX_F32 && c.page_size == 16 && (c.head_dim == 64 || c.head_dim == 128);
  s.layout = tiled ? spex::kMfmaTiled : spex::kRowMajor;
  s.page_tiles = c.page_stride_tiles ? c.page_stride_tiles : c.num_kv_heads;
  return s;
}

bool request_matches(const spex::Plan &pl, const spex_tree *t, const int32_t *leaves,
                     const int32_t *q_lens, const uint32_t *masks, int32_t n) {
  if (!pl.valid) return false;
  if (pl.req_prefix_chunk != t->prefix_chunk || pl.req_suffix_chunk != t->suffix_chunk ||
      pl.req_walk_row_tiles != t->walk_row_tiles || pl.req_walk_waves != t->walk_waves)
    return false;
  if (static_cast<int32_t>(pl.req_leaves.size()) != n) return false;
  if (n && std::memcmp(pl.req_leaves.data(), leaves, sizeof(int32_t) * n) != 0) return false;
  if (q_lens) {
    if (static_cast<int32_t>(pl.req_q_lens.size()) != n) return false;
    if (n && std::memcmp(pl.req_q_lens.data(), q_lens, sizeof(int32_t) * n) != 0) return false;
  } else if (!pl.req_q_lens.empty()) {
    return false;
  }
  // same leaves and q_lens, hence the same number of query tokens and of masks
  if ((masks != nullptr) != !pl.req_masks.empty()) return false;
  if (masks && std::memcmp(pl.req_masks.data(), masks, sizeof(uint32_t) * pl.req_masks.size()) != 0)
    return false;
  return true;
}

spex_status_t plan_status(spex_tree *t, spex::PlanError e) {
  switch (e) {
    case spex::PlanError::kOk: return SPEX_OK;
    case spex::PlanError::kBadNode: t->plan.valid = false; return SPEX_ERR_BAD_NODE;
    case spex::PlanError::kEmptyPath: t->plan.valid = false; return SPEX_ERR_EMPTY_PATH;
    case spex::PlanError::kTooLarge: t->plan.valid = false; return SPEX_ERR_UNSUPPORTED;
    default: t->plan.valid = false; return SPEX_ERR_INVALID_ARG;
  }
}

// Brings t->plan up to date for the request.  *state: 0 = the cached plan still holds, 1 = planned
// afresh, 2 = the cached plan was patched (tokens were appended to requested nodes without starting
// a page; the changed entries wait in t->pending_patches for the device copy).
spex_status_t make_plan(spex_tree *t, const int32_t *leaves, const int32_t *q_lens,
                        const uint32_t *masks, int32_t n, int *state) {
  *state = 0;
  const bool by_append = t->plan_patched_by_append;
  t->plan_patched_by_append = false;
  if (request_matches(t->plan, t, leaves, q_lens, masks, n)) {
    if (t->plan.table_version == t->pt->version()) {
      if (by_append) *state = 2;  // patched already, by the append launch
      return SPEX_OK;
    }
    if (t->planner.patch_lengths(*t->pt, &t->plan, &t->pending_patches)) {
      *state = 2;
      return SPEX_OK;
    }
    t->plan.valid = false;  // possibly half changed; replaced below
  }
  *state = 1;
  t->plan_on_device = false;
  t->pending_patches.clear();
  return plan_status(t, t->planner.begin(*t->pt, leaves, q_lens, masks, n, t->cfg.num_q_heads,
                                         t->cfg.num_kv_heads, t->prefix_chunk, t->suffix_chunk,
                                         t->walk_row_tiles, t->walk_waves, &t->plan));
}

// Longest tree-walk workgroup (in two-page blocks) up to which a launch of `items` workgroups
// (< 128) still goes to the tree-walk kernel.
int32_t short_walk_blocks(int64_t items) {
  return items <= 32 ? 20 : 20 + static_cast<int32_t>((items - 32) * 7 / 10);
}

// True if the automatic choice is certain to be the split path, judged from the request alone:
// an upper bound on the tree-walk workgroups (no request has more rows than a 16-row wavefront,
// so none is cut; every wavefront holds at least one request, so a root with r requests has at
// most ceil(r / 4) row blocks) stays below 128, and a lower bound on
// the longest workgroup (the longest path, two full pages per block) exceeds what that many
// workgroups may walk.  Saves building the tree-walk lists just to discard them.
bool obviously_split(const spex::Plan &pl) {
  const size_t n = pl.req_leaves.size();
  if (n == 0 || n > 512) return false;
  const int32_t G = pl.num_q_heads / pl.num_kv_heads;
  int32_t roots[512], counts[512], n_roots = 0;
  int32_t longest = 0;
  for (size_t i = 0; i < n; ++i) {
    const int32_t r = pl.path_nodes[pl.path_indptr[i]];
    int32_t k = 0;
    while (k < n_roots && roots[k] != r) ++k;
    if (k == n_roots) {
      roots[n_roots] = r;
      counts[n_roots++] = 0;
    }
    ++counts[k];
    const int32_t ql = pl.req_q_lens.empty() ? 1 : pl.req_q_lens[i];
    if (static_cast<int64_t>(ql) * G > 16) return false;  // may be cut into pieces: no simple bound
    longest = std::max(longest, pl.qt_limit[pl.qoff[i] + ql - 1]);  // the path's tokens
  }
  int64_t items = 0;
  for (int32_t k = 0; k < n_roots; ++k) items += (counts[k] + 3) / 4;
  items *= pl.num_kv_heads;
  return items < 128 && (longest + 31) / 32 > short_walk_blocks(items);
}

constexpr int kPlanArrays = 15;
// Index, in the device blob's array list, of the arrays a length patch can touch.
constexpr int kPatchTarget[5] = {2 /*pg_rec*/, 3 /*qt_rec*/, 12 /*walk_blocks*/, 13 /*walk_qt*/, 11 /*walk_items*/};

spex_status_t stage_reserve(spex_tree *t, size_t bytes) {
  t->stage_cur ^= 1;
  spex_tree::Stage &st = t->stage[t->stage_cur];
  t->h_stage = nullptr;
  if (st.pending) {
    HIP_TRY(hipEventSynchronize(st.event));
    st.pending = false;
  }
  if (bytes > st.cap) {
    if (st.h) HIP_TRY(hipHostFree(st.h));
    st.h = nullptr;
    st.cap = 0;
    const size_t cap = align_up(bytes + bytes / 2, 1 << 16);
    HIP_TRY(hipHostMalloc(&st.h, cap, hipHostMallocDefault));
    st.cap = cap;
  }
  t->h_stage = st.h;
  return SPEX_OK;
}

spex_status_t stage_send(spex_tree *t, void *dst, size_t bytes, hipStream_t stream) {
  spex_tree::Stage &st = t->stage[t->stage_cur];
  HIP_TRY(hipMemcpyAsync(dst, st.h, bytes, hipMemcpyHostToDevice, stream));
  if (!st.event) HIP_TRY(hipEventCreateWithFlags(&st.event, hipEventDisableTiming));
  HIP_TRY(hipEventRecord(st.event, stream));
  st.pending = true;
  return SPEX_OK;
}

// Copies every list that has been built to the device (one blob, arrays at 256-byte offsets).
spex_status_t upload_plan(spex_tree *t, hipStream_t stream) {
  const spex::Plan &pl = t->plan;
  const std::vector<int32_t> *arrays[kPlanArrays] = {
      &pl.prefix_items, &pl.suffix_items, &pl.pg_rec, &pl.qt_rec,
      &pl.part_indptr, &pl.part_base,    &pl.part_hstride, &pl.merge_qt,
      &pl.coop_items[0], &pl.coop_items[1], &pl.coop_items[2],
      &pl.walk_items, &pl.walk_blocks, &pl.walk_qt, &pl.qt_mask};
  size_t total = 0;
  for (int i = 0; i < kPlanArrays; ++i) {
    t->blob_off[i] = total;
    t->blob_ints[i] = arrays[i]->size();
    total += align_up(arrays[i]->size() * sizeof(int32_t) + 16, 256);
  }
  const spex_status_t rs = stage_reserve(t, total);
  if (rs != SPEX_OK) return rs;
  if (total > t->d_plan_cap) {
    if (t->d_plan) HIP_TRY(hipFree(t->d_plan));
    t->d_plan = nullptr;
    t->d_plan_cap = 0;
    // Freeing and allocating device memory synchronises the device, so the workspace grows in
    // large steps: at least 1 MiB, and twice what is needed now.
    const size_t cap = align_up(std::max<size_t>(2 * total, size_t(1) << 20), 1 << 16);
    HIP_TRY(hipMalloc(&t->d_plan, cap));
    t->d_plan_cap = cap;
  }
  char *h = static_cast<char *>(t->h_stage);
  for (int i = 0; i < kPlanArrays; ++i)
    if (!arrays[i]->empty())
      std::memcpy(h + t->blob_off[i], arrays[i]->data(), arrays[i]->size() * sizeof(int32_t));
  const spex_status_t ss = stage_send(t, t->d_plan, total, stream);
  if (ss != SPEX_OK) return ss;
  const char *d = static_cast<const char *>(t->d_plan);
  auto at = [&](int i) { return reinterpret_cast<const int32_t *>(d + t->blob_off[i]); };
  DevicePlan &dp = t->dplan;
  dp.prefix_items = at(0);
  dp.suffix_items = at(1);
  dp.pg_rec = at(2);
  dp.qt_rec = at(3);
  dp.part_indptr = at(4);
  dp.part_base = at(5);
  dp.part_hstride = at(6);
  dp.merge_qt = at(7);
  for (int c = 0; c < 3; ++c) dp.coop_items[c] = at(8 + c);
  dp.walk_items = at(11);
  dp.walk_blocks = at(12);
  dp.walk_qt = at(13);
  dp.qt_mask = pl.qt_mask.empty() ? nullptr : at(14);
  t->plan_on_device = true;
  t->device_has_split = pl.has_split;
  t->device_has_walk = pl.has_walk;
  t->pending_patches.clear();
  return SPEX_OK;
}

// Applies the pending length patches to the device copy of the plan with one small kernel.
spex_status_t send_patches(spex_tree *t, hipStream_t stream) {
  std::vector<int32_t> &pp = t->pending_patches;
  const size_t n_in = pp.size() / 3;
  const spex_status_t rs = stage_reserve(t, n_in * 2 * sizeof(int32_t));
  if (rs != SPEX_OK) return rs;
  int32_t *h = static_cast<int32_t *>(t->h_stage);
  size_t n = 0;
  for (size_t i = 0; i < n_in; ++i) {
    const int arr = kPatchTarget[pp[3 * i]];
    const size_t idx = static_cast<size_t>(pp[3 * i + 1]);
    if (idx >= t->blob_ints[arr]) continue;  // that list is not on the device
    h[2 * n] = static_cast<int32_t>(t->blob_off[arr] / sizeof(int32_t) + idx);
    h[2 * n + 1] = pp[3 * i + 2];
    ++n;
  }
  pp.clear();
  if (n == 0) return SPEX_OK;
  const size_t bytes = n * 2 * sizeof(int32_t);
  if (bytes > t->d_patch_cap) {
    if (t->d_patch) HIP_TRY(hipFree(t->d_patch));
    t->d_patch = nullptr;
    t->d_patch_cap = 0;
    const size_t cap = align_up(bytes + bytes / 2, 1 << 16);
    HIP_TRY(hipMalloc(&t->d_patch, cap));
    t->d_patch_cap = cap;
  }
  const spex_status_t ss = stage_send(t, t->d_patch, bytes, stream);
  if (ss != SPEX_OK) return ss;
  HIP_TRY(spex::launch_patch(static_cast<int32_t *>(t->d_plan), static_cast<const int32_t *>(t->d_patch),
                             static_cast<int32_t>(n), stream));
  return SPEX_OK;
}

spex_status_t ensure_partials(spex_tree *t, int64_t rows) {
  if (rows <= t->part_cap_rows) return SPEX_OK;
  if (t->d_part_o) HIP_TRY(hipFree(t->d_part_o));
  if (t->d_part_ml) HIP_TRY(hipFree(t->d_part_ml));
  t->d_part_o = t->d_part_ml = nullptr;
  t->part_cap_rows = 0;
  const int64_t cap = 2 * rows + 1024;  // grows in large steps: a reallocation synchronises the device
  HIP_TRY(hipMalloc(reinterpret_cast<void **>(&t->d_part_o),
                    static_cast<size_t>(cap) * t->cfg.head_dim * sizeof(float)));
  HIP_TRY(hipMalloc(reinterpret_cast<void **>(&t->d_part_ml), static_cast<size_t>(cap) * 2 * sizeof(float)));
  t->part_cap_rows = cap;
  return SPEX_OK;
}

// ---- device scratch of the entry point that allocates nothing ----------------------------------
// One array per GPU, held from the moment the library's code object is loaded on that GPU until
// the process ends.  Layout: the launch lists of the current call (kStaticPlanBytes), then the
// partial softmax states of the shared-prefix / suffix kernels.  In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels get the address that call returns for the
// current device.
constexpr size_t kStaticPlanBytes = size_t(16) << 20;
constexpr size_t kStaticPartBytes = size_t(48) << 20;
constexpr size_t kStaticScratchBytes = kStaticPlanBytes + kStaticPartBytes;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char *g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of the scratch array (looked up once per device).
spex_status_t static_scratch(unsigned char **out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) {
    g_last_error = "device index beyond the static scratch table";
    return SPEX_ERR_DEVICE;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) {
      g_last_error = "hipGetSymbolAddress returned no address for the static scratch";
      return SPEX_ERR_DEVICE;
    }
    g_scratch_ptr[dev] = static_cast<unsigned char *>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return SPEX_OK;
}

// Copies the lists of the current plan into the plan region of the static scratch (through a
// pageable host buffer of the handle: no pinned allocation) and fills dp with their addresses.
spex_status_t upload_plan_static(spex_tree *t, unsigned char *base, DevicePlan *dp, hipStream_t stream) {
  const spex::Plan &pl = t->plan;
  const std::vector<int32_t> *arrays[kPlanArrays] = {
      &pl.prefix_items, &pl.suffix_items, &pl.pg_rec, &pl.qt_rec,
      &pl.part_indptr, &pl.part_base,    &pl.part_hstride, &pl.merge_qt,
      &pl.coop_items[0], &pl.coop_items[1], &pl.coop_items[2],
      &pl.walk_items, &pl.walk_blocks, &pl.walk_qt, &pl.qt_mask};
  size_t off[kPlanArrays], total = 0;
  for (int i = 0; i < kPlanArrays; ++i) {
    off[i] = total;
    total += align_up(arrays[i]->size() * sizeof(int32_t) + 16, 256);
  }
  if (total > kStaticPlanBytes) return SPEX_ERR_CAPACITY;
  std::vector<char> &h = t->static_stage;
  if (h.size() < total) h.resize(total);
  for (int i = 0; i < kPlanArrays; ++i)
    if (!arrays[i]->empty()) std::memcpy(h.data() + off[i], arrays[i]->data(), arrays[i]->size() * sizeof(int32_t));
  HIP_TRY(hipMemcpyAsync(base, h.data(), total, hipMemcpyHostToDevice, stream));
  auto at = [&](int i) { return reinterpret_cast<const int32_t *>(base + off[i]); };
  dp->prefix_items = at(0);
  dp->suffix_items = at(1);
  dp->pg_rec = at(2);
  dp->qt_rec = at(3);
  dp->part_indptr = at(4);
  dp->part_base = at(5);
  dp->part_hstride = at(6);
  dp->merge_qt = at(7);
  for (int c = 0; c < 3; ++c) dp->coop_items[c] = at(8 + c);
  dp->walk_items = at(11);
  dp->walk_blocks = at(12);
  dp->walk_qt = at(13);
  dp->qt_mask = pl.qt_mask.empty() ? nullptr : at(14);
  return SPEX_OK;
}

}  // namespace

extern "C" {

const char *spex_status_string(spex_status_t s) {
  switch (s) {
    case SPEX_OK: return "ok";
    case SPEX_ERR_INVALID_ARG: return "invalid argument";
    case SPEX_ERR_BAD_NODE: return "unknown or pruned node";
    case SPEX_ERR_NOT_LEAF: return "node has live children";
    case SPEX_ERR_OOM_PAGES: return "page pool exhausted";
    case SPEX_ERR_EMPTY_PATH: return "path shorter than the number of queries";
    case SPEX_ERR_UNSUPPORTED: return "unsupported dtype or shape";
    case SPEX_ERR_DEVICE: return "HIP error";
    case SPEX_ERR_CAPACITY: return "output array too small";
  }
  return "unknown status";
}

const char *spex_last_device_error(void) { return g_last_error.c_str(); }

spex_status_t spex_pool_bytes(const spex_config_t *cfg, size_t *bytes_per_pool) {
  if (!cfg || !bytes_per_pool) return SPEX_ERR_INVALID_ARG;
  if (cfg->num_pages < 0 || cfg->num_kv_heads <= 0 || cfg->page_size <= 0 || cfg->head_dim <= 0 ||
      cfg->kv_dtype < 0 || cfg->kv_dtype > 2)
    return SPEX_ERR_INVALID_ARG;
  const size_t tiles = cfg->page_stride_tiles ? cfg->page_stride_tiles : cfg->num_kv_heads;
  const size_t tile_bytes = static_cast<size_t>(cfg->page_size) * cfg->head_dim * elem_size(cfg->kv_dtype);
  // A strided pool ends with the last page's own tiles, not with a full stride.
  *bytes_per_pool = cfg->num_pages == 0 ? 0
                                        : (static_cast<size_t>(cfg->num_pages - 1) * tiles +
                                           cfg->num_kv_heads) * tile_bytes;
  return SPEX_OK;
}

spex_status_t spex_tree_create(const spex_config_t *cfg, spex_tree_t **out) {
  if (!out) return SPEX_ERR_INVALID_ARG;
  const spex_status_t st = check_config(cfg);
  if (st != SPEX_OK) return st;
  if (cfg->free_order) {
    std::vector<char> seen(static_cast<size_t>(cfg->num_pages), 0);
    for (int64_t i = 0; i < cfg->num_pages; ++i) {
      const int32_t p = cfg->free_order[i];
      if (p < 0 || p >= cfg->num_pages || seen[p]) return SPEX_ERR_INVALID_ARG;
      seen[p] = 1;
    }
  }
  spex_tree *t = new (std::nothrow) spex_tree();
  if (!t) return SPEX_ERR_INVALID_ARG;
  t->cfg = *cfg;
  t->shape = make_shape(*cfg);
  t->pt = new (std::nothrow) spex::PageTable(cfg->num_pages, cfg->page_size, cfg->free_order);
  if (!t->pt) {
    delete t;
    return SPEX_ERR_INVALID_ARG;
  }
  t->cfg.free_order = nullptr;
  t->prefix_chunk = cfg->prefix_chunk_pages;
  t->suffix_chunk = cfg->suffix_chunk_pages;
  t->kernel_mode = cfg->kernel_mode;
  t->walk_row_tiles = cfg->walk_row_tiles;
  t->walk_waves = cfg->walk_waves;
  *out = t;
  return SPEX_OK;
}

void spex_tree_destroy(spex_tree_t *t) {
  if (!t) return;
  const bool used_device = t->d_plan || t->d_part_o || t->stage[0].h || t->stage[1].h || !t->prof.empty();
  if (used_device) (void)hipDeviceSynchronize();
  if (t->d_plan) (void)hipFree(t->d_plan);
  if (t->d_patch) (void)hipFree(t->d_patch);
  if (t->d_part_o) (void)hipFree(t->d_part_o);
  if (t->d_part_ml) (void)hipFree(t->d_part_ml);
  for (spex_tree::Stage &st : t->stage) {
    if (st.h) (void)hipHostFree(st.h);
    if (st.event) (void)hipEventDestroy(st.event);
  }
  for (auto &slot : t->prof)
    for (hipEvent_t e : slot.ev)
      if (e) (void)hipEventDestroy(e);
  delete t->pt;
  delete t;
}

spex_status_t spex_tree_fork(spex_tree_t *t, spex_node_t parent, int32_t n_children,
                             spex_node_t *out_children) {
  if (!t || n_children < 0 || (n_children > 0 && !out_children)) return SPEX_ERR_INVALID_ARG;
  if (parent != SPEX_NO_NODE && !t->pt->valid(parent)) return SPEX_ERR_BAD_NODE;
  if (static_cast<int64_t>(t->pt->num_nodes()) + n_children > INT32_MAX) return SPEX_ERR_UNSUPPORTED;
  if (n_children == 0) return SPEX_OK;
  const int32_t first = t->pt->fork(parent, n_children);
  for (int32_t i = 0; i < n_children; ++i) out_children[i] = first + i;
  return SPEX_OK;
}

spex_status_t spex_tree_append_new_pages(const spex_tree_t *t, spex_node_t node, int32_t n_tokens,
                                         int32_t *n_new_pages) {
  if (!t || !n_new_pages || n_tokens < 0) return SPEX_ERR_INVALID_ARG;
  if (!t->pt->valid(node)) return SPEX_ERR_BAD_NODE;
  *n_new_pages = t->pt->new_pages_needed(node, n_tokens);
  return SPEX_OK;
}

static spex_status_t append_step_impl(spex_tree_t *t, spex_node_t node, int32_t n_tokens, const void *k,
                                      const void *v, const float *k_scales, const float *v_scales,
                                      void *hip_stream, bool quantise) {
  if (!t || n_tokens < 0 || ((k == nullptr) != (v == nullptr))) return SPEX_ERR_INVALID_ARG;
  if (quantise && t->cfg.kv_dtype != SPEX_FP8_E4M3) return SPEX_ERR_UNSUPPORTED;
  if (!t->pt->valid(node)) return SPEX_ERR_BAD_NODE;
  if (t->pt->node(node).n_live_children > 0) return SPEX_ERR_NOT_LEAF;
  if (k && !t->cfg.k_pool) return SPEX_ERR_INVALID_ARG;
  if (n_tokens == 0) return SPEX_OK;
  const int32_t P = t->cfg.page_size;
  const int32_t old_tokens = t->pt->node(node).n_tokens;
  if (static_cast<int64_t>(old_tokens) + n_tokens > INT32_MAX / 2) return SPEX_ERR_UNSUPPORTED;
  const int32_t need = t->pt->new_pages_needed(node, n_tokens);
  if (k && !quantise && t->cfg.kv_dtype == SPEX_FP8_E4M3 && need > 0 && (!k_scales || !v_scales))
    return SPEX_ERR_INVALID_ARG;
  int32_t first_new = 0;
  if (!t->pt->append(node, n_tokens, &first_new)) return SPEX_ERR_OOM_PAGES;
  if (!k) return SPEX_OK;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const spex::Node &nd = t->pt->node(node);
  const int32_t new_total = old_tokens + n_tokens;
  const int32_t page_lo = old_tokens / P;  // first page written (continuing or new)
  const int32_t page_hi = (new_total + P - 1) / P;
  const size_t tok_bytes = static_cast<size_t>(t->cfg.num_kv_heads) * t->cfg.head_dim *
                           (quantise ? sizeof(uint16_t) : elem_size(t->cfg.kv_dtype));
  for (int32_t pa = page_lo; pa < page_hi; pa += spex::kMaxPagesPerScatter) {
    const int32_t pb = pa + spex::kMaxPagesPerScatter < page_hi ? pa + spex::kMaxPagesPerScatter : page_hi;
    spex::ScatterArgs a{};
    a.k_pool = t->cfg.k_pool;
    a.v_pool = t->cfg.v_pool;
    a.k_scale = t->cfg.k_scale;
    a.v_scale = t->cfg.v_scale;
    const int32_t tok_a = old_tokens > pa * P ? old_tokens : pa * P;
    const int32_t tok_b = new_total < pb * P ? new_total : pb * P;
    a.k_src = static_cast<const char *>(k) + static_cast<size_t>(tok_a - old_tokens) * tok_bytes;
    a.v_src = static_cast<const char *>(v) + static_cast<size_t>(tok_a - old_tokens) * tok_bytes;
    a.n_pages = pb - pa;
    a.first_slot = tok_a - pa * P;
    a.n_tokens = tok_b - tok_a;
    a.first_page_is_new = pa >= first_new ? 1 : 0;
    const int32_t first_new_in_launch = a.first_page_is_new ? pa : pa + 1;
    if (k_scales) {
      a.k_scale_src = k_scales + static_cast<size_t>(first_new_in_launch - first_new) * t->cfg.num_kv_heads;
      a.v_scale_src = v_scales + static_cast<size_t>(first_new_in_launch - first_new) * t->cfg.num_kv_heads;
    }
    for (int32_t i = 0; i < a.n_pages; ++i) a.page_ids[i] = nd.pages[pa + i];
    HIP_TRY(quantise ? spex::launch_scatter_quantise(t->shape, a, stream)
                     : spex::launch_scatter(t->shape, a, stream));
  }
  return SPEX_OK;
}

spex_status_t spex_tree_append_step(spex_tree_t *t, spex_node_t node, int32_t n_tokens,
                                    const void *k, const void *v, const float *k_scales,
                                    const float *v_scales, void *hip_stream) {
  return append_step_impl(t, node, n_tokens, k, v, k_scales, v_scales, hip_stream, false);
}

spex_status_t spex_tree_append_step_quantize(spex_tree_t *t, spex_node_t node, int32_t n_tokens,
                                             const void *k, const void *v, void *hip_stream) {
  return append_step_impl(t, node, n_tokens, k, v, nullptr, nullptr, hip_stream, true);
}

static spex_status_t append_tokens_impl(spex_tree_t *t, const spex_node_t *nodes, int32_t n_nodes,
                                        const void *k, const void *v, const float *k_scales,
                                        const float *v_scales, void *hip_stream, bool quantise) {
  if (!t || n_nodes < 0 || (n_nodes > 0 && !nodes) || ((k == nullptr) != (v == nullptr)))
    return SPEX_ERR_INVALID_ARG;
  if (quantise && t->cfg.kv_dtype != SPEX_FP8_E4M3) return SPEX_ERR_UNSUPPORTED;
  if (k && !t->cfg.k_pool) return SPEX_ERR_INVALID_ARG;
  if (n_nodes == 0) return SPEX_OK;
  // Check everything before touching the table: the call is all or nothing.
  const int32_t P = t->cfg.page_size;
  int64_t need = 0;
  std::vector<int32_t> sorted(nodes, nodes + n_nodes);
  std::sort(sorted.begin(), sorted.end());
  for (int32_t i = 0; i < n_nodes; ++i) {
    const int32_t u = sorted[i];
    if (!t->pt->valid(u)) return SPEX_ERR_BAD_NODE;
    if (i > 0 && sorted[i - 1] == u) return SPEX_ERR_INVALID_ARG;
    if (t->pt->node(u).n_live_children > 0) return SPEX_ERR_NOT_LEAF;
    if (t->pt->node(u).n_tokens >= INT32_MAX / 2) return SPEX_ERR_UNSUPPORTED;
    need += t->pt->new_pages_needed(u, 1);
  }
  if (need > t->pt->free_pages()) return SPEX_ERR_OOM_PAGES;
  if (k && t->cfg.kv_dtype == SPEX_FP8_E4M3 && need > 0 && (!k_scales || !v_scales))
    return SPEX_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // Staging holds the destination list and, behind it, the length patches of the cached plan that
  // this launch applies as well.  Room for 32 patches per node is reserved before anything
  // changes (a block started in the tree-walk lists takes 8 + one per kv head, each query token
  // one or two); if a plan needs more, its patches wait for the next decode_attention call instead.
  const size_t dst_ints = static_cast<size_t>(n_nodes) * 2;
  const size_t patch_room = static_cast<size_t>(n_nodes) * 32;  // {index, value} pairs
  const size_t bytes_max = (dst_ints + 2 * patch_room) * sizeof(int32_t);
  int32_t *h = nullptr;
  if (k) {
    const spex_status_t rs = stage_reserve(t, bytes_max);
    if (rs != SPEX_OK) return rs;
    if (bytes_max > t->d_patch_cap) {
      if (t->d_patch) HIP_TRY(hipFree(t->d_patch));
      t->d_patch = nullptr;
      t->d_patch_cap = 0;
      const size_t cap = align_up(bytes_max + bytes_max / 2, 1 << 16);
      HIP_TRY(hipMalloc(&t->d_patch, cap));
      t->d_patch_cap = cap;
    }
    h = static_cast<int32_t *>(t->h_stage);
  }
  for (int32_t i = 0; i < n_nodes; ++i) {
    const int32_t u = nodes[i];
    const int32_t old_tokens = t->pt->node(u).n_tokens;
    int32_t first_new = 0;
    t->pt->append(u, 1, &first_new);  // cannot fail: the pages were counted above
    if (h) {
      const spex::Node &nd = t->pt->node(u);
      const int32_t pi = old_tokens / P;
      h[2 * i] = nd.pages[pi];
      h[2 * i + 1] = (old_tokens % P) | ((pi >= first_new ? 1 : 0) << 8);
    }
  }
  if (!k) return SPEX_OK;
  // The cached plan, if its copy is on the device and nothing else is waiting for it, follows the
  // append right here: same request next time means no planning and no separate patch launch.
  size_t n_patch = 0;
  if (t->plan.valid && t->plan_on_device && t->pending_patches.empty() &&
      t->plan.table_version != t->pt->version()) {
    std::vector<int32_t> &pp = t->pending_patches;
    if (t->planner.patch_lengths(*t->pt, &t->plan, &pp)) {
      int32_t *hp = h + dst_ints;
      bool fits = true;
      for (size_t i = 0; i < pp.size() / 3 && fits; ++i) {
        const int arr = kPatchTarget[pp[3 * i]];
        const size_t idx = static_cast<size_t>(pp[3 * i + 1]);
        if (idx >= t->blob_ints[arr]) continue;  // that list is not on the device
        if (n_patch == patch_room) {
          fits = false;
          break;
        }
        hp[2 * n_patch] = static_cast<int32_t>(t->blob_off[arr] / sizeof(int32_t) + idx);
        hp[2 * n_patch + 1] = pp[3 * i + 2];
        ++n_patch;
      }
      if (fits && n_patch <= static_cast<size_t>(n_nodes) * t->cfg.num_kv_heads * t->cfg.head_dim) {
        pp.clear();
        t->plan_patched_by_append = true;
      } else {
        n_patch = 0;  // too many for this launch: decode_attention sends them
      }
    } else {
      // The lists cannot follow this append (and may be half changed): drop the plan, so that the
      // next call plans afresh instead of trying the same patch again on arrays already touched.
      pp.clear();
      t->plan.valid = false;
      t->plan_on_device = false;
    }
  }
  const size_t bytes = (dst_ints + 2 * n_patch) * sizeof(int32_t);
  const spex_status_t ss = stage_send(t, t->d_patch, bytes, stream);
  if (ss != SPEX_OK) return ss;
  spex::AppendTokensArgs a{};
  a.k_pool = t->cfg.k_pool;
  a.v_pool = t->cfg.v_pool;
  a.k_scale = t->cfg.k_scale;
  a.v_scale = t->cfg.v_scale;
  a.k_src = k;
  a.v_src = v;
  a.k_scale_src = k_scales;
  a.v_scale_src = v_scales;
  a.dst = static_cast<const int32_t *>(t->d_patch);
  a.n_nodes = n_nodes;
  a.quantise = quantise;
  a.plan = static_cast<int32_t *>(t->d_plan);
  a.patches = static_cast<const int32_t *>(t->d_patch) + dst_ints;
  a.n_patches = static_cast<int32_t>(n_patch);
  HIP_TRY(spex::launch_append_tokens(t->shape, a, stream));
  return SPEX_OK;
}

spex_status_t spex_tree_append_tokens(spex_tree_t *t, const spex_node_t *nodes, int32_t n_nodes,
                                      const void *k, const void *v, const float *k_scales,
                                      const float *v_scales, void *hip_stream) {
  return append_tokens_impl(t, nodes, n_nodes, k, v, k_scales, v_scales, hip_stream, false);
}

spex_status_t spex_tree_append_tokens_quantize(spex_tree_t *t, const spex_node_t *nodes, int32_t n_nodes,
                                               const void *k, const void *v, const float *k_scales,
                                               const float *v_scales, void *hip_stream) {
  return append_tokens_impl(t, nodes, n_nodes, k, v, k_scales, v_scales, hip_stream, true);
}

spex_status_t spex_tree_prune(spex_tree_t *t, spex_node_t node) {
  if (!t) return SPEX_ERR_INVALID_ARG;
  if (!t->pt->valid(node)) return SPEX_ERR_BAD_NODE;
  t->pt->prune(node);
  return SPEX_OK;
}

static spex_status_t decode_attention_impl(spex_tree_t *t, const spex_node_t *leaves, const int32_t *q_lens,
                                           const uint32_t *draft_masks, int32_t n_leaves, const void *q,
                                           float *out, float *lse, float sm_scale, void *hip_stream,
                                           bool use_static);

spex_status_t spex_tree_decode_attention(spex_tree_t *t, const spex_node_t *leaves,
                                         const int32_t *q_lens, int32_t n_leaves, const void *q,
                                         float *out, float *lse, float sm_scale, void *hip_stream) {
  return spex_tree_decode_attention_masked(t, leaves, q_lens, nullptr, n_leaves, q, out, lse, sm_scale,
                                           hip_stream);
}

spex_status_t spex_tree_decode_attention_masked(spex_tree_t *t, const spex_node_t *leaves,
                                                const int32_t *q_lens, const uint32_t *draft_masks,
                                                int32_t n_leaves, const void *q, float *out, float *lse,
                                                float sm_scale, void *hip_stream) {
  return decode_attention_impl(t, leaves, q_lens, draft_masks, n_leaves, q, out, lse, sm_scale, hip_stream,
                               false);
}

spex_status_t spex_tree_decode_attention_static(spex_tree_t *t, const spex_node_t *leaves,
                                                const int32_t *q_lens, int32_t n_leaves, const void *q,
                                                float *out, float *lse, float sm_scale, void *hip_stream) {
  return decode_attention_impl(t, leaves, q_lens, nullptr, n_leaves, q, out, lse, sm_scale, hip_stream, true);
}

static spex_status_t decode_attention_impl(spex_tree_t *t, const spex_node_t *leaves, const int32_t *q_lens,
                                           const uint32_t *draft_masks, int32_t n_leaves, const void *q,
                                           float *out, float *lse, float sm_scale, void *hip_stream,
                                           bool use_static) {
  if (!t || n_leaves < 0 || (n_leaves > 0 && (!leaves || !q || !out))) return SPEX_ERR_INVALID_ARG;
  if (!t->cfg.k_pool) return SPEX_ERR_INVALID_ARG;
  if (!(sm_scale > 0.f) || std::isinf(sm_scale)) return SPEX_ERR_INVALID_ARG;
  if (n_leaves == 0) return SPEX_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int plan_state = 0;
  if (draft_masks && !q_lens) return SPEX_ERR_INVALID_ARG;
  const spex_status_t st = make_plan(t, leaves, q_lens, draft_masks, n_leaves, &plan_state);
  if (st != SPEX_OK) return st;
  spex::Plan &pl = t->plan;
  // Which kernels: the tree-walk kernel when its lists exist and fill the chip, or when its
  // longest workgroup is short; else shared-prefix + suffix + merge, which can split long paths.
  // A tree-walk workgroup takes about 12 us + 0.8 us per two-page block on its path whatever else
  // runs, the three split-path launches take 26-45 us for up to 32 work items of this size and
  // grow with the item count: measured crossing points were 20 blocks at 8-32 items, 40 at 64
  // and 65 at 96 (bf16, 32 / 8 heads of 128).  Only the lists of the chosen kernels are built.
  bool want_walk = (t->kernel_mode == 0 || t->kernel_mode == 3) && spex::has_mfma_kernel(t->shape);
  const bool tree_masks = draft_masks != nullptr;
  if (want_walk && t->kernel_mode == 0 && !pl.has_walk && obviously_split(pl))
    want_walk = false;  // few requests with long paths: the split path without building the other lists
  if (want_walk) t->planner.ensure_walk(*t->pt, &pl);
  // Draft-tree masks are understood by every kernel but the tree-walk kernel that splits the path
  // (walk_waves 2).
  const bool walk_possible = want_walk && pl.walk_ok && (!tree_masks || pl.walk_waves != 2);
  if (t->kernel_mode == 3 && !walk_possible) return SPEX_ERR_UNSUPPORTED;
  const int32_t short_walk = short_walk_blocks(pl.walk_real_items);
  const bool use_walk = walk_possible && (t->kernel_mode == 3 || pl.walk_real_items >= 128 ||
                                          pl.walk_max_item_blocks <= short_walk);
  if (!use_walk) {
    const spex_status_t ss = plan_status(t, t->planner.ensure_split(*t->pt, &pl));
    if (ss != SPEX_OK) return ss;
  }
  unsigned char *sbase = nullptr;
  DevicePlan static_dp;
  if (use_static) {
    // Nothing is allocated on this path: the lists go into the per-device static array (all of them,
    // every call: another handle's call may have overwritten it), partial results follow them
    // there, and no events are made.  The handle's own device copy, if any, and the patches that
    // wait for it are left as they are.
    if (!use_walk && align_up(static_cast<size_t>(pl.n_partial_rows) * t->cfg.head_dim * 4, 256) +
                             static_cast<size_t>(pl.n_partial_rows) * 8 > kStaticPartBytes)
      return SPEX_ERR_CAPACITY;
    const spex_status_t gs = static_scratch(&sbase);
    if (gs != SPEX_OK) return gs;
    const spex_status_t us = upload_plan_static(t, sbase, &static_dp, stream);
    if (us != SPEX_OK) return us;
    if (!t->plan_on_device) t->pending_patches.clear();  // no device copy is waiting for them
  } else if (!t->plan_on_device || (use_walk ? !t->device_has_walk : !t->device_has_split)) {
    const spex_status_t us = upload_plan(t, stream);
    if (us != SPEX_OK) return us;
  } else if (!t->pending_patches.empty()) {
    const spex_status_t us = send_patches(t, stream);
    if (us != SPEX_OK) return us;
  }
  const DevicePlan &dp = use_static ? static_dp : t->dplan;

  spex_tree::ProfSlot *slot = nullptr;
  if (t->profiling && !use_static) {
    if (t->prof.empty()) t->prof.resize(spex_tree::kProfSlots);
    slot = &t->prof[t->prof_calls % spex_tree::kProfSlots];
    ++t->prof_calls;
    for (hipEvent_t &e : slot->ev)
      if (!e) HIP_TRY(hipEventCreate(&e));
    for (bool &b : slot->valid) b = false;
  }
  auto bracket = [&](int which, bool begin) -> hipError_t {
    if (!slot) return hipSuccess;
    if (!begin) slot->valid[which] = true;
    return hipEventRecord(slot->ev[2 * which + (begin ? 0 : 1)], stream);
  };

  if (use_walk) {
    spex::WalkArgs wa{};
    wa.k_pool = t->cfg.k_pool;
    wa.v_pool = t->cfg.v_pool;
    wa.k_scale = t->cfg.k_scale;
    wa.v_scale = t->cfg.v_scale;
    wa.q = q;
    wa.items = dp.walk_items;
    wa.n_items = static_cast<int32_t>(pl.walk_items.size() / pl.item_ints());
    wa.blocks = dp.walk_blocks;
    wa.qt_rec = dp.walk_qt;
    wa.out = out;
    wa.lse = lse;
    wa.scale_log2 = sm_scale * 1.4426950408889634f;
    wa.qt_mask = dp.qt_mask;
    HIP_TRY(bracket(3, true));
    HIP_TRY(spex::launch_tree_walk(t->shape, wa, pl.walk_row_tiles, pl.walk_waves, stream));
    HIP_TRY(bracket(3, false));
    t->info[0] = pl.unique_tokens;
    t->info[1] = pl.prefix_tokens;
    t->info[2] = pl.suffix_tokens;
    t->info[3] = pl.walk_real_items;
    t->info[4] = pl.walk_block_visits;
    t->info[5] = 0;
    t->info[6] = plan_state;
    t->info[7] = pl.walk_row_tiles + 256 * pl.walk_waves;
    return SPEX_OK;
  }

  float *part_o = nullptr, *part_ml = nullptr;
  if (use_static) {
    part_o = reinterpret_cast<float *>(sbase + kStaticPlanBytes);
    part_ml = reinterpret_cast<float *>(
        sbase + kStaticPlanBytes + align_up(static_cast<size_t>(pl.n_partial_rows) * t->cfg.head_dim * 4, 256));
  } else {
    const spex_status_t ps = ensure_partials(t, pl.n_partial_rows);
    if (ps != SPEX_OK) return ps;
    part_o = t->d_part_o;
    part_ml = t->d_part_ml;
  }

  spex::AttnArgs a{};
  a.k_pool = t->cfg.k_pool;
  a.v_pool = t->cfg.v_pool;
  a.k_scale = t->cfg.k_scale;
  a.v_scale = t->cfg.v_scale;
  a.q = q;
  a.pg_rec = dp.pg_rec;
  a.qt_rec = dp.qt_rec;
  a.part_o = part_o;
  a.part_ml = part_ml;
  a.part_indptr = dp.part_indptr;
  a.part_base = dp.part_base;
  a.part_hstride = dp.part_hstride;
  a.out = out;
  a.lse = lse;
  a.scale_log2 = sm_scale * 1.4426950408889634f;
  a.qt_mask = dp.qt_mask;
  const bool generic = t->kernel_mode == 1;

  const int32_t n_prefix_items = static_cast<int32_t>(pl.prefix_items.size() / spex::Plan::kItemInts);
  const int32_t n_suffix_items = static_cast<int32_t>(pl.suffix_items.size() / spex::Plan::kItemInts);
  int32_t n_coop_items = 0;
  for (int c = 0; c < 3; ++c)
    n_coop_items += static_cast<int32_t>(pl.coop_items[c].size() / spex::Plan::kItemInts);
  if (n_prefix_items + n_coop_items > 0) {
    HIP_TRY(bracket(0, true));
    if (n_prefix_items > 0) {
      a.items = dp.prefix_items;
      a.n_items = n_prefix_items;
      HIP_TRY(spex::launch_attention(t->shape, a, true, pl.prefix_row_tiles, generic, stream));
    }
    for (int c = 0; c < 3; ++c) {
      a.items = dp.coop_items[c];
      a.n_items = static_cast<int32_t>(pl.coop_items[c].size() / spex::Plan::kItemInts);
      if (a.n_items == 0) continue;
      if (generic || !spex::has_mfma_kernel(t->shape))  // generic kernels take any row count
        HIP_TRY(spex::launch_attention(t->shape, a, true, 4 << c, true, stream));
      else
        HIP_TRY(spex::launch_prefix_coop(t->shape, a, 1 << c, stream));
    }
    HIP_TRY(bracket(0, false));
  }
  if (n_suffix_items > 0) {
    a.items = dp.suffix_items;
    a.n_items = n_suffix_items;
    HIP_TRY(bracket(1, true));
    HIP_TRY(spex::launch_attention(t->shape, a, false, pl.suffix_row_tiles, generic, stream));
    HIP_TRY(bracket(1, false));
  }
  spex::MergeArgs m{};
  m.part_indptr = dp.part_indptr;
  m.part_base = dp.part_base;
  m.part_hstride = dp.part_hstride;
  m.part_o = part_o;
  m.part_ml = part_ml;
  m.out = out;
  m.lse = lse;
  // The MFMA suffix kernel finishes the rows of single-chunk suffixes itself; the generic kernels
  // leave every row to the merge kernel.
  const bool fused = !generic && spex::has_mfma_kernel(t->shape);
  m.qt_ids = fused ? dp.merge_qt : nullptr;
  m.n_qtok = fused ? static_cast<int32_t>(pl.merge_qt.size())
                   : static_cast<int32_t>(pl.qt_limit.size());
  HIP_TRY(bracket(2, true));
  HIP_TRY(spex::launch_merge(t->shape, m, stream));
  HIP_TRY(bracket(2, false));

  t->info[0] = pl.unique_tokens;
  t->info[1] = pl.prefix_tokens;
  t->info[2] = pl.suffix_tokens;
  t->info[3] = n_prefix_items + n_coop_items;
  t->info[4] = n_suffix_items;
  t->info[5] = pl.n_partial_rows;
  t->info[6] = plan_state;
  t->info[7] = 0;
  return SPEX_OK;
}

spex_status_t spex_tree_node_info(const spex_tree_t *t, spex_node_t node, spex_node_info_t *out) {
  if (!t || !out) return SPEX_ERR_INVALID_ARG;
  if (!t->pt->valid(node)) return SPEX_ERR_BAD_NODE;
  const spex::Node &nd = t->pt->node(node);
  out->parent = nd.parent;
  out->n_tokens = nd.n_tokens;
  out->n_pages = static_cast<int32_t>(nd.pages.size());
  out->n_live_children = nd.n_live_children;
  return SPEX_OK;
}

spex_status_t spex_tree_path_pages(const spex_tree_t *t, spex_node_t node, int32_t *pages,
                                   int32_t *valid, int32_t cap, int32_t *n) {
  if (!t || !n || cap < 0 || (cap > 0 && (!pages || !valid))) return SPEX_ERR_INVALID_ARG;
  if (!t->pt->valid(node)) return SPEX_ERR_BAD_NODE;
  std::vector<int32_t> chain;
  int64_t total = 0;
  for (int32_t u = node; u != spex::kNoNode; u = t->pt->node(u).parent) {
    chain.push_back(u);
    total += static_cast<int64_t>(t->pt->node(u).pages.size());
  }
  *n = static_cast<int32_t>(total);
  if (total > cap) return SPEX_ERR_CAPACITY;
  int32_t w = 0;
  for (auto it = chain.rbegin(); it != chain.rend(); ++it) {
    const spex::Node &nd = t->pt->node(*it);
    for (size_t i = 0; i < nd.pages.size(); ++i) {
      pages[w] = nd.pages[i];
      valid[w] = t->pt->page_valid(*it, static_cast<int32_t>(i));
      ++w;
    }
  }
  return SPEX_OK;
}

spex_status_t spex_tree_free_pages(const spex_tree_t *t, int32_t *pages, int32_t cap, int32_t *n) {
  if (!t || !n || cap < 0 || (cap > 0 && !pages)) return SPEX_ERR_INVALID_ARG;
  const std::vector<int32_t> fl = t->pt->free_list();
  *n = static_cast<int32_t>(fl.size());
  if (static_cast<int64_t>(fl.size()) > cap) return SPEX_ERR_CAPACITY;
  if (!fl.empty()) std::memcpy(pages, fl.data(), fl.size() * sizeof(int32_t));
  return SPEX_OK;
}

spex_status_t spex_tree_path_kv_bytes(const spex_tree_t *t, spex_node_t node, double *bytes) {
  if (!t || !bytes) return SPEX_ERR_INVALID_ARG;
  if (!t->pt->valid(node)) return SPEX_ERR_BAD_NODE;
  int64_t tokens = 0, pages = 0;
  for (int32_t u = node; u != spex::kNoNode; u = t->pt->node(u).parent) {
    tokens += t->pt->node(u).n_tokens;
    pages += static_cast<int64_t>(t->pt->node(u).pages.size());
  }
  double b = static_cast<double>(tokens) * 2.0 * t->cfg.num_kv_heads * t->cfg.head_dim *
             static_cast<double>(elem_size(t->cfg.kv_dtype));
  if (t->cfg.kv_dtype == SPEX_FP8_E4M3) b += static_cast<double>(pages) * 8.0 * t->cfg.num_kv_heads;
  *bytes = b;
  return SPEX_OK;
}

spex_status_t spex_tree_stats(const spex_tree_t *t, int64_t *live_nodes, int64_t *used_pages,
                              int64_t *free_pages) {
  if (!t) return SPEX_ERR_INVALID_ARG;
  if (live_nodes) *live_nodes = t->pt->live_nodes();
  if (used_pages) *used_pages = t->pt->used_pages();
  if (free_pages) *free_pages = t->pt->free_pages();
  return SPEX_OK;
}

spex_status_t spex_tree_plan_dump(spex_tree_t *t, const spex_node_t *leaves, const int32_t *q_lens,
                                  int32_t n_leaves, spex_plan_view_t *out) {
  if (!t || !out || n_leaves < 0 || (n_leaves > 0 && !leaves)) return SPEX_ERR_INVALID_ARG;
  int plan_state = 0;
  const spex_status_t st = make_plan(t, leaves, q_lens, nullptr, n_leaves, &plan_state);
  if (st != SPEX_OK) return st;
  t->planner.ensure_csr(*t->pt, &t->plan);
  const spex_status_t ss = plan_status(t, t->planner.ensure_split(*t->pt, &t->plan));
  if (ss != SPEX_OK) return ss;
  const spex::Plan &pl = t->plan;
  spex_plan_view_t v{};
  v.n_leaves = n_leaves;
  v.n_qtok = static_cast<int32_t>(pl.qt_limit.size());
  v.n_groups = static_cast<int32_t>(pl.group_node.size());
  v.n_tasks = static_cast<int32_t>(pl.task_pbase.size());
  v.n_prefix_tasks = pl.n_prefix_tasks;
  v.n_pg = static_cast<int32_t>(pl.pg_id.size());
  v.n_qt_list = static_cast<int32_t>(pl.qt_list.size());
  v.n_parts = static_cast<int32_t>(pl.part_base.size());
  v.n_partial_rows = pl.n_partial_rows;
  v.prefix_chunk_pages = pl.prefix_chunk_pages;
  v.suffix_chunk_pages = pl.suffix_chunk_pages;
  v.leaf_indptr = pl.leaf_indptr.data();
  v.leaf_pages = pl.leaf_pages.data();
  v.leaf_valid = pl.leaf_valid.data();
  v.qt_limit = pl.qt_limit.data();
  v.group_node = pl.group_node.data();
  v.task_pg_begin = pl.task_pg_begin.data();
  v.task_pg_count = pl.task_pg_count.data();
  v.task_qt_begin = pl.task_qt_begin.data();
  v.task_qt_count = pl.task_qt_count.data();
  v.task_pbase = pl.task_pbase.data();
  v.task_flags = pl.task_flags.data();
  v.pg_id = pl.pg_id.data();
  v.pg_valid = pl.pg_valid.data();
  v.pg_pos = pl.pg_pos.data();
  v.qt_list = pl.qt_list.data();
  v.part_indptr = pl.part_indptr.data();
  v.part_base = pl.part_base.data();
  v.part_hstride = pl.part_hstride.data();
  v.n_merge_qt = static_cast<int32_t>(pl.merge_qt.size());
  v.merge_qt = pl.merge_qt.data();
  *out = v;
  return SPEX_OK;
}

spex_status_t spex_tree_gather_kv(spex_tree_t *t, spex_node_t node, int32_t first, int32_t n,
                                  void *k_out, void *v_out, float *k_scale_out, float *v_scale_out,
                                  void *hip_stream) {
  if (!t || first < 0 || n < 0 || (n > 0 && (!k_out || !v_out))) return SPEX_ERR_INVALID_ARG;
  if (!t->pt->valid(node)) return SPEX_ERR_BAD_NODE;
  if (!t->cfg.k_pool) return SPEX_ERR_INVALID_ARG;
  const spex::Node &nd = t->pt->node(node);
  if (static_cast<int64_t>(first) + n > nd.n_tokens) return SPEX_ERR_INVALID_ARG;
  if (n == 0) return SPEX_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int32_t P = t->cfg.page_size;
  const size_t tok_bytes = static_cast<size_t>(t->cfg.num_kv_heads) * t->cfg.head_dim *
                           elem_size(t->cfg.kv_dtype);
  const int32_t page_lo = first / P, page_hi = (first + n + P - 1) / P;
  for (int32_t pa = page_lo; pa < page_hi; pa += spex::kMaxPagesPerScatter) {
    const int32_t pb = pa + spex::kMaxPagesPerScatter < page_hi ? pa + spex::kMaxPagesPerScatter : page_hi;
    spex::GatherArgs a{};
    a.k_pool = t->cfg.k_pool;
    a.v_pool = t->cfg.v_pool;
    a.k_scale = t->cfg.k_scale;
    a.v_scale = t->cfg.v_scale;
    const int32_t tok_a = first > pa * P ? first : pa * P;
    const int32_t tok_b = first + n < pb * P ? first + n : pb * P;
    const size_t done = static_cast<size_t>(tok_a - first);
    a.k_out = static_cast<char *>(k_out) + done * tok_bytes;
    a.v_out = static_cast<char *>(v_out) + done * tok_bytes;
    a.k_scale_out = k_scale_out ? k_scale_out + done * t->cfg.num_kv_heads : nullptr;
    a.v_scale_out = v_scale_out ? v_scale_out + done * t->cfg.num_kv_heads : nullptr;
    a.n_pages = pb - pa;
    a.first_slot = tok_a - pa * P;
    a.n_tokens = tok_b - tok_a;
    for (int32_t i = 0; i < a.n_pages; ++i) a.page_ids[i] = nd.pages[pa + i];
    HIP_TRY(spex::launch_gather(t->shape, a, stream));
  }
  return SPEX_OK;
}

spex_status_t spex_tree_set_tuning(spex_tree_t *t, int32_t prefix_chunk_pages,
                                   int32_t suffix_chunk_pages, int32_t kernel_mode,
                                   int32_t walk_row_tiles, int32_t walk_waves) {
  if (!t || prefix_chunk_pages < 0 || suffix_chunk_pages < 0 || kernel_mode < 0 || kernel_mode > 3 ||
      (walk_row_tiles != 0 && walk_row_tiles != 1 && walk_row_tiles != 2 && walk_row_tiles != 4) ||
      (walk_waves != 0 && walk_waves != 2 && walk_waves != 4 && walk_waves != 8))
    return SPEX_ERR_INVALID_ARG;
  t->prefix_chunk = prefix_chunk_pages;
  t->suffix_chunk = suffix_chunk_pages;
  t->kernel_mode = kernel_mode;
  t->walk_row_tiles = walk_row_tiles;
  t->walk_waves = walk_waves;
  return SPEX_OK;
}

spex_status_t spex_tree_walk_dump(spex_tree_t *t, const spex_node_t *leaves, const int32_t *q_lens,
                                  const uint32_t *draft_masks, int32_t n_leaves, spex_walk_view_t *out) {
  if (!t || !out || n_leaves < 0 || (n_leaves > 0 && !leaves)) return SPEX_ERR_INVALID_ARG;
  if (draft_masks && !q_lens) return SPEX_ERR_INVALID_ARG;
  int plan_state = 0;
  const spex_status_t st = make_plan(t, leaves, q_lens, draft_masks, n_leaves, &plan_state);
  if (st != SPEX_OK) return st;
  t->planner.ensure_walk(*t->pt, &t->plan);
  const spex::Plan &pl = t->plan;
  spex_walk_view_t v{};
  v.available = pl.walk_ok ? 1 : 0;
  v.row_tiles = pl.walk_row_tiles;
  v.waves = pl.walk_waves;
  v.plan_state = plan_state;
  v.n_row_blocks = pl.walk_ok ? static_cast<int32_t>(pl.walk_rb.size() / pl.rb_ints()) : 0;
  v.n_blocks = static_cast<int32_t>(pl.walk_blocks.size() / spex::Plan::kBlockInts);
  v.n_qt = static_cast<int32_t>(pl.walk_qt.size() / 2);
  v.n_items = pl.walk_ok ? static_cast<int32_t>(pl.walk_items.size() / pl.item_ints()) : 0;
  v.row_blocks = pl.walk_rb.data();
  v.blocks = pl.walk_blocks.data();
  v.qt = pl.walk_qt.data();
  v.items = pl.walk_items.data();
  *out = v;
  return SPEX_OK;
}

spex_status_t spex_tree_set_profiling(spex_tree_t *t, int32_t enabled) {
  if (!t) return SPEX_ERR_INVALID_ARG;
  t->profiling = enabled != 0;
  t->prof_calls = 0;
  return SPEX_OK;
}

spex_status_t spex_tree_read_profile(spex_tree_t *t, float *ms, int32_t cap, int32_t *n) {
  if (!t || !n || cap < 0 || (cap > 0 && !ms)) return SPEX_ERR_INVALID_ARG;
  const int64_t have = t->prof_calls < spex_tree::kProfSlots ? t->prof_calls : spex_tree::kProfSlots;
  *n = static_cast<int32_t>(have);
  if (have > cap) return SPEX_ERR_CAPACITY;
  const int64_t first = t->prof_calls - have;
  for (int64_t c = 0; c < have; ++c) {
    spex_tree::ProfSlot &slot = t->prof[(first + c) % spex_tree::kProfSlots];
    for (int i = 0; i < 4; ++i) {
      float r = 0.f;
      if (slot.valid[i]) {
        HIP_TRY(hipEventSynchronize(slot.ev[2 * i + 1]));
        HIP_TRY(hipEventElapsedTime(&r, slot.ev[2 * i], slot.ev[2 * i + 1]));
      }
      ms[c * 4 + i] = r;
    }
  }
  t->prof_calls = 0;
  return SPEX_OK;
}

spex_status_t spex_tree_last_launch_info(const spex_tree_t *t, int64_t info[8]) {
  if (!t || !info) return SPEX_ERR_INVALID_ARG;
  for (int i = 0; i < 8; ++i) info[i] = t->info[i];
  return SPEX_OK;
}

}  // extern "C"
