// Launch interface between the C ABI layer and the HIP kernels.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace spex {

enum Dtype : int32_t { kF32 = 0, kBF16 = 1, kFP8 = 2 };

// Element arrangement inside a (page, kv head) tile; see the pool layout in spex_tree.h.
enum Layout : int32_t { kRowMajor = 0, kMfmaTiled = 1 };

struct Shape {
  int32_t Hq, Hkv, G, D, P;
  int32_t q_dtype, kv_dtype, layout;
  int32_t page_tiles;  // tiles between the starts of consecutive pages inside a pool (>= Hkv)
};

// Everything the attention kernels read; all pointers DEVICE.
struct AttnArgs {
  const void *k_pool, *v_pool;
  const float *k_scale, *v_scale;
  const void *q;
  const int32_t *items;   // 8 ints per work item: {pg_begin, pg_count, qt_begin, qt_count, pbase,
                          //                       flags, kv_head, first_row}
  int32_t n_items;
  const int32_t *pg_rec;  // 2 ints per page entry: {page id, path position << 7 | valid tokens}
  const int32_t *qt_rec;  // 2 ints per row-set entry: {query token, visible path length}
  float *part_o;   // [partial rows][D] unnormalised sum of exp2(x - m) * V
  float *part_ml;  // [partial rows][2] = {m, l}: running maximum of x = score * log2(e), sum of exp2
  // Rows of tasks flagged final are finished in place: the other pieces of a row are read through
  // its merge list (all entries but the last, which is the task itself) and out / lse are written.
  const int32_t *part_indptr, *part_base, *part_hstride;
  float *out, *lse;  // lse may be null
  float scale_log2;
  // Draft-tree visibility, or null for the causal chain: 2 ints per query token {index i of the
  // query in its request, mask}; with base = limit - 1 - i the query sees path positions below base
  // and position base + k iff bit k of the mask is set.
  const int32_t *qt_mask;
};

// Tree-walk kernel: one workgroup per work item.
struct WalkArgs {
  const void *k_pool, *v_pool;
  const float *k_scale, *v_scale;
  const void *q;
  const int32_t *items;   // 16 (2 or 4 wavefronts of rows per row block) or 32 (8) ints per workgroup: {kv head,
                          //   first block, shared blocks, private blocks of wavefronts 0..NW-1,
                          //   first qt_rec entry of each wavefront, qt_rec entries of each
                          //   wavefront, zeros.., row block}; no blocks = padding
  int32_t n_items;
  const int32_t *blocks;  // 8 ints per 32-token block: {page a, pos_a << 7 | valid_a, page b,
                          //   pos_b << 7 | valid_b (0: no page b), first row | (last row + 1) << 16
                          //   within the row block, flags (bit 0: token mask needed), 0, 0}
  const int32_t *qt_rec;  // 2 ints per row-set entry: {query token, visible path length}
  float *out, *lse;       // lse may be null
  float scale_log2;
  const int32_t *qt_mask; // as in AttnArgs; null for the causal chain
};

struct MergeArgs {
  const int32_t *part_indptr, *part_base, *part_hstride;
  const float *part_o, *part_ml;
  float *out, *lse;
  const int32_t *qt_ids;  // query tokens to merge, or null for 0 .. n_qtok-1
  int32_t n_qtok;         // number of query tokens handled by the launch
};

constexpr int kMaxPagesPerScatter = 64;
struct ScatterArgs {
  void *k_pool, *v_pool;
  float *k_scale, *v_scale;              // pool scale arrays (fp8) or null
  const void *k_src, *v_src;             // [n_tokens][Hkv][D]
  const float *k_scale_src, *v_scale_src;  // [new pages][Hkv], already offset to this launch
  int32_t n_pages;                       // pages touched by this launch
  int32_t first_slot;                    // first written slot of page 0 (0 if it is new)
  int32_t n_tokens;                      // tokens written by this launch
  int32_t first_page_is_new;
  int32_t page_ids[kMaxPagesPerScatter];
};

// One token for each of n_nodes nodes in one launch.
struct AppendTokensArgs {
  void *k_pool, *v_pool;
  float *k_scale, *v_scale;                // pool scale arrays (fp8) or null
  const void *k_src, *v_src;               // [n_nodes][Hkv][D]
  const float *k_scale_src, *v_scale_src;  // [n_nodes][Hkv] (fp8; read only for nodes that start a page)
  const int32_t *dst;                      // 2 ints per node: {page id, slot | (page is new) << 8}
  int32_t n_nodes;
  // fp8 pools only: k_src / v_src hold bf16 values, which the kernel encodes with the scale of the
  // page the token lands in (k_scale_src / v_scale_src for a page it starts)
  bool quantise;
  // Length patches of the cached plan, applied by the same launch (thread i < n_patches stores
  // patches[2 i + 1] into plan[patches[2 i]]); n_patches <= number of threads, 0 = none.
  int32_t *plan;
  const int32_t *patches;
  int32_t n_patches;
};

struct GatherArgs {
  const void *k_pool, *v_pool;
  const float *k_scale, *v_scale;
  void *k_out, *v_out;
  float *k_scale_out, *v_scale_out;
  int32_t n_pages, first_slot, n_tokens;
  int32_t page_ids[kMaxPagesPerScatter];
};

// prefix == true launches the shared-prefix kernel, else the suffix kernel; row_tiles is the
// number of 16-row MFMA tiles per wavefront the item list was built for.
hipError_t launch_attention(const Shape &sh, const AttnArgs &a, bool prefix, int row_tiles,
                            bool force_generic, hipStream_t stream);
hipError_t launch_merge(const Shape &sh, const MergeArgs &a, hipStream_t stream);
hipError_t launch_scatter(const Shape &sh, const ScatterArgs &a, hipStream_t stream);
// fp8 pools: k_src / v_src hold bf16 values; page scales are computed (started pages) or reused.
hipError_t launch_scatter_quantise(const Shape &sh, const ScatterArgs &a, hipStream_t stream);
hipError_t launch_gather(const Shape &sh, const GatherArgs &a, hipStream_t stream);
hipError_t launch_append_tokens(const Shape &sh, const AppendTokensArgs &a, hipStream_t stream);
bool has_mfma_kernel(const Shape &sh);
// blob[pairs[2i]] = pairs[2i+1] for i < n (all DEVICE): patches the device copy of a plan.
hipError_t launch_patch(int32_t *blob, const int32_t *pairs, int32_t n, hipStream_t stream);
// Cooperative shared-prefix kernel; ntw in {1, 2, 4} = 16-row tiles per wavefront (64 * ntw rows
// per workgroup).  One work item per workgroup.  Only for shapes with has_mfma_kernel().
hipError_t launch_prefix_coop(const Shape &sh, const AttnArgs &a, int ntw, hipStream_t stream);
// Tree-walk kernel; ntw in {1, 2, 4} = 16-row tiles per wavefront and waves in {2, 4, 8} = wavefronts
// of rows per row block the lists were built for (2: run by four wavefronts, two on each set of
// rows, which split the path between them; ntw 1 or 2, no draft masks).
hipError_t launch_tree_walk(const Shape &sh, const WalkArgs &a, int ntw, int waves, hipStream_t stream);

}  // namespace spex
