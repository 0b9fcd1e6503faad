// HIP kernels for tree decode attention on gfx950 (CDNA4, 64-lane wavefronts).
//
//   spex_tree_walk_kernel  (the default path)
//       One workgroup per (row block, kv head) carries up to 16 * NTW * NW query rows from the root
//       to their requested nodes in one launch: blocks whose rows span several wavefronts are
//       fetched once per workgroup and staged in LDS as MFMA operand images, blocks of one
//       wavefront stream straight into its operand registers, and the online-softmax state stays
//       in registers until the finished rows are written -- no partial results, no merge.
//   spex_prefix_coop_kernel
//       The shared-prefix step of the split path for nodes with many stacked rows: one workgroup
//       per (task, kv head, span of rows), operand images in LDS as in the tree-walk kernel.
//   spex_prefix_attn_kernel / spex_suffix_attn_kernel
//       One wavefront per work item = (task, kv head, row tile).  A task is a run of KV pages
//       (a chunk of a shared-prefix group or of a private suffix) and a set of query rows; the
//       wavefront streams the pages once, contracts them against its rows on the matrix cores
//       (S^T = K Q^T and O^T = V^T P^T with MFMA 16x16x32 bf16, fp32 accumulation), keeps an
//       online softmax per row and emits the partial state (m, l, o).  The shared-prefix kernel
//       stacks the rows of all branches below a node, so the node's pages are read once for all
//       of them; the suffix kernel has the few rows of one branch and is bound by HBM bandwidth.
//   spex_generic_attn_kernel
//       Same contract without matrix cores, for fp32 KV and shapes the MFMA kernels do not cover.
//   spex_lse_merge_kernel
//       Combines the partial states of every query row (log-sum-exp rule) and normalises.
//   spex_scatter_kv_kernel / spex_scatter_quant_kernel / spex_append_tokens_kernel / spex_gather_kv_kernel
//       Write appended tokens into (a run for one node, the same quantised to e4m3 on the way, one
//       token for each of many nodes) / read tokens out of the paged pool.
//   spex_patch_plan_kernel
//       Applies {index, value} patches to the device copy of the cached launch lists.
#include "kernels.hpp"

#include <climits>

namespace spex {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kNegInf = -__builtin_huge_valf();
// Start value of the tree-walk kernel's softmax reference: finite, so that (-inf) - m stays -inf,
// and so far below any score that the first visible score replaces it.
constexpr float kWalkMInit = -1.0e30f;

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Wave-uniform read of plan data through the scalar (constant) path.  The plan arrays are
// written by the host before the launch and never by a kernel.  Going through scalar loads keeps
// these small reads out of the vector-memory queue, whose in-order completion counter would
// otherwise make every page-record lookup wait for all K/V loads in flight.
typedef const int32_t __attribute__((address_space(4))) const_i32;
__device__ __forceinline__ int sload(const int32_t *base, int64_t idx) {
  return ((const_i32 *)(uintptr_t)base)[idx];
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Maximum over lanes l, l^16, l^32, l^48 (the four lane groups that hold one query row), by the
// gfx950 row-swap instructions: v_permlane16_swap exchanges the odd 16-lane rows of its first
// operand with the even rows of its second, v_permlane32_swap the upper half of the first with
// the lower half of the second; with both operands equal, the pair afterwards holds the value of
// the lane and of its partner.  Two wait states separate a vector write from a swap that reads it.
// The compiler does not track hazards of instructions inside inline assembly, so the argument must
// be the result of an ordinary vector ALU instruction (here: the v_max that folds in the running
// maximum) -- never directly of an MFMA, whose results need many more wait states before they can
// be read.
__device__ __forceinline__ float row_group_max(float v) {
  float a = v, b = v;
  asm("s_nop 1\n\t"
      "v_permlane16_swap_b32 %0, %1\n\t"
      "v_max_f32 %0, %0, %1\n\t"
      "v_mov_b32 %1, %0\n\t"
      "s_nop 1\n\t"
      "v_permlane32_swap_b32 %0, %1\n\t"
      "v_max_f32 %0, %0, %1"
      : "+v"(a), "+v"(b));
  return a;
}

// 128-bit K/V load.  Every K/V byte is used once per launch, so the loads carry the non-temporal
// hint: measured on MI355X, a streaming read of the pool reaches 7.0 TB/s with it against
// 6.2 TB/s without (the lines do not displace each other in the last-level caches).
__device__ __forceinline__ u32x4 load_kv(const char *p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

// ---- element offsets inside a (page, kv head) tile ------------------------------------------
template <int KV, int LAYOUT>
__device__ __forceinline__ int k_offset(int t, int d, int D) {
  if (LAYOUT == kRowMajor) return t * D + d;
  const int tt = 4 * (t >> 3) + (t & 3);
  if (KV == kFP8)
    return ((t >> 2) & 1) * 8 * D + (d >> 6) * 512 + ((d & 31) >> 3) * 128 + tt * 16 +
           ((d >> 5) & 1) * 8 + (d & 7);
  return ((t >> 2) & 1) * 8 * D + (d >> 5) * 256 + ((d & 31) >> 3) * 64 + tt * 8 + (d & 7);
}

template <int KV, int LAYOUT>
__device__ __forceinline__ int v_offset(int t, int d, int D) {
  if (LAYOUT == kRowMajor) return t * D + d;
  if (KV == kFP8)
    return (d >> 5) * 512 + (t >> 3) * 256 + (d & 15) * 16 + ((d >> 4) & 1) * 8 + (t & 7);
  return (d >> 4) * 256 + (t >> 3) * 128 + (d & 15) * 8 + (t & 7);
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __builtin_bit_cast(float, static_cast<uint32_t>(b) << 16);
}

// OCP e4m3fn code -> fp32 (exact).
__device__ __forceinline__ float e4m3_to_float(uint8_t c) {
  const f32x2 r = __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(c), false);
  return r[0];
}

template <int KV>
__device__ __forceinline__ float load_elem(const void *base, int64_t idx) {
  if (KV == kF32) return static_cast<const float *>(base)[idx];
  if (KV == kBF16) return bf16_bits_to_float(static_cast<const uint16_t *>(base)[idx]);
  return e4m3_to_float(static_cast<const uint8_t *>(base)[idx]);
}

// V of a bf16 pool in the MFMA-tiled layout is stored as IEEE half precision, so that a tile is an
// fp16 operand image of the PV product as it lies in memory.  The append kernels convert once,
// rounding toward zero: exact for magnitudes in [2^-17, 65504] (a bf16 has 8 significant bits, an
// fp16 11, and subnormal fp16 still resolve 2^-24); a finite magnitude above 65504 becomes +-65504
// instead of infinity (0 * inf in the PV product would poison a whole row), one below 2^-17 keeps
// the multiples of 2^-24 it contains.  K stays bf16.
template <int KV, int LAYOUT>
__device__ __forceinline__ constexpr bool v_is_f16() {
  return KV == kBF16 && LAYOUT == kMfmaTiled;
}
__device__ __forceinline__ uint16_t bf16_bits_to_f16_bits(uint16_t b) {
  const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(bf16_bits_to_float(b), 0.f));
  return static_cast<uint16_t>(w & 0xffffu);
}
// Back to bf16 by truncation: exact for everything bf16_bits_to_f16_bits produced.
__device__ __forceinline__ uint16_t f16_bits_to_bf16_bits(uint16_t h) {
  const float f = static_cast<float>(__builtin_bit_cast(_Float16, h));
  return static_cast<uint16_t>(__builtin_bit_cast(uint32_t, f) >> 16);
}
template <int KV, int LAYOUT>
__device__ __forceinline__ float load_v_elem(const void *base, int64_t idx) {
  if (v_is_f16<KV, LAYOUT>())
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<const uint16_t *>(base)[idx]));
  return load_elem<KV>(base, idx);
}

template <int KV>
__device__ __forceinline__ constexpr int elem_size() {
  return KV == kF32 ? 4 : (KV == kBF16 ? 2 : 1);
}

// ---- MFMA attention ------------------------------------------------------------------------
// Two fp32 -> one dword of two bf16 (truncation): low half from a, high half from b.
__device__ __forceinline__ uint32_t pack_hi16(float a, float b) {
  return __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, b), __builtin_bit_cast(uint32_t, a),
                               0x07060302u);
}

// Eight e4m3 codes (two dwords) -> eight bf16 (exact: 3 mantissa bits fit in 7).  The scaled
// conversion of gfx950 turns two codes into two packed 16-bit values in one instruction; it uses
// only the exponent of its scale operand (checked on the device for all codes), here 2^0.
__device__ __forceinline__ bf16x8 fp8x8_to_bf16x8(uint32_t w0, uint32_t w1) {
  u32x4 r;
  r[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(w0), 1.0f, false));
  r[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(w0), 1.0f, true));
  r[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(w1), 1.0f, false));
  r[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(w1), 1.0f, true));
  return __builtin_bit_cast(bf16x8, r);
}

// Wave-uniform description of one work item.
struct Item {
  int pg_begin, pg_count, qt_begin, qt_count, pbase, flags, g, row0;
};

__device__ __forceinline__ Item load_item(const int32_t *items, int idx) {
  const int64_t r = static_cast<int64_t>(uniform(idx)) * 8;
  Item it;
  it.pg_begin = sload(items, r + 0);
  it.pg_count = sload(items, r + 1);
  it.qt_begin = sload(items, r + 2);
  it.qt_count = sload(items, r + 3);
  it.pbase = sload(items, r + 4);
  it.flags = sload(items, r + 5);
  it.g = sload(items, r + 6);
  it.row0 = sload(items, r + 7);
  return it;
}

// Page ids / valid counts / positions of one 32-token block, wave-uniform.
struct BlockMeta {
  int pid_a, pid_b, vp_a, vp_b;  // vp = position << 7 | valid; vp_b = 0 when the block has one page
};

__device__ __forceinline__ BlockMeta load_block_meta(const int32_t *pg_rec, const Item &it, int b) {
  const int ia = it.pg_begin + 2 * b;
  const bool has_b = 2 * b + 1 < it.pg_count;
  const int ib = has_b ? ia + 1 : ia;
  BlockMeta bm;
  bm.pid_a = sload(pg_rec, 2 * ia);
  bm.vp_a = sload(pg_rec, 2 * ia + 1);
  bm.pid_b = sload(pg_rec, 2 * ib);
  bm.vp_b = has_b ? sload(pg_rec, 2 * ib + 1) : 0;
  return bm;
}

// Per-wavefront state of NT tiles of 16 query rows.  Lane (n = lane % 16, jj = lane / 16) works
// on row n of every tile; its accumulators hold dims dt*16 + 4*jj .. +3.
template <int D, int NT>
struct RowState {
  bf16x8 qf[NT][D / 32];  // query operand: dims s*32 + 8*jj .. +7
  int limit[NT], qtok[NT];
  int qidx[NT];           // draft token trees: index of the row's query in its request
  uint32_t dmask[NT];     //   and its visibility mask among the request's drafts
  f32x4 o[NT][D / 16];
  float m[NT], l[NT];     // l is this lane's share; summed over the four jj at the end
};

// Scores of the lane's 8 tokens that the row does not see become -inf.  Chain: the first
// limit - pos positions of the page are visible.  Draft token tree: positions below
// base = limit - 1 - qidx are visible, position base + k iff bit k of the row's mask is set; shifting
// {mask, 32 ones} right by (first position of the lane's tokens - base + 32) puts the visibility of
// the lane's 8 tokens into the low 8 bits.
template <bool TREE>
__device__ __forceinline__ void mask_scores(float (&x)[8], int limit, int qidx, uint32_t dmask, int valid_l,
                                            int pos_l, bool row_in) {
  const int jj = (threadIdx.x & 63) >> 4;
  const int first = 8 * (jj & 1);
  if (TREE) {
    const int base = limit - 1 - qidx;
    const int sh = pos_l + first - base + 32;
    const uint64_t bits = (static_cast<uint64_t>(dmask) << 32) | 0xffffffffull;
    uint32_t vm = sh <= 0 ? 0xffu : (sh >= 64 ? 0u : static_cast<uint32_t>(bits >> sh) & 0xffu);
    const int have = valid_l - first;  // tokens of the lane's 8 that exist
    vm = row_in ? vm : 0u;
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (i < have && ((vm >> i) & 1u)) ? x[i] : kNegInf;
  } else {
    int vis = limit - pos_l;
    vis = vis < valid_l ? vis : valid_l;
    vis -= first;
    vis = row_in ? vis : 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = i < vis ? x[i] : kNegInf;
  }
}

template <int D, int NT>
__device__ __forceinline__ void load_rows(const AttnArgs &p, const Shape &sh, const Item &cur,
                                          int row_base, RowState<D, NT> &st) {
  const int lane = threadIdx.x & 63, m16 = lane & 15, jj = lane >> 4;
  const int G = sh.G, rows = cur.qt_count * G;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int r = row_base + nt * 16 + m16;
    st.limit[nt] = INT_MAX;
    st.qtok[nt] = 0;
    st.qidx[nt] = 0;
    st.dmask[nt] = 0;
    st.m[nt] = kNegInf;
    st.l[nt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) st.o[nt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (r < rows) {
      const int2 qr = *reinterpret_cast<const int2 *>(p.qt_rec + 2 * (cur.qt_begin + r / G));
      st.limit[nt] = qr.y;
      st.qtok[nt] = qr.x;
      if (p.qt_mask) {
        const int2 dm = *reinterpret_cast<const int2 *>(p.qt_mask + 2 * qr.x);
        st.qidx[nt] = dm.x;
        st.dmask[nt] = static_cast<uint32_t>(dm.y);
      }
      const uint16_t *qp = static_cast<const uint16_t *>(p.q) +
                           (static_cast<int64_t>(qr.x) * sh.Hq + cur.g * G + r % G) * D + jj * 8;
#pragma unroll
      for (int s = 0; s < D / 32; ++s)
        st.qf[nt][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(qp + s * 32));
    } else {
#pragma unroll
      for (int s = 0; s < D / 32; ++s) st.qf[nt][s] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
    }
  }
}

// One 32-token block (pages A and B of one kv head) against the wavefront's rows.
// kf[t][s]: K half-tile t (tokens {0-3, 8-11} + 4t of each page), dims s*32..; rows 0-7 of the MFMA
// tile come from page A, rows 8-15 from page B.  vf[dt]: V^T, dims dt*16.., tokens 8*(jj&1)..+7 of
// page jj/2.  After the two score tiles this lane holds the scores of exactly those 8 tokens, i.e.
// the operand layout of the PV product, so P never leaves the registers.
// VF16: vf holds fp16 (V of a bf16 pool as stored), else bf16 (widened fp8 codes).
template <bool TREE, bool VF16, int D, int NT>
__device__ __forceinline__ void block_math(RowState<D, NT> &st, const bf16x8 (&kf)[2][D / 32],
                                           const bf16x8 (&vf)[D / 16], bool masked, int valid_l,
                                           int pos_l, float c, float vs) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
      sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][s], st.qf[nt][s], sa, 0, 0, 0);
      sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][s], st.qf[nt][s], sb, 0, 0, 0);
    }
    float x[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[i] = sa[i] * c;
      x[4 + i] = sb[i] * c;
    }
    if (masked) mask_scores<TREE>(x, st.limit[nt], st.qidx[nt], st.dmask[nt], valid_l, pos_l, true);
    float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                     fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(st.m[nt], mx);
    const float m_safe = m_new == kNegInf ? 0.f : m_new;
    const float alpha = fast_exp2(st.m[nt] - m_safe);
    float pr[8];
    float lsum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pr[i] = fast_exp2(x[i] - m_safe);
      lsum += pr[i];
    }
    st.l[nt] = st.l[nt] * alpha + lsum;
    st.m[nt] = m_new;
    if (!__all(alpha == 1.0f)) {
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) st.o[nt][dt] *= alpha;
    }
    // P as two pieces (hi + lo, each rounded toward zero, lo from the exact fp32 remainder) so that
    // the product keeps ~16 (bf16 pieces) or ~22 (fp16 pieces) bits of each weight.
    u32x4 phi, plo;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float a0 = pr[2 * i] * vs, a1 = pr[2 * i + 1] * vs;
      if (VF16) {  // weights are at most 1 here: no overflow
        const auto h = __builtin_amdgcn_cvt_pkrtz(a0, a1);
        phi[i] = __builtin_bit_cast(uint32_t, h);
        plo[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a0 - static_cast<float>(h[0]),
                                                                         a1 - static_cast<float>(h[1])));
      } else {
        const float h0 = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, a0) & 0xffff0000u);
        const float h1 = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, a1) & 0xffff0000u);
        phi[i] = pack_hi16(h0, h1);
        plo[i] = pack_hi16(a0 - h0, a1 - h1);
      }
    }
    if (VF16) {
      const f16x8 ph = __builtin_bit_cast(f16x8, phi);
      const f16x8 pl = __builtin_bit_cast(f16x8, plo);
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) {
        const f16x8 vh = __builtin_bit_cast(f16x8, vf[dt]);
        st.o[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vh, ph, st.o[nt][dt], 0, 0, 0);
        st.o[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vh, pl, st.o[nt][dt], 0, 0, 0);
      }
    } else {
      const bf16x8 ph = __builtin_bit_cast(bf16x8, phi);
      const bf16x8 pl = __builtin_bit_cast(bf16x8, plo);
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) {
        st.o[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], ph, st.o[nt][dt], 0, 0, 0);
        st.o[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pl, st.o[nt][dt], 0, 0, 0);
      }
    }
  }
}

// Floats of LDS one wavefront needs to transpose a 16-row tile.
template <int D>
constexpr int stage_floats() { return 16 * (D + 4); }

// Emit the rows of a wavefront: partial state (m, l, o) for the merge step, or -- for a task
// flagged final -- the finished output rows after folding in the rows' other pieces.  The
// accumulators hold 4 consecutive dims of one row per lane (64 B runs at a 512 B stride); they are
// transposed through the wave-private LDS tile `my` so that every store instruction writes whole
// rows (1 KiB contiguous) instead of half-filled cache lines.
template <int D, int NT, bool ALLOW_FINAL>
__device__ __forceinline__ void finish_rows(const AttnArgs &p, const Shape &sh, const Item &cur,
                                            int row_base, f32x4 (&o)[NT][D / 16],
                                            const float (&m_in)[NT], const float (&l_in)[NT],
                                            const int (&qtok)[NT], float *my) {
  constexpr int kRowPad = D + 4;  // the pad spreads rows over LDS banks
  const int lane = threadIdx.x & 63, m16 = lane & 15, jj = lane >> 4;
  const int G = sh.G, rows = cur.qt_count * G, g = cur.g;
  const bool final_task = ALLOW_FINAL && (cur.flags & 2) != 0;
  constexpr int kLanesPerRow = D / 4;  // 16-byte pieces per row
  constexpr int kRowsPerInst = 64 / kLanesPerRow;
  const int sub = lane / kLanesPerRow, piece = lane % kLanesPerRow;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    float l = l_in[nt];
    float m = m_in[nt];
    const int r0w = row_base + nt * 16;  // first row of this tile
    if (r0w >= rows) break;              // wave-uniform
    const bool row_ok = r0w + m16 < rows;
    const int hh = (r0w + m16) % G;
    int64_t dst_row;  // row index in part_o, or in out for a final task
    if (ALLOW_FINAL && final_task) {
      // Fold in the other pieces of this row (written by the shared-prefix kernels, which ran
      // before on the same stream) and normalise.  All rows of a suffix belong to one requested
      // node, so they have the same number of pieces.
      int e0 = 0, n_other = 0;
      if (row_ok) {
        e0 = p.part_indptr[qtok[nt]];
        n_other = p.part_indptr[qtok[nt] + 1] - 1 - e0;
      }
      const int n_max = uniform(n_other);
      auto fold = [&](const f32x2 ml, const f32x4 (&oj)[D / 16], bool use) {
        const float mj = use ? ml[0] : kNegInf;
        const float m_new = fmaxf(m, mj);
        const float m_safe = m_new == kNegInf ? 0.f : m_new;
        const float fa = fast_exp2(m - m_safe), fb = fast_exp2(mj - m_safe);
        l = l * fa + ml[1] * fb;
        m = m_new;
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) o[nt][dt] = o[nt][dt] * fa + oj[dt] * fb;
      };
      if (n_max > 0) {
        // The first 8 pieces are fetched four at a time with all loads of a batch in flight
        // together.  Indices past a row's last piece are clamped to it (a repeated, finite read
        // that is weighted with zero), which keeps the batches free of per-piece branches.
        constexpr int kBatch = 4;
        int64_t slot[2 * kBatch];
#pragma unroll
        for (int j = 0; j < 2 * kBatch; ++j) {
          const int last = n_other - 1;
          const int e = e0 + max(0, j < last ? j : last);
          slot[j] = static_cast<int64_t>(p.part_base[e]) + static_cast<int64_t>(g) * p.part_hstride[e] + hh;
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          if (q * kBatch < n_max) {
            f32x2 ml[kBatch];
            f32x4 oj[kBatch][D / 16];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
              ml[k] = *reinterpret_cast<const f32x2 *>(p.part_ml + slot[q * kBatch + k] * 2);
              const float *src = p.part_o + slot[q * kBatch + k] * D + jj * 4;
#pragma unroll
              for (int dt = 0; dt < D / 16; ++dt) oj[k][dt] = *reinterpret_cast<const f32x4 *>(src + dt * 16);
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) fold(ml[k], oj[k], q * kBatch + k < n_other);
          }
        }
        for (int j = 2 * kBatch; j < n_max; ++j) {  // deeper paths: one piece at a time
          const int last = n_other - 1;
          const int e = e0 + max(0, j < last ? j : last);
          const int64_t sl = static_cast<int64_t>(p.part_base[e]) + static_cast<int64_t>(g) * p.part_hstride[e] + hh;
          const f32x2 ml = *reinterpret_cast<const f32x2 *>(p.part_ml + sl * 2);
          f32x4 oj[D / 16];
          const float *src = p.part_o + sl * D + jj * 4;
#pragma unroll
          for (int dt = 0; dt < D / 16; ++dt) oj[dt] = *reinterpret_cast<const f32x4 *>(src + dt * 16);
          fold(ml, oj, j < n_other);
        }
      }
      const float inv = 1.0f / l;
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) o[nt][dt] *= inv;
      dst_row = static_cast<int64_t>(qtok[nt]) * sh.Hq + g * G + hh;
      if (row_ok && jj == 0 && p.lse) p.lse[dst_row] = (m + __builtin_log2f(l)) * 0.6931471805599453f;
    } else {
      dst_row = static_cast<int64_t>(cur.pbase) + static_cast<int64_t>(g) * rows + r0w + m16;
      if (row_ok && jj == 0) *reinterpret_cast<f32x2 *>(p.part_ml + dst_row * 2) = f32x2{m, l};
    }
    float *dst = final_task ? p.out : p.part_o;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
      *reinterpret_cast<f32x4 *>(my + m16 * kRowPad + dt * 16 + jj * 4) = o[nt][dt];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < 16 / kRowsPerInst; ++i) {
      const int row = i * kRowsPerInst + sub;
      const f32x4 v = *reinterpret_cast<const f32x4 *>(my + row * kRowPad + piece * 4);
      // destination row index of tile row `row`, held by lane `row` (k-group 0)
      const int lo = __shfl(static_cast<int>(dst_row & 0xffffffff), row);
      const int hi = __shfl(static_cast<int>(dst_row >> 32), row);
      const int64_t drow = (static_cast<int64_t>(hi) << 32) | static_cast<uint32_t>(lo);
      if (r0w + row < rows) *reinterpret_cast<f32x4 *>(dst + drow * D + piece * 4) = v;
    }
  }
}

// Raw 128-bit pieces of one 32-token block (two pages) of one kv head, as loaded.
template <int KV, int D>
struct RawBlock {
  static constexpr int NK = (KV == kFP8) ? D / 64 : D / 32;  // loads per K half-tile
  static constexpr int NV = (KV == kFP8) ? D / 32 : D / 16;
  u32x4 k[2][NK];
  u32x4 v[NV];
  int valid_a, valid_b, pos_a, pos_b;
  float ks, vs;  // this lane's page scales (fp8), else 1
};

// ---- wavefront kernel: one wavefront per work item ---------------------------------------------
// The K/V loads of block b+1 are in flight while block b is computed.  The steady-state loop is
// free of conditional loads on purpose: the vector-memory completion counter is in-order, and a
// load that is issued on one path only would force the compiler to wait for everything
// outstanding at the join.
template <int KV, int D, int NT, bool SUFFIX, bool TREE>
__device__ __forceinline__ void attn_wave(const AttnArgs &p, const Shape &sh) {
  constexpr int ESZ = (KV == kFP8) ? 1 : 2;
  constexpr int TILE_BYTES = 16 * D * ESZ;
  const int lane = threadIdx.x & 63;
  const int m16 = lane & 15;
  const int jj = lane >> 4;
  const int item_idx = uniform(blockIdx.x * 4 + (threadIdx.x >> 6));
  if (item_idx >= p.n_items) return;
  const char *kpool = static_cast<const char *>(p.k_pool);
  const char *vpool = static_cast<const char *>(p.v_pool);
  // Byte offset of this lane inside a K half-tile / a V tile.
  const int k_lane_off = jj * 128 + (m16 & 7) * 16;
  const int v_lane_off = (jj & 1) * 256 + m16 * 16;

  const Item cur = load_item(p.items, item_idx);
  if (cur.pg_count == 0) return;  // padding item
  const int g = cur.g;
  const int nblk = (cur.pg_count + 1) >> 1;

  auto issue_loads = [&](RawBlock<KV, D> &rb, const BlockMeta &bm) {
    rb.valid_a = bm.vp_a & 127;
    rb.valid_b = bm.vp_b & 127;
    rb.pos_a = bm.vp_a >> 7;
    rb.pos_b = bm.vp_b >> 7;
    const int64_t tile_a = (static_cast<int64_t>(bm.pid_a) * sh.page_tiles + g);
    const int64_t tile_b = (static_cast<int64_t>(bm.pid_b) * sh.page_tiles + g);
    const char *kp = kpool + (m16 < 8 ? tile_a : tile_b) * TILE_BYTES + k_lane_off;
    const char *vp = vpool + (jj < 2 ? tile_a : tile_b) * TILE_BYTES + v_lane_off;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int s = 0; s < RawBlock<KV, D>::NK; ++s)
        rb.k[t][s] = load_kv(kp + t * (TILE_BYTES / 2) + s * 512);
#pragma unroll
    for (int s = 0; s < RawBlock<KV, D>::NV; ++s)
      rb.v[s] = load_kv(vp + s * 512);
    if (KV == kFP8) {
      const int sidx = (jj < 2 ? bm.pid_a : bm.pid_b) * sh.Hkv + g;
      rb.ks = p.k_scale[sidx];
      rb.vs = p.v_scale[sidx];
    } else {
      rb.ks = 1.f;
      rb.vs = 1.f;
    }
  };
  // page records of block min(b, nblk - 1)
  auto meta = [&](int b) { return load_block_meta(p.pg_rec, cur, b < nblk ? b : nblk - 1); };

  const bool task_masked = (cur.flags & 1) != 0;
  RowState<D, NT> st;
  load_rows<D, NT>(p, sh, cur, cur.row0, st);

  RawBlock<KV, D> r0, r1;
  issue_loads(r0, meta(0));

  auto compute_block = [&](const RawBlock<KV, D> &rb) {
    bf16x8 kf[2][D / 32];
    bf16x8 vf[D / 16];
    if (KV == kFP8) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int s = 0; s < D / 64; ++s) {
          kf[t][2 * s] = fp8x8_to_bf16x8(rb.k[t][s][0], rb.k[t][s][1]);
          kf[t][2 * s + 1] = fp8x8_to_bf16x8(rb.k[t][s][2], rb.k[t][s][3]);
        }
#pragma unroll
      for (int s = 0; s < D / 32; ++s) {
        vf[2 * s] = fp8x8_to_bf16x8(rb.v[s][0], rb.v[s][1]);
        vf[2 * s + 1] = fp8x8_to_bf16x8(rb.v[s][2], rb.v[s][3]);
      }
    } else {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int s = 0; s < D / 32; ++s) kf[t][s] = __builtin_bit_cast(bf16x8, rb.k[t][s]);
#pragma unroll
      for (int s = 0; s < D / 16; ++s) vf[s] = __builtin_bit_cast(bf16x8, rb.v[s]);
    }
    // This lane's score registers cover tokens 8*(jj&1) .. +7 of page A (jj < 2) or B.
    block_math<TREE, KV == kBF16, D, NT>(st, kf, vf, task_masked || rb.valid_b == 0, jj < 2 ? rb.valid_a : rb.valid_b,
                      jj < 2 ? rb.pos_a : rb.pos_b, p.scale_log2 * rb.ks, rb.vs);
  };

  BlockMeta bm1 = meta(1);
  int b = 0;
  for (; b + 2 < nblk; b += 2) {  // blocks b, b+1, b+2 all exist
    const BlockMeta bm2 = meta(b + 2);
    issue_loads(r1, bm1);
    compute_block(r0);
    bm1 = meta(b + 3);
    issue_loads(r0, bm2);
    compute_block(r1);
  }
  if (b + 1 < nblk) {
    issue_loads(r1, bm1);
    compute_block(r0);
    compute_block(r1);
  } else {
    compute_block(r0);
  }

  __shared__ float stage[4][stage_floats<D>()];
  float l_tot[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {  // the row sum is spread over the four lane groups
    float l = st.l[nt];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    l_tot[nt] = l;
  }
  finish_rows<D, NT, SUFFIX>(p, sh, cur, cur.row0, st.o, st.m, l_tot, st.qtok, stage[threadIdx.x >> 6]);
}

template <int KV, int D, int NT, bool TREE>
__global__ __launch_bounds__(256, NT == 1 ? 2 : 1) void spex_prefix_attn_kernel(AttnArgs p, Shape sh) {
  attn_wave<KV, D, NT, false, TREE>(p, sh);
}

template <int KV, int D, int NT, bool TREE>
__global__ __launch_bounds__(256, NT == 1 ? 2 : 1) void spex_suffix_attn_kernel(AttnArgs p, Shape sh) {
  attn_wave<KV, D, NT, true, TREE>(p, sh);
}

// Block step of the cooperative kernel.  Same contraction as block_math, tuned for many row
// tiles per wavefront, where the vector ALU work of the softmax -- not the matrix cores -- sets
// the pace:
//  * P is rounded once to fp16 (11 significant bits; toward zero, one instruction per pair: the
//    row sum is taken from the same rounded weights, so the mean shortfall cancels in o / l and
//    what remains has the spread of round-to-nearest) and V^T arrives as fp16 operand images, so
//    PV is one MFMA per tile instead of a hi and a lo one;
//  * the row sums come from one more MFMA against a tile of ones, which also adds up the four
//    lane groups and uses the same rounded weights as the numerator;
//  * with a page-independent scale (bf16 KV) the running maximum is kept on the raw scores and
//    scale and subtraction fuse into one FMA per score.
// m is in units of raw score for bf16 KV and of scaled score for fp8 KV (c differs per page).
template <bool FP8, bool TREE, int D, int NT>
__device__ __forceinline__ void block_math_f16(const bf16x8 (&qf)[NT][D / 32], const int (&limit)[NT],
                                               const int (&qidx)[NT], const uint32_t (&dmask)[NT],
                                               f32x4 (&o)[NT][D / 16], float (&m)[NT],
                                               f32x4 (&lacc)[NT], const bf16x8 (&kf)[2][D / 32],
                                               const f16x8 (&vh)[D / 16], bool masked, int valid_l,
                                               int pos_l, float c) {
  const _Float16 one = static_cast<_Float16>(1.0f);
  const f16x8 ones = {one, one, one, one, one, one, one, one};
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
      sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][s], qf[nt][s], sa, 0, 0, 0);
      sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][s], qf[nt][s], sb, 0, 0, 0);
    }
    float x[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[i] = FP8 ? sa[i] * c : sa[i];
      x[4 + i] = FP8 ? sb[i] * c : sb[i];
    }
    if (masked) mask_scores<TREE>(x, limit[nt], qidx[nt], dmask[nt], valid_l, pos_l, true);
    float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                     fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m[nt], mx);
    const float m_safe = m_new == kNegInf ? 0.f : m_new;
    float alpha, pr[8];
    if (FP8) {
      alpha = fast_exp2(m[nt] - m_safe);
#pragma unroll
      for (int i = 0; i < 8; ++i) pr[i] = fast_exp2(x[i] - m_safe);
    } else {
      const float mc = m_safe * c;
      alpha = fast_exp2(m[nt] * c - mc);
#pragma unroll
      for (int i = 0; i < 8; ++i) pr[i] = fast_exp2(__builtin_fmaf(x[i], c, -mc));
    }
    m[nt] = m_new;
    if (!__all(alpha == 1.0f)) {
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) o[nt][dt] *= alpha;
      lacc[nt] *= alpha;
    }
    u32x4 pw;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      pw[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(pr[2 * i], pr[2 * i + 1]));
    const f16x8 ph = __builtin_bit_cast(f16x8, pw);
    lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, ph, lacc[nt], 0, 0, 0);
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
      o[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vh[dt], ph, o[nt][dt], 0, 0, 0);
  }
}

// Largest V page scale the fp16 operand images can hold: 448 * 146 = 65408 <= 65504.  A larger
// scale is read as this one (the page's values shrink together instead of turning into infinities).
constexpr float kMaxVScaleF16 = 146.0f;
// Smallest K page scale used in a product with a masked (-inf) score: a scale of 0 (an all-zero
// page) would turn -inf into NaN; with this value the page's scores are 0 to within 1e-27.
constexpr float kMinKScale = 1.0e-30f;

// Eight e4m3 codes times a page scale (finite, 0 <= scale <= kMaxVScaleF16) -> eight fp16.  The
// scale is taken apart as 2^e * m with m in [1, 2): the scaled conversion applies 2^e (exact while
// the result is a normal fp16), a packed fp16 multiply applies m rounded to fp16.  Against
// code * scale in exact arithmetic the result is off by at most 2^-10 relative (two roundings to
// 11 bits), and below 2^-14 in magnitude by less than 2^-23 absolute.  A scale of 0 (or an fp32
// subnormal) gives zeros.
__device__ __forceinline__ u32x4 fp8x8_to_f16x8(uint32_t w0, uint32_t w1, float scale) {
  const uint32_t sb = __builtin_bit_cast(uint32_t, scale);
  const float pow2 = __builtin_bit_cast(float, sb & 0x7f800000u);
  const _Float16 mant = static_cast<_Float16>(__builtin_bit_cast(float, (sb & 0x007fffffu) | 0x3f800000u));
  const f16x2 m2 = {mant, mant};
  u32x4 r;
  r[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(static_cast<int>(w0), pow2, false) * m2);
  r[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(static_cast<int>(w0), pow2, true) * m2);
  r[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(static_cast<int>(w1), pow2, false) * m2);
  r[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(static_cast<int>(w1), pow2, true) * m2);
  return r;
}

// ---- cooperative shared-prefix kernel: one workgroup (4 wavefronts) per work item --------------
// For groups with many stacked rows.  The workgroup covers up to 64 * NTW rows of one (task, kv
// head); wavefront w owns rows row0 + w*16*NTW .. .  Each 32-token block is fetched from global
// memory once per workgroup -- every wavefront loads a quarter of it -- and is placed in LDS as
// ready-made MFMA operand images (K as bf16, V^T as fp16, fp8 widened on the way and V multiplied
// by its page scale) that all four wavefronts read (lane * 16 B, conflict free).  Two LDS buffers
// and one barrier per block.
template <int KV, int D, int NTW, bool TREE>
__global__ __launch_bounds__(256, NTW <= 2 ? 2 : 1) void spex_prefix_coop_kernel(AttnArgs p, Shape sh) {
  constexpr bool FP8 = KV == kFP8;
  constexpr int ESZ = FP8 ? 1 : 2;
  constexpr int TILE_BYTES = 16 * D * ESZ;
  constexpr int NKI = 2 * (D / 32);        // K operand images per block
  constexpr int NI = NKI + D / 16;         // all operand images per block (1 KiB each)
  constexpr int RAW = FP8 ? NI / 2 : NI;   // 1 KiB global loads per block
  constexpr int RK = FP8 ? NKI / 2 : NKI;  // of which K
  constexpr int PER = RAW / 4;             // global loads per wavefront and block
  static_assert(RAW % 4 == 0, "block must split evenly over four wavefronts");
  constexpr int kImgFloats = NI * 64 * 4;  // one buffer, in 4-byte units
  constexpr int kLdsFloats =
      2 * kImgFloats > 4 * stage_floats<D>() ? 2 * kImgFloats : 4 * stage_floats<D>();
  __shared__ __attribute__((aligned(16))) float lds[kLdsFloats];
  u32x4 *img = reinterpret_cast<u32x4 *>(lds);  // [buf][image][lane]

  const int lane = threadIdx.x & 63, m16 = lane & 15, jj = lane >> 4;
  const int w = uniform(threadIdx.x >> 6);
  const Item cur = load_item(p.items, blockIdx.x);
  if (cur.pg_count == 0) return;  // padding item (whole workgroup)
  const int g = cur.g;
  const int nblk = (cur.pg_count + 1) >> 1;
  const int rows = cur.qt_count * sh.G;
  const int row_base = cur.row0 + w * 16 * NTW;
  const bool has_rows = row_base < rows;
  const bool task_masked = (cur.flags & 1) != 0;
  const char *kpool = static_cast<const char *>(p.k_pool);
  const char *vpool = static_cast<const char *>(p.v_pool);
  const int k_lane_off = jj * 128 + (m16 & 7) * 16;
  const int v_lane_off = (jj & 1) * 256 + m16 * 16;

  RowState<D, NTW> st;
  load_rows<D, NTW>(p, sh, cur, row_base, st);
  f32x4 lacc[NTW];
#pragma unroll
  for (int nt = 0; nt < NTW; ++nt) lacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Wavefront w fetches raw pieces w, w + 4, ... of the block (K pieces first, then V).
  struct Raw {
    u32x4 r[PER];
    float vs;
  };
  auto stage_load = [&](Raw &raw, const BlockMeta &bm) {
    const int64_t tile_a = (static_cast<int64_t>(bm.pid_a) * sh.page_tiles + g);
    const int64_t tile_b = (static_cast<int64_t>(bm.pid_b) * sh.page_tiles + g);
    const char *kp = kpool + (m16 < 8 ? tile_a : tile_b) * TILE_BYTES + k_lane_off;
    const char *vp = vpool + (jj < 2 ? tile_a : tile_b) * TILE_BYTES + v_lane_off;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      const int idx = k * 4 + w;  // wave-uniform
      const char *src = idx < RK ? kp + (idx / (RK / 2)) * (TILE_BYTES / 2) + (idx % (RK / 2)) * 512
                                 : vp + (idx - RK) * 512;
      raw.r[k] = load_kv(src);
    }
    raw.vs = FP8 ? fminf(p.v_scale[(jj < 2 ? bm.pid_a : bm.pid_b) * sh.Hkv + g], kMaxVScaleF16) : 1.f;
  };
  auto stage_store = [&](const Raw &raw, int buf) {
    u32x4 *dst = img + buf * (NI * 64) + lane;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      const int idx = k * 4 + w;
      if (FP8) {
        if (idx < RK) {
          dst[(2 * idx) * 64] = __builtin_bit_cast(u32x4, fp8x8_to_bf16x8(raw.r[k][0], raw.r[k][1]));
          dst[(2 * idx + 1) * 64] = __builtin_bit_cast(u32x4, fp8x8_to_bf16x8(raw.r[k][2], raw.r[k][3]));
        } else {
          dst[(2 * idx) * 64] = fp8x8_to_f16x8(raw.r[k][0], raw.r[k][1], raw.vs);
          dst[(2 * idx + 1) * 64] = fp8x8_to_f16x8(raw.r[k][2], raw.r[k][3], raw.vs);
        }
      } else {
        dst[idx * 64] = raw.r[k];  // bf16 pool: K is a bf16 and V an fp16 operand image as stored
      }
    }
  };
  auto compute = [&](int b, const BlockMeta &bm) {
    if (!has_rows) return;
    const u32x4 *src = img + (b & 1) * (NI * 64) + lane;
    bf16x8 kf[2][D / 32];
    f16x8 vh[D / 16];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int s = 0; s < D / 32; ++s)
        kf[t][s] = __builtin_bit_cast(bf16x8, src[(t * (D / 32) + s) * 64]);
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) vh[dt] = __builtin_bit_cast(f16x8, src[(NKI + dt) * 64]);
    const int valid_a = bm.vp_a & 127, valid_b = bm.vp_b & 127;
    float c = p.scale_log2;
    if (FP8) c *= fmaxf(p.k_scale[(jj < 2 ? bm.pid_a : bm.pid_b) * sh.Hkv + g], kMinKScale);
    block_math_f16<FP8, TREE, D, NTW>(st.qf, st.limit, st.qidx, st.dmask, st.o, st.m, lacc, kf, vh,
                                task_masked || valid_b == 0, jj < 2 ? valid_a : valid_b,
                                jj < 2 ? (bm.vp_a >> 7) : (bm.vp_b >> 7), c);
  };
  auto meta = [&](int b) { return load_block_meta(p.pg_rec, cur, b < nblk ? b : nblk - 1); };

  // LDS holds block b while it is computed; the pieces of block b+1 are requested before the
  // computation and moved to the other LDS buffer after it.
  Raw x;
  BlockMeta bm = meta(0);
  stage_load(x, bm);
  stage_store(x, 0);
  __syncthreads();
  for (int b = 0; b < nblk; ++b) {
    const bool more = b + 1 < nblk;  // uniform over the workgroup
    const BlockMeta nbm = meta(b + 1);
    if (more) stage_load(x, nbm);
    compute(b, bm);
    if (more) stage_store(x, (b + 1) & 1);
    bm = nbm;
    __syncthreads();
  }
  // The operand images are dead after the last barrier; the same LDS now serves the transposes.
  if (has_rows) {
    float m_out[NTW], l_out[NTW];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
      m_out[nt] = FP8 ? st.m[nt] : st.m[nt] * p.scale_log2;
      l_out[nt] = lacc[nt][0];
    }
    finish_rows<D, NTW, false>(p, sh, cur, row_base, st.o, m_out, l_out, st.qtok,
                               lds + w * stage_floats<D>());
  }
}

// ---- tree-walk kernel: one workgroup carries a block of query rows from the root to the leaves --
// A work item is a row block (up to NW = 4 or 8 wavefronts x 16 * NTW rows of the requested nodes below one
// root, neighbours in the tree next to each other) and a kv head.  Its block list covers every
// page on the rows' paths exactly once, each block with the range of rows whose path contains it.
// Phase 1 walks the blocks whose rows span several wavefronts: the workgroup fetches each block
// once into LDS operand images (as the cooperative kernel does) and every wavefront contracts it
// with the row tiles inside the range.  Phase 2: every wavefront streams the blocks that only its
// own rows need straight into registers.  The softmax state (m, l, o) of a row stays in registers
// from the first block to the last, so the only global writes are the finished output rows.
struct WalkBlock {
  int pid_a, vp_a, pid_b, vp_b, rows, flags;
  float ka, kb, va, vb;  // fp8: K and V scales of pages a and b for the item's kv head; else unused
};

__device__ __forceinline__ float sload_f(const float *base, int64_t idx) {
  typedef const float __attribute__((address_space(4))) const_f32;
  return ((const_f32 *)(uintptr_t)base)[idx];
}

// The record of a block and, for fp8, the page scales it will need.  Workgroups whose whole
// block list fits (kWalkRecCap blocks) copy it into LDS once, at the start, with ordinary vector
// loads, and read records from there: a scalar load inside the loop misses the scalar cache every
// other record and, because scalar loads return out of order, the next LDS wait of the wavefront
// becomes a wait for that miss -- measured at ~1.4 us per block.  Longer lists fall back to the
// scalar path, requested one or two blocks ahead.
constexpr int kWalkRecCap = 256;

template <bool FP8>
__device__ __forceinline__ WalkBlock load_walk_block(const WalkArgs &p, int idx, int g, int Hkv,
                                                     bool in_lds, const int32_t *rec, const float *scl,
                                                     int first) {
  WalkBlock b;
  if (in_lds) {
    const int at = uniform(idx) - first;
    const u32x4 lo = *reinterpret_cast<const u32x4 *>(rec + at * 8);
    const u32x2 hi = *reinterpret_cast<const u32x2 *>(rec + at * 8 + 4);
    b.pid_a = uniform(static_cast<int>(lo[0]));
    b.vp_a = uniform(static_cast<int>(lo[1]));
    b.pid_b = uniform(static_cast<int>(lo[2]));
    b.vp_b = uniform(static_cast<int>(lo[3]));
    b.rows = uniform(static_cast<int>(hi[0]));
    b.flags = uniform(static_cast<int>(hi[1]));
    if (FP8) {
      const f32x4 sc = *reinterpret_cast<const f32x4 *>(scl + at * 4);
      b.ka = fmaxf(sc[0], kMinKScale);
      b.kb = fmaxf(sc[1], kMinKScale);
      b.va = fminf(sc[2], kMaxVScaleF16);
      b.vb = fminf(sc[3], kMaxVScaleF16);
    } else {
      b.ka = b.kb = b.va = b.vb = 1.f;
    }
    return b;
  }
  const int64_t r = static_cast<int64_t>(uniform(idx)) * 8;
  b.pid_a = sload(p.blocks, r + 0);
  b.vp_a = sload(p.blocks, r + 1);
  b.pid_b = sload(p.blocks, r + 2);
  b.vp_b = sload(p.blocks, r + 3);
  b.rows = sload(p.blocks, r + 4);
  b.flags = sload(p.blocks, r + 5);
  if (FP8) {
    const int64_t ia = static_cast<int64_t>(b.pid_a) * Hkv + g, ib = static_cast<int64_t>(b.pid_b) * Hkv + g;
    b.ka = fmaxf(sload_f(p.k_scale, ia), kMinKScale);
    b.kb = fmaxf(sload_f(p.k_scale, ib), kMinKScale);
    b.va = fminf(sload_f(p.v_scale, ia), kMaxVScaleF16);
    b.vb = fminf(sload_f(p.v_scale, ib), kMaxVScaleF16);
  } else {
    b.ka = b.kb = b.va = b.vb = 1.f;
  }
  return b;
}

// Scores of one 32-token block for the row tiles that intersect the wave-relative row range
// [lo, hi): S^T = K Q^T (see block_math for the operand layout).
template <int D, int NT>
__device__ __forceinline__ void walk_scores(const bf16x8 (&qf)[NT][D / 32], const bf16x8 (&kf)[2][D / 32],
                                            int lo, int hi, f32x4 (&sa)[NT], f32x4 (&sb)[NT]) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (nt * 16 >= hi || nt * 16 + 16 <= lo) continue;  // wave-uniform
    f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
      a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][s], qf[nt][s], a, 0, 0, 0);
      b = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][s], qf[nt][s], b, 0, 0, 0);
    }
    sa[nt] = a;
    sb[nt] = b;
  }
}

// Online softmax and O^T += V^T P^T for the same tiles; P rounded to fp16, row sums by MFMA
// against ones (see block_math_f16).  Rows of a tile outside [lo, hi) see nothing of the block.
template <bool FP8, bool TREE, int D, int NT>
__device__ __forceinline__ void walk_softmax_pv(const int (&limit)[NT], const int (&qidx)[NT],
                                                const uint32_t (&dmask)[NT], f32x4 (&o)[NT][D / 16],
                                                float (&m)[NT], f32x4 (&lacc)[NT],
                                                const f32x4 (&sa)[NT], const f32x4 (&sb)[NT],
                                                const f16x8 (&vh)[D / 16], bool tok_masked,
                                                int valid_l, int pos_l, float c, float slack, int lo,
                                                int hi) {
  const int lane = threadIdx.x & 63, m16 = lane & 15, jj = lane >> 4;
  const _Float16 one = static_cast<_Float16>(1.0f);
  const f16x8 ones = {one, one, one, one, one, one, one, one};
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (nt * 16 >= hi || nt * 16 + 16 <= lo) continue;  // wave-uniform
    const bool partial_tile = lo > nt * 16 || hi < nt * 16 + 16;
    // Scores stay raw; scale and subtraction of the reference fuse into one FMA per score.  With
    // one scale for the whole path (bf16 KV) the reference m is kept on raw scores; with a scale
    // per page (fp8 KV) it is kept in scaled units (log2 e folded in), and the largest scaled score
    // of the lane is c * the largest raw one (c > 0, and rounding is monotonic).
    float x[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[i] = sa[nt][i];
      x[4 + i] = sb[nt][i];
    }
    if (tok_masked || partial_tile) {
      const int row = nt * 16 + m16;
      const bool row_in = row >= lo && row < hi;
      if (TREE) {
        // Draft tree: positions below base = T - q_len are visible, position base + k iff bit k of
        // the row's mask is set.  The lane's 8 tokens start at relative position rel; shifting
        // {mask, 32 ones} right by rel + 32 puts their visibility into the low 8 bits.
        const int base = limit[nt] - 1 - qidx[nt];
        const int first = 8 * (jj & 1);
        const int sh = pos_l + first - base + 32;
        const uint64_t bits = (static_cast<uint64_t>(dmask[nt]) << 32) | 0xffffffffull;
        uint32_t vm = sh <= 0 ? 0xffu : (sh >= 64 ? 0u : static_cast<uint32_t>(bits >> sh) & 0xffu);
        const int have = valid_l - first;  // tokens of the lane's 8 that exist
        vm = row_in ? vm : 0u;
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = (i < have && ((vm >> i) & 1u)) ? x[i] : kNegInf;
      } else {
        int vis = limit[nt] - pos_l;
        vis = vis < valid_l ? vis : valid_l;
        vis -= 8 * (jj & 1);
        vis = row_in ? vis : 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = i < vis ? x[i] : kNegInf;
      }
    }
    const float mx8_raw = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                                fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    const float mx8 = FP8 ? mx8_raw * c : mx8_raw;
    // Lazy reference: m is the value the row's weights are taken relative to, not its exact
    // running maximum.  It moves (and o and l are rescaled) only when a score of the row exceeds it
    // by more than `slack` (2^8 in weight); until then weights are at most 2^8, which fp16 and
    // the fp32 sums hold.  The decision is taken per row from the row's own scores, so a row's
    // result does not depend on its neighbours in the tile; most blocks skip the cross-lane
    // maximum and the rescaling altogether.  m starts at kWalkMInit (finite, far below any score).
    if (__any(mx8 > m[nt] + slack)) {
      const float rmax = row_group_max(mx8);
      const float m_new = rmax > m[nt] + slack ? rmax : m[nt];
      const float alpha = fast_exp2(FP8 ? m[nt] - m_new : (m[nt] - m_new) * c);
      m[nt] = m_new;
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) o[nt][dt] *= alpha;
      lacc[nt] *= alpha;
    }
    float pr[8];
    if (FP8) {
      const float neg_m = -m[nt];
#pragma unroll
      for (int i = 0; i < 8; ++i) pr[i] = fast_exp2(__builtin_fmaf(x[i], c, neg_m));
    } else {
      const float mc = m[nt] * c;
#pragma unroll
      for (int i = 0; i < 8; ++i) pr[i] = fast_exp2(__builtin_fmaf(x[i], c, -mc));
    }
    u32x4 pw;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      pw[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(pr[2 * i], pr[2 * i + 1]));
    const f16x8 ph = __builtin_bit_cast(f16x8, pw);
    lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, ph, lacc[nt], 0, 0, 0);
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
      o[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vh[dt], ph, o[nt][dt], 0, 0, 0);
  }
}

// Normalise and store the finished rows of one wavefront.  As in finish_rows the tile goes through
// a wave-private LDS area so that every store instruction writes whole 4 * D byte rows.
template <int D, int NT>
__device__ __forceinline__ void walk_write_rows(float *out, float *lse, const Shape &sh, int g, int rows,
                                                f32x4 (&o)[NT][D / 16], const float (&m_log2)[NT],
                                                const f32x4 (&lacc)[NT], const int (&qtok)[NT], float *my) {
  constexpr int kRowPad = D + 4;
  constexpr int kLanesPerRow = D / 4;
  constexpr int kRowsPerInst = 64 / kLanesPerRow;
  const int lane = threadIdx.x & 63, m16 = lane & 15, jj = lane >> 4;
  const int sub = lane / kLanesPerRow, piece = lane % kLanesPerRow;
  const int G = sh.G;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int r0w = nt * 16;
    if (r0w >= rows) break;  // wave-uniform
    const bool row_ok = r0w + m16 < rows;
    const float l = lacc[nt][0];
    const float inv = 1.0f / l;
    const int64_t dst_row = static_cast<int64_t>(qtok[nt]) * sh.Hq + g * G + (r0w + m16) % G;
    if (row_ok && jj == 0 && lse) lse[dst_row] = (m_log2[nt] + __builtin_log2f(l)) * 0.6931471805599453f;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
      *reinterpret_cast<f32x4 *>(my + m16 * kRowPad + dt * 16 + jj * 4) = o[nt][dt] * inv;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < 16 / kRowsPerInst; ++i) {
      const int row = i * kRowsPerInst + sub;
      const f32x4 v = *reinterpret_cast<const f32x4 *>(my + row * kRowPad + piece * 4);
      const int lo32 = __shfl(static_cast<int>(dst_row & 0xffffffff), row);
      const int hi32 = __shfl(static_cast<int>(dst_row >> 32), row);
      const int64_t drow = (static_cast<int64_t>(hi32) << 32) | static_cast<uint32_t>(lo32);
      if (r0w + row < rows) *reinterpret_cast<f32x4 *>(out + drow * D + piece * 4) = v;
    }
  }
}

// KS = 1: wavefront w holds rows w * C .. of the row block.  KS = 2 (NW = 4): the lists are made
// for LW = 2 wavefronts of rows; wavefronts w and w + 2 hold the same rows and split the row
// block's path between them -- shared blocks alternate between the two halves of the workgroup
// (two blocks per barrier, each staged by the pair that computes on it), a list wavefront's private
// blocks alternate likewise -- and at the end the upper pair hands its softmax state to the lower
// one through LDS.  Per block a wavefront then works on twice the rows, so half as many operand
// images cross the LDS per row, and a row block's longest path takes half as many steps.
template <int KV, int D, int NTW, int NW, bool TREE, int KS = 1>
__global__ __launch_bounds__(64 * NW, (NW == 4 && NTW <= 2) ? 2 : 1) void spex_tree_walk_kernel(WalkArgs p, Shape sh) {
  constexpr bool FP8 = KV == kFP8;
  constexpr int ESZ = FP8 ? 1 : 2;
  constexpr int TILE_BYTES = 16 * D * ESZ;
  constexpr int C = 16 * NTW;              // rows per wavefront
  constexpr int NKI = 2 * (D / 32);        // K operand images per block
  constexpr int NI = NKI + D / 16;         // all operand images per block (1 KiB each)
  constexpr int RAW = FP8 ? NI / 2 : NI;   // 1 KiB global loads per block
  constexpr int RK = FP8 ? NKI / 2 : NKI;  // of which K
  static_assert(KS == 1 || (KS == 2 && NW == 4), "the path is split between the two halves of four wavefronts");
  constexpr int LW = NW / KS;               // wavefronts the lists were made for (each holds C rows)
  constexpr int PER = (RAW + LW - 1) / LW;  // global loads per wavefront and block in the shared phase
  constexpr bool kEven = RAW % LW == 0;     // else the last wavefronts have no piece to fetch
  // When K and V each split evenly over the wavefronts, a wavefront's first KPER pieces are K and
  // the others V whatever its index, so the widening code is chosen at compile time instead of
  // being run for every piece and selected away.
  constexpr bool kSplitKV = RK % LW == 0 && (RAW - RK) % LW == 0;
  constexpr int KPER = kSplitKV ? RK / LW : 0;
  constexpr int kItemInts = LW <= 4 ? 16 : 32;
  constexpr int kImgFloats = NI * 64 * 4;
  // KS = 2: what a wavefront of the upper pair hands over at the end: o, l (as accumulator) and m
  constexpr int kFoldWaveFloats = NTW * (D / 16) * 256 + NTW * 256 + NTW * 64;
  // output staging of the wavefronts that write rows (all, or the lower pair), then the hand-over area
  constexpr int kTailFloats = LW * stage_floats<D>() + (KS == 2 ? LW * kFoldWaveFloats : 0);
  constexpr int kLdsFloats = 2 * KS * kImgFloats > kTailFloats ? 2 * KS * kImgFloats : kTailFloats;
  __shared__ __attribute__((aligned(16))) float lds[kLdsFloats];
  __shared__ __attribute__((aligned(16))) int32_t rec_lds[kWalkRecCap * 8];
  __shared__ __attribute__((aligned(16))) float scl_lds[FP8 ? kWalkRecCap * 4 : 4];
  u32x4 *img = reinterpret_cast<u32x4 *>(lds);  // [buf][image][lane]

  const int lane = threadIdx.x & 63, m16 = lane & 15, jj = lane >> 4;
  const int w = uniform(threadIdx.x >> 6);
  const int64_t ir = static_cast<int64_t>(blockIdx.x) * kItemInts;
  const int g = sload(p.items, ir + 0);
  const int blk_begin = sload(p.items, ir + 1);
  const int n_shared = sload(p.items, ir + 2);
  // per wavefront: private blocks | room << 16; a wavefront's records are followed by the unused
  // part of its room, so n_all spans records that no wavefront walks
  const int rw = KS == 1 ? w : w % LW;  // the list wavefront whose rows this wavefront holds
  const int ks = KS == 1 ? 0 : w / LW;  // which part of the path it walks
  int n_all = n_shared, n_priv = 0, priv_begin = blk_begin + n_shared;
#pragma unroll
  for (int v = 0; v < LW; ++v) {
    const uint32_t packed = static_cast<uint32_t>(sload(p.items, ir + 3 + v));
    const int npv = static_cast<int>(packed & 0xffffu), room = static_cast<int>(packed >> 16);
    n_all += room;
    n_priv = v == rw ? npv : n_priv;
    priv_begin += v < rw ? room : 0;
  }
  if (n_all == 0) return;  // padding item (whole workgroup)
  if (KS == 2) n_priv = (n_priv + 1 - ks) >> 1;  // private blocks ks, ks + 2, .. of the list wavefront
  const bool rec_in_lds = n_all <= kWalkRecCap;  // uniform over the workgroup
  if (rec_in_lds) {
    const u32x4 *src = reinterpret_cast<const u32x4 *>(p.blocks + static_cast<int64_t>(blk_begin) * 8);
    for (int i = threadIdx.x; i < n_all * 2; i += 64 * NW) reinterpret_cast<u32x4 *>(rec_lds)[i] = src[i];
    if (FP8) {
      __syncthreads();
      for (int i = threadIdx.x; i < n_all * 4; i += 64 * NW) {
        const int page = rec_lds[(i >> 2) * 8 + ((i & 1) ? 2 : 0)];
        scl_lds[i] = ((i & 2) ? p.v_scale : p.k_scale)[static_cast<int64_t>(page) * sh.Hkv + g];
      }
    }
    __syncthreads();
  }
  const int qt_begin = sload(p.items, ir + 3 + LW + rw);
  const int qt_count = sload(p.items, ir + 3 + 2 * LW + rw);
  const int rows = qt_count * sh.G;
  const bool has_rows = rows > 0;
  const char *kpool = static_cast<const char *>(p.k_pool);
  const char *vpool = static_cast<const char *>(p.v_pool);
  const int k_lane_off = jj * 128 + (m16 & 7) * 16;
  const int v_lane_off = (jj & 1) * 256 + m16 * 16;

  // how far a score may exceed a row's softmax reference before the reference moves (log2 units: 8)
  const float slack = FP8 ? 8.f : 8.f / p.scale_log2;
  // ---- rows of this wavefront
  bf16x8 qf[NTW][D / 32];
  int limit[NTW], qtok[NTW], qidx[NTW];
  uint32_t dmask[NTW];
  f32x4 o[NTW][D / 16], lacc[NTW];
  float m[NTW];
#pragma unroll
  for (int nt = 0; nt < NTW; ++nt) {
    const int r = nt * 16 + m16;
    limit[nt] = INT_MAX;
    qtok[nt] = 0;
    qidx[nt] = 0;
    dmask[nt] = 0;
    m[nt] = kWalkMInit;
    lacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) o[nt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (r < rows) {
      const int2 qr = *reinterpret_cast<const int2 *>(p.qt_rec + 2 * (qt_begin + r / sh.G));
      qtok[nt] = qr.x;
      limit[nt] = qr.y;
      if (TREE) {
        const int2 dm = *reinterpret_cast<const int2 *>(p.qt_mask + 2 * qr.x);
        qidx[nt] = dm.x;
        dmask[nt] = static_cast<uint32_t>(dm.y);
      }
      const uint16_t *qp = static_cast<const uint16_t *>(p.q) +
                           (static_cast<int64_t>(qr.x) * sh.Hq + g * sh.G + r % sh.G) * D + jj * 8;
#pragma unroll
      for (int s = 0; s < D / 32; ++s)
        qf[nt][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(qp + s * 32));
    } else {
#pragma unroll
      for (int s = 0; s < D / 32; ++s) qf[nt][s] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
    }
  }

  // The two phases run in either order (the online softmax does not care).  The shared phase is
  // bound by the matrix cores and LDS, the private phase by memory; workgroups that start together
  // would all be in the same phase at the same time, so every other pair of workgroups of an XCD
  // (workgroup n runs on XCD n % 8; the pair n, n + 8 are row blocks of one root and kv head when
  // a root has several, and stay in step so that one finds the other's shared blocks in L2),
  // alternating again with every round of 256, takes its private blocks first: the loop below
  // then runs twice, one phase per turn.  Not with four row tiles per wavefront (registers).
  constexpr bool kStagger = NTW <= 2 && KS == 1;
  const bool private_first = kStagger && (((blockIdx.x >> 4) ^ (blockIdx.x >> 8)) & 1) != 0;
#pragma nounroll
  for (int ph = 0; ph < (kStagger ? 2 : 1); ++ph) {
  const bool run_shared = !kStagger || (ph == 0) != private_first;
  const bool run_private = !kStagger || (ph == 0) == private_first;
  // ---- phase 1: blocks shared by several wavefronts, through LDS
  if (run_shared && n_shared > 0) {
    struct Raw {
      u32x4 r[PER];
      float vs;
    };
    // A block that another row block reads too (flag bit 1) is loaded with the ordinary cache
    // policy, so that the second reader finds it in the L2 of the XCD both run on; everything
    // else is streamed.
    auto stage_load = [&](Raw &raw, const WalkBlock &bm) {
      const int64_t tile_a = (static_cast<int64_t>(bm.pid_a) * sh.page_tiles + g);
      const int64_t tile_b = (static_cast<int64_t>(bm.pid_b) * sh.page_tiles + g);
      const char *kp = kpool + (m16 < 8 ? tile_a : tile_b) * TILE_BYTES + k_lane_off;
      const char *vp = vpool + (jj < 2 ? tile_a : tile_b) * TILE_BYTES + v_lane_off;
#pragma unroll
      for (int k = 0; k < PER; ++k) {
        const bool is_k = kSplitKV ? k < KPER : k * LW + rw < RK;
        const int idx = kSplitKV ? (k < KPER ? k * LW + rw : RK + (k - KPER) * LW + rw) : k * LW + rw;  // wave-uniform
        if (!kEven && idx >= RAW) continue;
        const char *src = is_k ? kp + (idx / (RK / 2)) * (TILE_BYTES / 2) + (idx % (RK / 2)) * 512
                               : vp + (idx - RK) * 512;
        raw.r[k] = (bm.flags & 2) ? *reinterpret_cast<const u32x4 *>(src) : load_kv(src);
      }
      raw.vs = jj < 2 ? bm.va : bm.vb;
    };
    auto stage_store = [&](const Raw &raw, int buf) {
      u32x4 *dst = img + (buf * KS + ks) * (NI * 64) + lane;
#pragma unroll
      for (int k = 0; k < PER; ++k) {
        const bool is_k = kSplitKV ? k < KPER : k * LW + rw < RK;
        const int idx = kSplitKV ? (k < KPER ? k * LW + rw : RK + (k - KPER) * LW + rw) : k * LW + rw;
        if (!kEven && idx >= RAW) continue;
        if (FP8) {
          if (is_k) {
            dst[(2 * idx) * 64] = __builtin_bit_cast(u32x4, fp8x8_to_bf16x8(raw.r[k][0], raw.r[k][1]));
            dst[(2 * idx + 1) * 64] = __builtin_bit_cast(u32x4, fp8x8_to_bf16x8(raw.r[k][2], raw.r[k][3]));
          } else {
            dst[(2 * idx) * 64] = fp8x8_to_f16x8(raw.r[k][0], raw.r[k][1], raw.vs);
            dst[(2 * idx + 1) * 64] = fp8x8_to_f16x8(raw.r[k][2], raw.r[k][3], raw.vs);
          }
        } else {
          dst[idx * 64] = raw.r[k];  // bf16 pool: K is a bf16 and V an fp16 operand image as stored
        }
      }
    };
    auto compute = [&](int b, const WalkBlock &bm) {
      const int lo = (bm.rows & 0xffff) - rw * C, hi = (bm.rows >> 16) - rw * C;
      if (!has_rows || hi <= 0 || lo >= C) return;  // wave-uniform: none of this wavefront's rows
      const u32x4 *src = img + ((b & 1) * KS + ks) * (NI * 64) + lane;
      const float c = p.scale_log2 * (jj < 2 ? bm.ka : bm.kb);
      f32x4 sa[NTW], sb[NTW];
      {
        bf16x8 kf[2][D / 32];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int s = 0; s < D / 32; ++s)
            kf[t][s] = __builtin_bit_cast(bf16x8, src[(t * (D / 32) + s) * 64]);
        walk_scores<D, NTW>(qf, kf, lo, hi, sa, sb);
      }
      // The V images are fetched only now, into the registers the K images have left, and their
      // LDS latency passes under the softmax arithmetic.
      __builtin_amdgcn_sched_barrier(0);
      f16x8 vh[D / 16];
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) vh[dt] = __builtin_bit_cast(f16x8, src[(NKI + dt) * 64]);
      walk_softmax_pv<FP8, TREE, D, NTW>(limit, qidx, dmask, o, m, lacc, sa, sb, vh, (bm.flags & 1) != 0,
                                   (jj < 2 ? bm.vp_a : bm.vp_b) & 127, (jj < 2 ? bm.vp_a : bm.vp_b) >> 7,
                                   c, slack, lo, hi);
    };
    auto meta = [&](int b) {
      return load_walk_block<FP8>(p, blk_begin + (b < n_shared ? b : n_shared - 1), g, sh.Hkv, rec_in_lds,
                                  rec_lds, scl_lds, blk_begin);
    };

    // Software pipeline, PF blocks deep: while block c is computed from one LDS buffer, blocks
    // c+1 .. c+PF-1 are already in (or on their way to) registers, block c+1 moves to the other
    // LDS buffer after the computation, and the global loads of block c+PF are issued.  The loads
    // are unconditional (indices past the end repeat the last block) because a load issued on
    // one path only would make every later wait a wait for all outstanding loads.  (PF = 4 was
    // measured for one row tile per wavefront and for fp8 with two, where the registers allow it:
    // no gain.)
    if (KS == 2) {
      // Two blocks per barrier: step s holds blocks 2 s (lower pair of wavefronts) and 2 s + 1
      // (upper pair); each pair stages and computes its own.  The loads of step s + 1 are in
      // flight while step s is computed.  With an odd number of blocks the upper pair's last
      // step only moves a copy of the last block.
      const int n_steps = (n_shared + 1) >> 1;
      Raw x;
      WalkBlock cur = meta(ks);
      stage_load(x, cur);
      stage_store(x, 0);
      __syncthreads();
      for (int st = 0; st < n_steps; ++st) {
        const WalkBlock nxt = meta(2 * (st + 1) + ks);
        stage_load(x, nxt);
        if (2 * st + ks < n_shared) compute(st, cur);
        stage_store(x, (st + 1) & 1);
        cur = nxt;
        __syncthreads();
      }
    }
    constexpr int PF = 2;
    Raw x[PF];
    WalkBlock bmq[PF];
    if (KS == 1) {
#pragma unroll
      for (int k = 0; k < PF; ++k) {
        bmq[k] = meta(k);
        stage_load(x[k], bmq[k]);
      }
      stage_store(x[0], 0);
      __syncthreads();
    }
    for (int b = 0; KS == 1 && b < n_shared; b += PF) {
#pragma unroll
      for (int k = 0; k < PF; ++k) {
        const int c = b + k;             // block computed in this step; x[k] is free again
        const WalkBlock cur = bmq[k];
        bmq[k] = meta(c + PF);
        stage_load(x[k], bmq[k]);
        // no early exit from the group of PF steps: a step past the end only moves (clamped)
        // data, so that every path through the loop body issues and waits for the same loads
        if (c < n_shared) compute(c, cur);
        // Unconditional: after the last block this stores a copy of that block (the loads are
        // clamped) into the buffer nobody reads any more.  A store skipped on one path would leave
        // its loads unwaited there, and the compiler would then drain every outstanding load at
        // the top of the loop -- the prefetch of the next block included.
        stage_store(x[(k + 1) % PF], (c + 1) & 1);
        __syncthreads();
      }
    }
  }

  // ---- phase 2: blocks of this wavefront alone, straight into registers
  if (run_private && has_rows && n_priv > 0) {
    constexpr int NK = FP8 ? D / 64 : D / 32;  // 128-bit loads per K half-tile
    constexpr int NV = FP8 ? D / 32 : D / 16;
    auto issue_k = [&](u32x4 (&kr)[2][NK], const WalkBlock &bm) {
      const int64_t tile_a = (static_cast<int64_t>(bm.pid_a) * sh.page_tiles + g);
      const int64_t tile_b = (static_cast<int64_t>(bm.pid_b) * sh.page_tiles + g);
      const char *kp = kpool + (m16 < 8 ? tile_a : tile_b) * TILE_BYTES + k_lane_off;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int s = 0; s < NK; ++s) kr[t][s] = load_kv(kp + t * (TILE_BYTES / 2) + s * 512);
    };
    auto issue_v = [&](u32x4 (&vr)[NV], const WalkBlock &bm) {
      const int64_t tile_a = (static_cast<int64_t>(bm.pid_a) * sh.page_tiles + g);
      const int64_t tile_b = (static_cast<int64_t>(bm.pid_b) * sh.page_tiles + g);
      const char *vp = vpool + (jj < 2 ? tile_a : tile_b) * TILE_BYTES + v_lane_off;
#pragma unroll
      for (int s = 0; s < NV; ++s) vr[s] = load_kv(vp + s * 512);
    };
    // One block: scores from the K registers, which are then refilled (with the block `refill`,
    // if `more`) while the softmax runs; the V registers are refilled as soon as they are widened.
    auto step = [&](u32x4 (&kr)[2][NK], u32x4 (&vr)[NV], const WalkBlock &bm, const WalkBlock &refill, bool more) {
      const int lo = (bm.rows & 0xffff) - rw * C, hi = (bm.rows >> 16) - rw * C;
      const float c = p.scale_log2 * (jj < 2 ? bm.ka : bm.kb), vs = jj < 2 ? bm.va : bm.vb;
      bf16x8 kf[2][D / 32];
      if (FP8) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int s = 0; s < D / 64; ++s) {
            kf[t][2 * s] = fp8x8_to_bf16x8(kr[t][s][0], kr[t][s][1]);
            kf[t][2 * s + 1] = fp8x8_to_bf16x8(kr[t][s][2], kr[t][s][3]);
          }
      } else {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int s = 0; s < D / 32; ++s) kf[t][s] = __builtin_bit_cast(bf16x8, kr[t][s]);
      }
      f32x4 sa[NTW], sb[NTW];
      walk_scores<D, NTW>(qf, kf, lo, hi, sa, sb);
      if (more) issue_k(kr, refill);
      f16x8 vh[D / 16];
      if (FP8) {
#pragma unroll
        for (int s = 0; s < D / 32; ++s) {
          vh[2 * s] = __builtin_bit_cast(f16x8, fp8x8_to_f16x8(vr[s][0], vr[s][1], vs));
          vh[2 * s + 1] = __builtin_bit_cast(f16x8, fp8x8_to_f16x8(vr[s][2], vr[s][3], vs));
        }
      } else {
#pragma unroll
        for (int s = 0; s < D / 16; ++s) vh[s] = __builtin_bit_cast(f16x8, vr[s]);
      }
      if (more) issue_v(vr, refill);
      walk_softmax_pv<FP8, TREE, D, NTW>(limit, qidx, dmask, o, m, lacc, sa, sb, vh, (bm.flags & 1) != 0,
                                   (jj < 2 ? bm.vp_a : bm.vp_b) & 127, (jj < 2 ? bm.vp_a : bm.vp_b) >> 7,
                                   c, slack, lo, hi);
    };
    // the j-th private block of this wavefront (past the end: the last one)
    auto rec_at = [&](int j) {
      const int jc = j < n_priv ? j : n_priv - 1;
      return load_walk_block<FP8>(p, priv_begin + ks + KS * jc, g, sh.Hkv, rec_in_lds, rec_lds, scl_lds, blk_begin);
    };
    {
      u32x4 kr[2][NK], vr[NV];
      WalkBlock cur = rec_at(0);
      WalkBlock nxt = rec_at(1);
      issue_k(kr, cur);
      issue_v(vr, cur);
      for (int i = 0; i + 1 < n_priv; ++i) {
        const WalkBlock nxt2 = rec_at(i + 2);
        step(kr, vr, cur, nxt, true);
        cur = nxt;
        nxt = nxt2;
      }
      step(kr, vr, cur, cur, false);
    }
  }
  }  // phases

  // ---- KS = 2: the upper pair hands its state to the lower pair, which folds it into its own
  // (log-sum-exp rule on the two references).  The LDS images are dead after the last barrier of
  // phase 1, and phase 2 does not touch LDS, so the hand-over area may lie behind the output staging.
  if (KS == 2) {
    float *fold = lds + LW * stage_floats<D>() + rw * kFoldWaveFloats;
    f32x4 *fo = reinterpret_cast<f32x4 *>(fold) + lane;                               // [nt][dt][lane]
    f32x4 *fl = reinterpret_cast<f32x4 *>(fold + NTW * (D / 16) * 256) + lane;         // [nt][lane]
    float *fm = fold + NTW * (D / 16) * 256 + NTW * 256 + lane;                        // [nt][lane]
    if (has_rows && ks == 1) {
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) {
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) fo[(nt * (D / 16) + dt) * 64] = o[nt][dt];
        fl[nt * 64] = lacc[nt];
        fm[nt * 64] = m[nt];
      }
    }
    __syncthreads();
    if (has_rows && ks == 0) {
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) {
        const float m1 = fm[nt * 64];
        const float mn = fmaxf(m[nt], m1);
        // a side that saw nothing still has the (finite) start value of m: its factor is 0, or 1
        // where neither saw anything (rows past the end of the wavefront's rows)
        const float a0 = fast_exp2(FP8 ? m[nt] - mn : (m[nt] - mn) * p.scale_log2);
        const float a1 = fast_exp2(FP8 ? m1 - mn : (m1 - mn) * p.scale_log2);
        m[nt] = mn;
        lacc[nt] = lacc[nt] * a0 + fl[nt * 64] * a1;
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) o[nt][dt] = o[nt][dt] * a0 + fo[(nt * (D / 16) + dt) * 64] * a1;
      }
    }
  }

  // ---- output.  The LDS images are dead after the last barrier of phase 1.
  if (has_rows && ks == 0) {
    float m_log2[NTW];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) m_log2[nt] = FP8 ? m[nt] : m[nt] * p.scale_log2;
    walk_write_rows<D, NTW>(p.out, p.lse, sh, g, rows, o, m_log2, lacc, qtok, lds + w * stage_floats<D>());
  }
}

// ---- generic attention (no matrix cores) ------------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// One wavefront per (work item, row): blockIdx.y strides over the item's rows.  Lane = token for
// the scores, lane = dim (d, d+64, ..) for the weighted sum.  The loops over dims and tokens fetch
// eight elements before they use them (in the same order as one at a time), so that a lane does not
// sit out a memory latency per element.
template <int KV, int QT, int LAYOUT>
__global__ __launch_bounds__(64) void spex_generic_attn_kernel(AttnArgs p, Shape sh, int rows_per_item) {
  constexpr int kU = 8;  // elements fetched before they are used
  __shared__ float qs[256];
  const int lane = threadIdx.x;
  const int32_t *rec = p.items + static_cast<int64_t>(blockIdx.x) * 8;
  const int pg_begin = rec[0];
  const int pg_count = rec[1];
  const int qt_begin = rec[2];
  const int qt_count = rec[3];
  const int pbase = rec[4];
  const int g = rec[6];
  const int row0 = rec[7];
  if (pg_count == 0) return;  // padding item
  const int D = sh.D, P = sh.P, G = sh.G;
  const int rows = qt_count * G;
  const int64_t tile_elems = static_cast<int64_t>(P) * D;
  const int n_tok_slots = pg_count * P;
  const int r_end = min(rows, row0 + rows_per_item);

  for (int r = row0 + static_cast<int>(blockIdx.y); r < r_end; r += static_cast<int>(gridDim.y)) {
    const int qt = p.qt_rec[2 * (qt_begin + r / G)];
    const int hh = r % G;
    const int limit = p.qt_rec[2 * (qt_begin + r / G) + 1];
    const int d_base = p.qt_mask ? limit - 1 - p.qt_mask[2 * qt] : 0;
    const uint32_t d_mask = p.qt_mask ? static_cast<uint32_t>(p.qt_mask[2 * qt + 1]) : 0u;
    const int64_t qbase = (static_cast<int64_t>(qt) * sh.Hq + g * G + hh) * D;
    __syncthreads();
    for (int d = lane; d < D; d += 64) qs[d] = load_elem<QT>(p.q, qbase + d);
    __syncthreads();

    float m = kNegInf, l = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int t0 = 0; t0 < n_tok_slots; t0 += 64) {
      const int ti = t0 + lane;
      const int e = pg_begin + ti / P;
      const int slot = ti % P;
      bool ok = ti < n_tok_slots;
      float s = kNegInf;
      if (ok) {
        const int vp = p.pg_rec[2 * e + 1];
        const int pos = (vp >> 7) + slot;
        bool seen = pos < limit;
        if (p.qt_mask) {  // draft tree: everything before the drafts, then the mask's bits
          const int rel = pos - d_base;
          seen = rel < 0 || (rel < 32 && ((d_mask >> rel) & 1u));
        }
        ok = slot < (vp & 127) && seen;
      }
      if (ok) {
        const int64_t tile = (static_cast<int64_t>(p.pg_rec[2 * e]) * sh.page_tiles + g);
        float dot = 0.f;
        int d = 0;
        for (; d + kU <= D; d += kU) {
          float kv[kU];
#pragma unroll
          for (int u = 0; u < kU; ++u)
            kv[u] = load_elem<KV>(p.k_pool, tile * tile_elems + k_offset<KV, LAYOUT>(slot, d + u, D));
#pragma unroll
          for (int u = 0; u < kU; ++u) dot += qs[d + u] * kv[u];
        }
        for (; d < D; ++d)
          dot += qs[d] * load_elem<KV>(p.k_pool, tile * tile_elems + k_offset<KV, LAYOUT>(slot, d, D));
        if (KV == kFP8) dot *= p.k_scale[p.pg_rec[2 * e] * sh.Hkv + g];
        s = dot * p.scale_log2;
      }
      const float m_new = fmaxf(m, wave_max(s));
      if (m_new == kNegInf) continue;
      const float alpha = fast_exp2(m - m_new);
      const float pw = ok ? fast_exp2(s - m_new) : 0.f;
      l = l * alpha + wave_sum(pw);
      m = m_new;
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[c] *= alpha;
      const int n_here = min(64, n_tok_slots - t0);
      for (int tb = 0; tb < n_here; tb += kU) {
        float wt[kU], vv[kU][4];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
          const int t = tb + u;
          const float pt = t < n_here ? __shfl(pw, t & 63) : 0.f;
          wt[u] = pt;
#pragma unroll
          for (int c = 0; c < 4; ++c) vv[u][c] = 0.f;
          if (pt == 0.f) continue;  // wave-uniform: pt is a broadcast value
          const int e2 = pg_begin + (t0 + t) / P;
          const int slot2 = (t0 + t) % P;
          const int64_t tile = (static_cast<int64_t>(p.pg_rec[2 * e2]) * sh.page_tiles + g);
          if (KV == kFP8) wt[u] = pt * p.v_scale[p.pg_rec[2 * e2] * sh.Hkv + g];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int d = lane + 64 * c;
            if (d < D) vv[u][c] = load_v_elem<KV, LAYOUT>(p.v_pool, tile * tile_elems + v_offset<KV, LAYOUT>(slot2, d, D));
          }
        }
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[c] += wt[u] * vv[u][c];
      }
    }
    const int64_t out_slot = static_cast<int64_t>(pbase) + static_cast<int64_t>(g) * rows + r;
    if (lane == 0) {
      p.part_ml[out_slot * 2] = m;
      p.part_ml[out_slot * 2 + 1] = l;
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int d = lane + 64 * c;
      if (d < D) p.part_o[out_slot * D + d] = acc[c];
    }
  }
}

// ---- merge -----------------------------------------------------------------------------------
// Thread = (query token, query head, VEC consecutive dims).
template <int VEC>
__global__ __launch_bounds__(256) void spex_lse_merge_kernel(MergeArgs a, Shape sh) {
  const int dv = sh.D / VEC;
  const int64_t tid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int64_t row = tid / dv;
  const int c = static_cast<int>(tid % dv);
  if (row >= static_cast<int64_t>(a.n_qtok) * sh.Hq) return;
  const int qt = a.qt_ids ? a.qt_ids[row / sh.Hq] : static_cast<int>(row / sh.Hq);
  const int h = static_cast<int>(row % sh.Hq);
  const int g = h / sh.G, hh = h % sh.G;
  const int e0 = a.part_indptr[qt], e1 = a.part_indptr[qt + 1];
  float m = kNegInf;
  for (int e = e0; e < e1; ++e) {
    const int64_t slot = static_cast<int64_t>(a.part_base[e]) + static_cast<int64_t>(g) * a.part_hstride[e] + hh;
    m = fmaxf(m, a.part_ml[slot * 2]);
  }
  float l = 0.f;
  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
  for (int e = e0; e < e1; ++e) {
    const int64_t slot = static_cast<int64_t>(a.part_base[e]) + static_cast<int64_t>(g) * a.part_hstride[e] + hh;
    const float mj = a.part_ml[slot * 2];
    const float lj = a.part_ml[slot * 2 + 1];
    if (lj == 0.f) continue;
    const float f = fast_exp2(mj - m);
    l += lj * f;
    const float *op = a.part_o + slot * sh.D + c * VEC;
    if (VEC == 4) {
      const f32x4 o = *reinterpret_cast<const f32x4 *>(op);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] += o[i] * f;
    } else {
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] += op[i] * f;
    }
  }
  const float inv = 1.0f / l;
  const int64_t orow = static_cast<int64_t>(qt) * sh.Hq + h;
  float *out = a.out + orow * sh.D + c * VEC;
  if (VEC == 4) {
    *reinterpret_cast<f32x4 *>(out) = f32x4{acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
  } else {
#pragma unroll
    for (int i = 0; i < VEC; ++i) out[i] = acc[i] * inv;
  }
  if (a.lse && c == 0) a.lse[orow] = (m + __builtin_log2f(l)) * 0.6931471805599453f;
}

// ---- append scatter / gather -----------------------------------------------------------------
template <int KV, int LAYOUT>
__global__ __launch_bounds__(256) void spex_scatter_kv_kernel(ScatterArgs a, Shape sh) {
  typedef typename std::conditional<KV == kF32, float,
                                    typename std::conditional<KV == kBF16, uint16_t, uint8_t>::type>::type T;
  const int D = sh.D, P = sh.P, H = sh.Hkv;
  const int64_t total = static_cast<int64_t>(a.n_pages) * H * P * D;
  const int64_t tid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (tid >= total) return;
  const int d = static_cast<int>(tid % D);
  const int slot = static_cast<int>((tid / D) % P);
  const int g = static_cast<int>((tid / (static_cast<int64_t>(D) * P)) % H);
  const int pi = static_cast<int>(tid / (static_cast<int64_t>(D) * P * H));
  const bool is_new = pi > 0 || a.first_page_is_new;
  const int tok = pi * P + slot - a.first_slot;  // index among the tokens of this launch
  const int64_t tile = (static_cast<int64_t>(a.page_ids[pi]) * sh.page_tiles + g);
  const int sidx = a.page_ids[pi] * H + g;
  const int64_t tile_elems = static_cast<int64_t>(P) * D;
  T *kp = static_cast<T *>(a.k_pool) + tile * tile_elems + k_offset<KV, LAYOUT>(slot, d, D);
  T *vp = static_cast<T *>(a.v_pool) + tile * tile_elems + v_offset<KV, LAYOUT>(slot, d, D);
  if (tok >= 0 && tok < a.n_tokens) {
    const int64_t src = (static_cast<int64_t>(tok) * H + g) * D + d;
    *kp = static_cast<const T *>(a.k_src)[src];
    const T vx = static_cast<const T *>(a.v_src)[src];
    *vp = v_is_f16<KV, LAYOUT>() ? static_cast<T>(bf16_bits_to_f16_bits(static_cast<uint16_t>(vx))) : vx;
  } else if (tok >= a.n_tokens && is_new) {
    *kp = T(0);
    *vp = T(0);
  }
  if (KV == kFP8 && is_new && d == 0 && slot == 0) {
    const int idx_new = pi - (a.first_page_is_new ? 0 : 1);
    a.k_scale[sidx] = a.k_scale_src[idx_new * H + g];
    a.v_scale[sidx] = a.v_scale_src[idx_new * H + g];
  }
}

// fp32 -> OCP e4m3fn code, round to nearest even, saturating at +-448 (0x7E / 0xFE); NaN -> 0x7F
// with the sign.  Integer arithmetic on the bit pattern, so the result does not depend on
// floating-point compile flags.  Normal range (|y| >= 2^-6): the fp32 mantissa is rounded to 3
// bits with the usual add-half-and-LSB trick, a carry moves into the exponent by itself.  Below
// that the grid is the multiples of 2^-9, and 8 * 2^-9 is the smallest normal (code 0x08).
__device__ __forceinline__ uint32_t encode_e4m3(float y) {
  const uint32_t u = __builtin_bit_cast(uint32_t, y);
  const uint32_t sign = (u >> 24) & 0x80u, a = u & 0x7fffffffu;
  uint32_t code;
  if (a > 0x7f800000u) {
    code = 0x7fu;
  } else if (a >= 0x43e00000u) {  // 448.0f and above (infinity included)
    code = 0x7eu;
  } else if (a >= 0x3c800000u) {  // 2^-6
    const uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u);
    code = (((r >> 23) - 120u) << 3) | ((r >> 20) & 7u);
  } else {
    code = static_cast<uint32_t>(__builtin_rintf(__builtin_bit_cast(float, a) * 512.0f));
  }
  return code | sign;
}

// A run of bf16 tokens of one node into an fp8 pool, quantised on the way: one workgroup per
// (page, kv head).  For a page this append starts, the workgroup first takes the largest magnitude
// of the tokens it puts there, separately for K and V, and sets scale = max(amax / 448, 2^-40);
// a page that was partially filled before keeps its scale.  Then code = e4m3(x * (1 / scale)).
// Unused slots of a started page are zeroed.  Inputs must be finite.
template <int LAYOUT>
__global__ __launch_bounds__(256) void spex_scatter_quant_kernel(ScatterArgs a, Shape sh) {
  const int D = sh.D, P = sh.P, H = sh.Hkv;
  const int g = blockIdx.x % H, pi = blockIdx.x / H;
  const bool is_new = pi > 0 || a.first_page_is_new;
  const int page = a.page_ids[pi];
  const int sidx = page * H + g;
  const uint16_t *ksrc = static_cast<const uint16_t *>(a.k_src), *vsrc = static_cast<const uint16_t *>(a.v_src);
  auto widen = [](uint16_t b) { return __builtin_bit_cast(float, static_cast<uint32_t>(b) << 16); };
  __shared__ float red[2][4];
  float ks, vs;
  if (is_new) {  // uniform over the workgroup
    float ka = 0.f, va = 0.f;
    for (int e = threadIdx.x; e < P * D; e += 256) {
      const int tok = pi * P + e / D - a.first_slot;
      if (tok >= 0 && tok < a.n_tokens) {
        const int64_t src = (static_cast<int64_t>(tok) * H + g) * D + e % D;
        ka = fmaxf(ka, __builtin_fabsf(widen(ksrc[src])));
        va = fmaxf(va, __builtin_fabsf(widen(vsrc[src])));
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      ka = fmaxf(ka, __shfl_xor(ka, o));
      va = fmaxf(va, __shfl_xor(va, o));
    }
    if ((threadIdx.x & 63) == 0) {
      red[0][threadIdx.x >> 6] = ka;
      red[1][threadIdx.x >> 6] = va;
    }
    __syncthreads();
    ka = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
    va = fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3]));
    ks = fmaxf(ka / 448.0f, 0x1p-40f);
    vs = fmaxf(va / 448.0f, 0x1p-40f);
    if (threadIdx.x == 0) {
      a.k_scale[sidx] = ks;
      a.v_scale[sidx] = vs;
    }
  } else {
    ks = a.k_scale[sidx];
    vs = a.v_scale[sidx];
  }
  const float kinv = 1.0f / ks, vinv = 1.0f / vs;
  const int64_t tile = (static_cast<int64_t>(page) * sh.page_tiles + g) * (static_cast<int64_t>(P) * D);
  uint8_t *kp = static_cast<uint8_t *>(a.k_pool) + tile, *vp = static_cast<uint8_t *>(a.v_pool) + tile;
  for (int e = threadIdx.x; e < P * D; e += 256) {
    const int slot = e / D, d = e % D;
    const int tok = pi * P + slot - a.first_slot;
    if (tok >= 0 && tok < a.n_tokens) {
      const int64_t src = (static_cast<int64_t>(tok) * H + g) * D + d;
      kp[k_offset<kFP8, LAYOUT>(slot, d, D)] = static_cast<uint8_t>(encode_e4m3(widen(ksrc[src]) * kinv));
      vp[v_offset<kFP8, LAYOUT>(slot, d, D)] = static_cast<uint8_t>(encode_e4m3(widen(vsrc[src]) * vinv));
    } else if (tok >= a.n_tokens && is_new) {
      kp[k_offset<kFP8, LAYOUT>(slot, d, D)] = 0;
      vp[v_offset<kFP8, LAYOUT>(slot, d, D)] = 0;
    }
  }
}

// One appended token per node: thread = (node, kv head, dim).  Writes the token's K and V element
// into its slot; where the token starts a page it also zeroes the page's other slots (so that
// nothing stale can be read from a partial page) and stores the page's fp8 scales.  The first
// n_patches threads also write one length patch each into the device copy of the cached plan.  QUANT (fp8
// pools): the source holds bf16 values and the code is encode_e4m3(x * (1 / scale)), scale being
// the one given for a page the token starts, else the one the page already has.
template <int KV, int LAYOUT, bool QUANT>
__global__ __launch_bounds__(256) void spex_append_tokens_kernel(AppendTokensArgs a, Shape sh) {
  typedef typename std::conditional<KV == kF32, float,
                                    typename std::conditional<KV == kBF16, uint16_t, uint8_t>::type>::type T;
  const int D = sh.D, P = sh.P, H = sh.Hkv;
  const int64_t total = static_cast<int64_t>(a.n_nodes) * H * D;
  const int64_t tid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (tid >= total) return;
  // the cached launch lists follow the append in the same launch: new valid counts and limits
  if (tid < a.n_patches) a.plan[a.patches[2 * tid]] = a.patches[2 * tid + 1];
  const int d = static_cast<int>(tid % D);
  const int g = static_cast<int>((tid / D) % H);
  const int node = static_cast<int>(tid / (static_cast<int64_t>(D) * H));
  const int page = a.dst[2 * node], code = a.dst[2 * node + 1];
  const int slot = code & 0xff;
  const bool is_new = (code >> 8) != 0;
  const int64_t tile = (static_cast<int64_t>(page) * sh.page_tiles + g) * (static_cast<int64_t>(P) * D);
  T *kp = static_cast<T *>(a.k_pool) + tile, *vp = static_cast<T *>(a.v_pool) + tile;
  T kx, vx;
  if (QUANT) {
    const float ks = is_new ? a.k_scale_src[node * H + g] : a.k_scale[page * H + g];
    const float vs = is_new ? a.v_scale_src[node * H + g] : a.v_scale[page * H + g];
    const float kf = __builtin_bit_cast(float, static_cast<uint32_t>(static_cast<const uint16_t *>(a.k_src)[tid]) << 16);
    const float vf = __builtin_bit_cast(float, static_cast<uint32_t>(static_cast<const uint16_t *>(a.v_src)[tid]) << 16);
    kx = static_cast<T>(encode_e4m3(kf * (1.0f / ks)));
    vx = static_cast<T>(encode_e4m3(vf * (1.0f / vs)));
  } else {
    kx = static_cast<const T *>(a.k_src)[tid];
    vx = static_cast<const T *>(a.v_src)[tid];
    if (v_is_f16<KV, LAYOUT>()) vx = static_cast<T>(bf16_bits_to_f16_bits(static_cast<uint16_t>(vx)));
  }
  kp[k_offset<KV, LAYOUT>(slot, d, D)] = kx;
  vp[v_offset<KV, LAYOUT>(slot, d, D)] = vx;
  if (is_new) {
    for (int s2 = 0; s2 < P; ++s2)
      if (s2 != slot) {
        kp[k_offset<KV, LAYOUT>(s2, d, D)] = T(0);
        vp[v_offset<KV, LAYOUT>(s2, d, D)] = T(0);
      }
    if (KV == kFP8 && d == 0) {
      a.k_scale[page * H + g] = a.k_scale_src[node * H + g];
      a.v_scale[page * H + g] = a.v_scale_src[node * H + g];
    }
  }
}

template <int KV, int LAYOUT>
__global__ __launch_bounds__(256) void spex_gather_kv_kernel(GatherArgs a, Shape sh) {
  typedef typename std::conditional<KV == kF32, float,
                                    typename std::conditional<KV == kBF16, uint16_t, uint8_t>::type>::type T;
  const int D = sh.D, P = sh.P, H = sh.Hkv;
  const int64_t total = static_cast<int64_t>(a.n_tokens) * H * D;
  const int64_t tid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (tid >= total) return;
  const int d = static_cast<int>(tid % D);
  const int g = static_cast<int>((tid / D) % H);
  const int tok = static_cast<int>(tid / (static_cast<int64_t>(D) * H));
  const int pi = (tok + a.first_slot) / P;
  const int slot = (tok + a.first_slot) % P;
  const int64_t tile = (static_cast<int64_t>(a.page_ids[pi]) * sh.page_tiles + g);
  const int sidx = a.page_ids[pi] * H + g;
  const int64_t tile_elems = static_cast<int64_t>(P) * D;
  static_cast<T *>(a.k_out)[tid] =
      static_cast<const T *>(a.k_pool)[tile * tile_elems + k_offset<KV, LAYOUT>(slot, d, D)];
  const T vx = static_cast<const T *>(a.v_pool)[tile * tile_elems + v_offset<KV, LAYOUT>(slot, d, D)];
  static_cast<T *>(a.v_out)[tid] =
      v_is_f16<KV, LAYOUT>() ? static_cast<T>(f16_bits_to_bf16_bits(static_cast<uint16_t>(vx))) : vx;
  if (KV == kFP8 && d == 0) {
    if (a.k_scale_out) a.k_scale_out[static_cast<int64_t>(tok) * H + g] = a.k_scale[sidx];
    if (a.v_scale_out) a.v_scale_out[static_cast<int64_t>(tok) * H + g] = a.v_scale[sidx];
  }
}

template <int KV, int D, int NT>
hipError_t launch_mfma(const Shape &sh, const AttnArgs &a, bool prefix, hipStream_t stream) {
  const dim3 grid((a.n_items + 3) / 4), block(256);
  if (a.qt_mask) {  // draft token trees: visibility masks per query
    if (prefix)
      hipLaunchKernelGGL((spex_prefix_attn_kernel<KV, D, NT, true>), grid, block, 0, stream, a, sh);
    else
      hipLaunchKernelGGL((spex_suffix_attn_kernel<KV, D, NT, true>), grid, block, 0, stream, a, sh);
  } else if (prefix) {
    hipLaunchKernelGGL((spex_prefix_attn_kernel<KV, D, NT, false>), grid, block, 0, stream, a, sh);
  } else {
    hipLaunchKernelGGL((spex_suffix_attn_kernel<KV, D, NT, false>), grid, block, 0, stream, a, sh);
  }
  return hipGetLastError();
}

template <int KV, int D>
hipError_t launch_mfma_nt(const Shape &sh, const AttnArgs &a, bool prefix, int nt, hipStream_t s) {
  return nt == 1 ? launch_mfma<KV, D, 1>(sh, a, prefix, s) : launch_mfma<KV, D, 2>(sh, a, prefix, s);
}

template <int KV, int QT>
hipError_t launch_generic(const Shape &sh, const AttnArgs &a, int rows_per_item, hipStream_t stream) {
  const dim3 grid(a.n_items, rows_per_item), block(64);
  if (sh.layout == kMfmaTiled)
    hipLaunchKernelGGL((spex_generic_attn_kernel<KV, QT, kMfmaTiled>), grid, block, 0, stream, a, sh,
                       rows_per_item);
  else
    hipLaunchKernelGGL((spex_generic_attn_kernel<KV, QT, kRowMajor>), grid, block, 0, stream, a, sh,
                       rows_per_item);
  return hipGetLastError();
}

}  // namespace

bool has_mfma_kernel(const Shape &sh) {
  return sh.layout == kMfmaTiled && sh.q_dtype == kBF16 &&
         (sh.kv_dtype == kBF16 || sh.kv_dtype == kFP8) && sh.P == 16 && (sh.D == 64 || sh.D == 128);
}

hipError_t launch_attention(const Shape &sh, const AttnArgs &a, bool prefix, int row_tiles,
                            bool force_generic, hipStream_t stream) {
  if (a.n_items <= 0) return hipSuccess;
  if (!force_generic && has_mfma_kernel(sh)) {
    if (sh.kv_dtype == kBF16)
      return sh.D == 64 ? launch_mfma_nt<kBF16, 64>(sh, a, prefix, row_tiles, stream)
                        : launch_mfma_nt<kBF16, 128>(sh, a, prefix, row_tiles, stream);
    return sh.D == 64 ? launch_mfma_nt<kFP8, 64>(sh, a, prefix, row_tiles, stream)
                      : launch_mfma_nt<kFP8, 128>(sh, a, prefix, row_tiles, stream);
  }
  const int rows_per_item = 16 * row_tiles;
  if (sh.kv_dtype == kF32 && sh.q_dtype == kF32) return launch_generic<kF32, kF32>(sh, a, rows_per_item, stream);
  if (sh.kv_dtype == kBF16 && sh.q_dtype == kBF16) return launch_generic<kBF16, kBF16>(sh, a, rows_per_item, stream);
  if (sh.kv_dtype == kFP8 && sh.q_dtype == kBF16) return launch_generic<kFP8, kBF16>(sh, a, rows_per_item, stream);
  return hipErrorInvalidValue;
}

template <int KV, int D>
static hipError_t launch_coop_ntw(const Shape &sh, const AttnArgs &a, int ntw, hipStream_t stream) {
  const dim3 grid(a.n_items), block(256);
  if (a.qt_mask) {
    if (ntw == 1)
      hipLaunchKernelGGL((spex_prefix_coop_kernel<KV, D, 1, true>), grid, block, 0, stream, a, sh);
    else if (ntw == 2)
      hipLaunchKernelGGL((spex_prefix_coop_kernel<KV, D, 2, true>), grid, block, 0, stream, a, sh);
    else
      hipLaunchKernelGGL((spex_prefix_coop_kernel<KV, D, 4, true>), grid, block, 0, stream, a, sh);
  } else if (ntw == 1) {
    hipLaunchKernelGGL((spex_prefix_coop_kernel<KV, D, 1, false>), grid, block, 0, stream, a, sh);
  } else if (ntw == 2) {
    hipLaunchKernelGGL((spex_prefix_coop_kernel<KV, D, 2, false>), grid, block, 0, stream, a, sh);
  } else {
    hipLaunchKernelGGL((spex_prefix_coop_kernel<KV, D, 4, false>), grid, block, 0, stream, a, sh);
  }
  return hipGetLastError();
}

hipError_t launch_prefix_coop(const Shape &sh, const AttnArgs &a, int ntw, hipStream_t stream) {
  if (a.n_items <= 0) return hipSuccess;
  if (!has_mfma_kernel(sh) || (ntw != 1 && ntw != 2 && ntw != 4)) return hipErrorInvalidValue;
  if (sh.kv_dtype == kBF16)
    return sh.D == 64 ? launch_coop_ntw<kBF16, 64>(sh, a, ntw, stream)
                      : launch_coop_ntw<kBF16, 128>(sh, a, ntw, stream);
  return sh.D == 64 ? launch_coop_ntw<kFP8, 64>(sh, a, ntw, stream)
                    : launch_coop_ntw<kFP8, 128>(sh, a, ntw, stream);
}

template <int KV, int D, int NW, bool TREE>
static hipError_t launch_walk_ntw(const Shape &sh, const WalkArgs &a, int ntw, hipStream_t stream) {
  const dim3 grid(a.n_items), block(64 * NW);
  if (ntw == 1)
    hipLaunchKernelGGL((spex_tree_walk_kernel<KV, D, 1, NW, TREE>), grid, block, 0, stream, a, sh);
  else if (ntw == 2)
    hipLaunchKernelGGL((spex_tree_walk_kernel<KV, D, 2, NW, TREE>), grid, block, 0, stream, a, sh);
  else
    hipLaunchKernelGGL((spex_tree_walk_kernel<KV, D, 4, NW, TREE>), grid, block, 0, stream, a, sh);
  return hipGetLastError();
}

template <int KV, int D>
static hipError_t launch_walk_nw(const Shape &sh, const WalkArgs &a, int ntw, int waves, hipStream_t stream) {
  if (a.qt_mask)  // draft-tree masks: not in the kernel that splits the path
    return waves == 4   ? launch_walk_ntw<KV, D, 4, true>(sh, a, ntw, stream)
           : waves == 8 ? launch_walk_ntw<KV, D, 8, true>(sh, a, ntw, stream)
                        : hipErrorInvalidValue;
  if (waves == 2) {  // lists for two wavefronts of rows, walked by four: the path is split in two
    const dim3 grid(a.n_items), block(256);
    if (ntw == 1)
      hipLaunchKernelGGL((spex_tree_walk_kernel<KV, D, 1, 4, false, 2>), grid, block, 0, stream, a, sh);
    else if (ntw == 2)
      hipLaunchKernelGGL((spex_tree_walk_kernel<KV, D, 2, 4, false, 2>), grid, block, 0, stream, a, sh);
    else
      return hipErrorInvalidValue;
    return hipGetLastError();
  }
  return waves == 4 ? launch_walk_ntw<KV, D, 4, false>(sh, a, ntw, stream)
                    : launch_walk_ntw<KV, D, 8, false>(sh, a, ntw, stream);
}

hipError_t launch_tree_walk(const Shape &sh, const WalkArgs &a, int ntw, int waves, hipStream_t stream) {
  if (a.n_items <= 0) return hipSuccess;
  if (!has_mfma_kernel(sh) || (ntw != 1 && ntw != 2 && ntw != 4) || (waves != 2 && waves != 4 && waves != 8))
    return hipErrorInvalidValue;
  if (sh.kv_dtype == kBF16)
    return sh.D == 64 ? launch_walk_nw<kBF16, 64>(sh, a, ntw, waves, stream)
                      : launch_walk_nw<kBF16, 128>(sh, a, ntw, waves, stream);
  return sh.D == 64 ? launch_walk_nw<kFP8, 64>(sh, a, ntw, waves, stream)
                    : launch_walk_nw<kFP8, 128>(sh, a, ntw, waves, stream);
}

namespace {
// blob[pairs[2i]] = pairs[2i + 1]: brings the device copy of a plan up to date after appends.
__global__ __launch_bounds__(256) void spex_patch_plan_kernel(int32_t *blob, const int32_t *pairs, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) blob[pairs[2 * i]] = pairs[2 * i + 1];
}
}  // namespace

hipError_t launch_patch(int32_t *blob, const int32_t *pairs, int32_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(spex_patch_plan_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, blob, pairs, n);
  return hipGetLastError();
}

hipError_t launch_merge(const Shape &sh, const MergeArgs &a, hipStream_t stream) {
  if (a.n_qtok <= 0) return hipSuccess;
  const int vec = (sh.D % 4 == 0) ? 4 : 1;
  const int64_t threads = static_cast<int64_t>(a.n_qtok) * sh.Hq * (sh.D / vec);
  const dim3 grid(static_cast<unsigned>((threads + 255) / 256)), block(256);
  if (vec == 4)
    hipLaunchKernelGGL(spex_lse_merge_kernel<4>, grid, block, 0, stream, a, sh);
  else
    hipLaunchKernelGGL(spex_lse_merge_kernel<1>, grid, block, 0, stream, a, sh);
  return hipGetLastError();
}

template <int KV>
static hipError_t scatter_layout(const Shape &sh, const ScatterArgs &a, hipStream_t stream) {
  const int64_t total = static_cast<int64_t>(a.n_pages) * sh.Hkv * sh.P * sh.D;
  const dim3 grid(static_cast<unsigned>((total + 255) / 256)), block(256);
  if (sh.layout == kMfmaTiled)
    hipLaunchKernelGGL((spex_scatter_kv_kernel<KV, kMfmaTiled>), grid, block, 0, stream, a, sh);
  else
    hipLaunchKernelGGL((spex_scatter_kv_kernel<KV, kRowMajor>), grid, block, 0, stream, a, sh);
  return hipGetLastError();
}

hipError_t launch_scatter_quantise(const Shape &sh, const ScatterArgs &a, hipStream_t stream) {
  if (a.n_pages <= 0) return hipSuccess;
  if (sh.kv_dtype != kFP8) return hipErrorInvalidValue;
  const dim3 grid(static_cast<unsigned>(a.n_pages * sh.Hkv)), block(256);
  if (sh.layout == kMfmaTiled)
    hipLaunchKernelGGL((spex_scatter_quant_kernel<kMfmaTiled>), grid, block, 0, stream, a, sh);
  else
    hipLaunchKernelGGL((spex_scatter_quant_kernel<kRowMajor>), grid, block, 0, stream, a, sh);
  return hipGetLastError();
}

hipError_t launch_scatter(const Shape &sh, const ScatterArgs &a, hipStream_t stream) {
  if (a.n_pages <= 0) return hipSuccess;
  switch (sh.kv_dtype) {
    case kF32: return scatter_layout<kF32>(sh, a, stream);
    case kBF16: return scatter_layout<kBF16>(sh, a, stream);
    case kFP8: return scatter_layout<kFP8>(sh, a, stream);
  }
  return hipErrorInvalidValue;
}

template <int KV>
static hipError_t gather_layout(const Shape &sh, const GatherArgs &a, hipStream_t stream) {
  const int64_t total = static_cast<int64_t>(a.n_tokens) * sh.Hkv * sh.D;
  const dim3 grid(static_cast<unsigned>((total + 255) / 256)), block(256);
  if (sh.layout == kMfmaTiled)
    hipLaunchKernelGGL((spex_gather_kv_kernel<KV, kMfmaTiled>), grid, block, 0, stream, a, sh);
  else
    hipLaunchKernelGGL((spex_gather_kv_kernel<KV, kRowMajor>), grid, block, 0, stream, a, sh);
  return hipGetLastError();
}

hipError_t launch_gather(const Shape &sh, const GatherArgs &a, hipStream_t stream) {
  if (a.n_tokens <= 0) return hipSuccess;
  switch (sh.kv_dtype) {
    case kF32: return gather_layout<kF32>(sh, a, stream);
    case kBF16: return gather_layout<kBF16>(sh, a, stream);
    case kFP8: return gather_layout<kFP8>(sh, a, stream);
  }
  return hipErrorInvalidValue;
}

template <int KV, bool QUANT>
static hipError_t append_tokens_layout(const Shape &sh, const AppendTokensArgs &a, hipStream_t stream) {
  const int64_t total = static_cast<int64_t>(a.n_nodes) * sh.Hkv * sh.D;
  const dim3 grid(static_cast<unsigned>((total + 255) / 256)), block(256);
  if (sh.layout == kMfmaTiled)
    hipLaunchKernelGGL((spex_append_tokens_kernel<KV, kMfmaTiled, QUANT>), grid, block, 0, stream, a, sh);
  else
    hipLaunchKernelGGL((spex_append_tokens_kernel<KV, kRowMajor, QUANT>), grid, block, 0, stream, a, sh);
  return hipGetLastError();
}

hipError_t launch_append_tokens(const Shape &sh, const AppendTokensArgs &a, hipStream_t stream) {
  if (a.n_nodes <= 0) return hipSuccess;
  if (a.quantise)
    return sh.kv_dtype == kFP8 ? append_tokens_layout<kFP8, true>(sh, a, stream) : hipErrorInvalidValue;
  switch (sh.kv_dtype) {
    case kF32: return append_tokens_layout<kF32, false>(sh, a, stream);
    case kBF16: return append_tokens_layout<kBF16, false>(sh, a, stream);
    case kFP8: return append_tokens_layout<kFP8, false>(sh, a, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace spex
