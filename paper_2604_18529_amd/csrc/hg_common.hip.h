// Device code of the partitioned decode-attention library (gfx950, wave64): definitions shared by
// all kernels -- argument structures, the work split, storage traits and small helpers.
//
//   hg_stream_valu.hip.h   hg_partial_kernel: streams the K and V rows of a span of tokens once and
//                          folds them into softmax statistics (m, l, O) per query head (paper
//                          Section 4.2: the per-token logit stage, run here per positional
//                          range); also the logits-export and concat modes.
//   hg_stream_gqa.hip.h    hg_partial_gqa_kernel: the same on the matrix cores for grouped-query
//                          attention.
//   hg_combine.hip.h       hg_segment_reduce_kernel (segment records -> range triple or, for the
//                          unsplit path, normalised output), hg_merge_kernel (exact recombination
//                          of range triples: Section 4.2.3, Token Concatenator, in statistics
//                          form), the concat path's reduce kernel, table uploads.
//   hg_select.hip.h        hg_select_kernel: Post-QK^T top-k selection.
//
// Work distribution.  The tokens of all ranges, repeated for every stream (KV head x chunk of
// query heads), form one linear space of `total` positions: position p = s * ltok + x, where
// x runs over the concatenated ranges.  Workgroup w owns positions [w * span, (w+1) * span), so
// every workgroup streams the same number of bytes whatever the shape of the partition table,
// and the launch is sized to the chip (one workgroup per compute unit for long inputs).  A
// workgroup's span is cut into segments at range and stream boundaries; each segment yields one
// (m, l, O) record in slot  w + s * n_ranges + r  (strictly increasing along the linear order,
// hence unique), and the records of a (range, stream) pair occupy a contiguous run of slots.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hg {

constexpr int kInlineRanges = 64;   // range-table entries carried inside the kernel arguments
constexpr int kFusedGroups = 16;    // groups of a launch in which one workgroup takes a whole (group, stream)
constexpr int kInlineGroups = 256;  // CSR offsets carried inside the merge kernel's arguments
constexpr int kUploadRanges = 128;  // entries per table-upload launch
constexpr int kUploadInts = 512;
// Waves per streaming workgroup and workgroups per compute unit (tuning constants).
#ifndef HG_VALU_WAVES
#define HG_VALU_WAVES 4
#endif
#ifndef HG_GQA_WAVES
#define HG_GQA_WAVES 4
#endif
#ifndef HG_VALU_U
#define HG_VALU_U 4  // rows in flight per 16-lane group (kernels with 1 or 2 heads per stream)
#endif
#ifndef HG_VALU_WG_PER_CU
#define HG_VALU_WG_PER_CU 1
#endif
#ifndef HG_GQA_WG_PER_CU
#define HG_GQA_WG_PER_CU 1
#endif
constexpr int kValuWaves = HG_VALU_WAVES;
constexpr int kGqaWaves = HG_GQA_WAVES;
constexpr int kValuBlock = 64 * kValuWaves;
constexpr int kGqaBlock = 64 * kGqaWaves;
constexpr int kValuWorkgroupsPerCu = HG_VALU_WG_PER_CU;
constexpr int kGqaWorkgroupsPerCu = HG_GQA_WG_PER_CU;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// "no token seen yet" marker for running maxima (log2 domain).  Finite, so that
// exp2(marker - marker) = 1 multiplies an all-zero state instead of producing NaN.
constexpr float kNegBig = -3.0e38f;

// pre = number of tokens in the ranges before this one (prefix sum of the range lengths).
struct RangeEntry {
    int32_t seq, begin, end, pre, pad;
};

// What a streaming kernel instance does with the rows it reads.
constexpr int kModeStats = 0;   // K and V -> (m, l, O) records                     (hg_attn_partial / hg_attn_full)
constexpr int kModeLogits = 1;  // K only  -> raw scaled logits                     (hg_attn_logits)
constexpr int kModeConcat = 2;  // V and given logits -> (m, l, O) records over those logits     (hg_attn_concat)
constexpr int kModeFilter = 3;  // K only  -> logits at or above a running lower bound of the k-th largest, densely (hg_attn_topk)

// The range table travels by value in the kernel arguments when it is small; otherwise `ext`
// points at a device copy.  Entry n_ranges is a sentinel whose pre is ltok.
struct RangeTable {
    const RangeEntry *ext;
    int32_t n_ranges;
    int32_t pad;
    RangeEntry inl[kInlineRanges + 1];
};

// How the linear work space is laid out and cut (shared by the streaming and reduce kernels).
struct WorkSplit {
    int64_t total;    // n_streams * ltok
    int32_t ltok;     // tokens in all ranges together
    int32_t span;     // positions per workgroup
    int32_t group;    // query heads per KV head
    int32_t gt;       // query heads per stream (chunk of a group)
    int32_t n_chunks; // streams per KV head
    int32_t n_q_heads;
};

// Paged cache: token t of sequence b lives in physical block table[b * max_blocks + (t >> shift)]
// at row t & mask; stride_b is then the distance between physical blocks.  table == nullptr
// means a contiguous cache.
struct PageMap {
    const int32_t *table;
    int32_t shift, mask, max_blocks, pad;
};

// Byte offset of row `tok` of a paged cache whose table entry is `page`.  The host admits paged
// descriptors only with a block stride below 4 GiB and a row stride below 16 MiB, so one
// 32x32->64 multiply-add and one 24-bit multiply (full rate) do; a generic 64-bit product would
// cost two quarter-rate multiplies per row.
__device__ __forceinline__ int64_t paged_row_offset(int page, int tok, int mask, uint32_t block_b32, uint32_t row_b32)
{
    return (int64_t)((uint64_t)(uint32_t)page * block_b32 + __umul24((uint32_t)(tok & mask), row_b32));
}

struct PartialArgs {
    const void *q, *k, *v;
    int64_t stride_b, stride_h, stride_t;  // elements
    PageMap pages;
    float qscale;                          // scale * log2(e); plain scale in logits mode
    float *ws_m, *ws_l, *ws_o;             // segment records [slot][gt], [slot][gt][D]; m in log2 units
    // direct mode (statistics only): no (range, stream) pair is cut by a span boundary, so every
    // segment IS a whole pair and its result goes straight to the caller's arrays; the reduce
    // kernel is not launched.  normalise as in ReduceArgs.
    int32_t direct, normalise;
    float *out_m, *out_l, *out_o;
    float *logits;                         // [Hq][ltok]: written in logits mode, read in concat mode
    // filter mode: every segment is cut into n_sub consecutive sub-spans (one per wave); the
    // survivors of sub-span j of head h -- logit and column, in ascending column order -- are
    // written to surv_val / surv_col [Hq][ltok] starting at the sub-span's own first column, and
    // their number to surv_cnt[(slot * n_sub + j) * gt + head in stream]
    float *surv_val;
    int32_t *surv_col, *surv_cnt;
    int32_t filter_rank, filter_k;         // bound = filter_rank-th (0-based) largest of every lane's own elements; top_k
    // Bounds shared between the workgroups that scan the same (range, stream) pair:
    // gbound[(slot * gt + head in stream) * 64 + 16 * wave + lane position], order-preserving keys of logits,
    // 0 (below every key) before the launch.  An entry is what its workgroup has published so far
    // (see the filter mode).
    uint32_t *gbound;
    // filter mode: words the first workgroup sets to zero for the selection that follows the scan
    // (its count of finished workgroups per (group, head))
    uint32_t *tail_cnt;
    int64_t n_tail;
    // FUSED variant of the vector kernel (hg_attn_partial_merge on small inputs): workgroup
    // (group i, stream) takes the ranges fused_groups[i] .. fused_groups[i + 1] - 1 one after the
    // other, writes their triples itself and the group's merged output at the end
    int32_t fused_n_groups;
    int32_t fused_groups[kFusedGroups + 1];
    float *merged_out, *merged_lse;  // [n_groups][Hq][D], [n_groups][Hq] or NULL
    WorkSplit ws;
    RangeTable tab;
};

// Tokens per sub-span of a segment of `len` tokens in filter mode (a multiple of every streaming
// kernel's tokens per wave iteration).
__host__ __device__ __forceinline__ int filter_sub_len(int len, int n_sub)
{
    return (len + n_sub * 64 - 1) / (n_sub * 64) * 64;
}

// Sub-spans of a segment of `len` tokens that hold at least 16 tokens (every one of the 16 lanes
// of a head then owns a logit after the wave's first block): the waves that take part in the
// shared bound.
__host__ __device__ __forceinline__ int filter_valid_waves(int len, int n_sub)
{
    if (len < 16) return 0;
    const int v = (len - 16) / filter_sub_len(len, n_sub) + 1;
    return v < n_sub ? v : n_sub;
}

struct ReduceArgs {
    const float *ws_m, *ws_l, *ws_o;
    int32_t normalise;  // 0: write the range triple (m, l, o); 1: write out = O/L and lse
    float *m_out, *l_out, *o_out;  // [n_ranges][Hq](..[D])  or  out/lse when normalise
    WorkSplit ws;
    RangeTable tab;
};

struct GroupTable {
    const int32_t *ext;
    int32_t n_groups;
    int32_t inl[kInlineGroups + 1];
};

struct MergeArgs {
    const float *m, *l, *o;
    float *out, *lse;
    int32_t n_q_heads;
    GroupTable tab;
    // second producer (hg_attn_merge2): its own triple arrays and CSR; m_b == nullptr: none
    const float *m_b, *l_b, *o_b;
    GroupTable tab_b;
};

struct ConcatReduceArgs {
    const float *ws_m, *ws_l, *ws_o;  // segment records over the given logits, m in log2 units
    float *out, *lse;
    WorkSplit ws;
    GroupTable groups;
    RangeTable tab;
};

constexpr int kSelectBlock = 1024;  // threads of the selection kernel (16 waves)
constexpr int kMaxTopK = 4096;      // kept tokens per (group, head): their columns and logits sit in LDS

struct SelectArgs {
    const float *logits;  // [Hq][ltok], natural-log units
    const void *v;
    int64_t stride_b, stride_h, stride_t;  // elements
    int32_t ltok, n_q_heads, group, top_k;
    int32_t *sel;         // [n_groups][Hq][top_k] or NULL
    float *m, *l, *o;     // [n_groups][Hq](..[D])
    // two-stage selection of long groups: every group is cut into `parts` column intervals whose
    // own top_k candidates (value, column; -inf padded) are the input of the second stage
    int32_t parts;
    float *cand_val;      // [n_groups][Hq][parts][top_k]
    int32_t *cand_col;
    // when parts * top_k is more than one workgroup selects from quickly, a middle stage reduces
    // the candidates of each (group, head) to parts2 * top_k (0: no middle stage)
    int32_t parts2, pad2;
    float *cand2_val;     // [n_groups][Hq][parts2][top_k]
    int32_t *cand2_col;
    PageMap pages;        // table == nullptr: contiguous cache
    // hg_attn_topk: instead of the full logits rows, the first stage selects among the survivors
    // of the filter pass: dense_cnt[group][head] entries (logit, column; ascending columns) that
    // start at the group's first column of row `head` of dense_val / dense_col [Hq][ltok].
    // dense_cnt == nullptr: select from `logits`.
    const float *dense_val;
    const int32_t *dense_col, *dense_cnt;
    // dense lists only, staged selection: a (group, head) whose list has at most direct_limit
    // entries is selected by the one-workgroup stage (launched first) and skipped by the staged
    // kernels; a longer list the other way round.  0: no such split.
    int32_t direct_limit, pad3;
    // hg_select_survivors_kernel: the filter pass's own lists (see PartialArgs), the split they were
    // written under, the workgroups per (group, head) of this launch and their count of finished
    // ones (zero at the start)
    const float *surv_val;
    const int32_t *surv_col, *surv_cnt;
    uint32_t *tail_cnt;
    int32_t n_sub, tail_parts;
    WorkSplit ws;
    GroupTable groups;
    RangeTable tab;
};

// Gathers the survivors that the filter pass left per (segment, sub-span, head) into one dense,
// column-ordered list per (group, head).
struct CompactArgs {
    const float *surv_val;
    const int32_t *surv_col, *surv_cnt;
    float *dense_val;
    int32_t *dense_col, *dense_cnt;
    int32_t n_sub, chunks;  // sub-spans per segment; workgroups that share the copying of one (group, head)
    WorkSplit ws;
    GroupTable groups;
    RangeTable tab;
};

constexpr int kSelectDirect = 0;      // one workgroup selects from the group's logits row
constexpr int kSelectCandidates = 1;  // stage 1: per part, write its top_k candidates
constexpr int kSelectFromCands = 2;   // last stage: select among the candidates
constexpr int kSelectMidCands = 3;    // middle stage: candidates of a chunk of the candidates

struct RangeChunk {
    RangeEntry e[kUploadRanges];
};
struct IntChunk {
    int32_t e[kUploadInts];
};

// ---- small device helpers ----------------------------------------------------------------------

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// Sum over the 16 lanes of a DPP row; every lane of the row ends with the total.
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
    x += dpp_move<0x141>(x);  // row_half_mirror: quads 0<->1, 2<->3
    x += dpp_move<0x140>(x);  // row_mirror: halves swap
    return x;
}

// Sum over a lane group of LPR = 16 or 8 lanes (8: the two halves of a DPP row are separate groups).
template <int LPR>
__device__ __forceinline__ float lane_group_sum(float x)
{
    x += dpp_move<0xB1>(x);
    x += dpp_move<0x4E>(x);
    x += dpp_move<0x141>(x);
    if constexpr (LPR == 16) x += dpp_move<0x140>(x);
    return x;
}

// Order-preserving integer keys of fp32 values: larger float <=> larger key.
__device__ __forceinline__ uint32_t order_key(float x)
{
    uint32_t u = __float_as_uint(x);
    u = u == 0x80000000u ? 0u : u;                      // -0.0 and +0.0 are one value: they tie
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // larger float <=> larger key
}

__device__ __forceinline__ float key_to_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

// Hand-over of a float between the waves of a workgroup through LDS, without a barrier: relaxed
// atomics keep the accesses real LDS instructions at the place they are written (a volatile
// access compiled to a FLAT instruction, which ties up the vector-memory counters as well).
__device__ __forceinline__ void lds_publish(float *p, float x) { __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
__device__ __forceinline__ float lds_peek(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }

__device__ __forceinline__ RangeEntry table_entry(const RangeTable &tab, int i)
{
    return tab.ext ? tab.ext[i] : tab.inl[i];
}

// Largest r with pre[r] <= x (0 <= x < ltok); it contains x because empty ranges share their
// successor's prefix.
__device__ __forceinline__ int find_range(const RangeTable &tab, int x)
{
    int lo = 0, hi = tab.n_ranges;  // invariant: pre[lo] <= x < pre[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (table_entry(tab, mid).pre <= x)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

// Walk the segments of this workgroup's span.  f(stream, range index, range entry, t0, t1, col0, slot) is
// called by every thread of the workgroup, in the same order (the control flow is uniform);
// col0 is the position of token t0 in the concatenation of all ranges.
template <typename F>
__device__ __forceinline__ void for_each_segment(const WorkSplit &ws, const RangeTable &tab, F &&f)
{
    int64_t p = (int64_t)blockIdx.x * ws.span;
    const int64_t p_end = p + ws.span < ws.total ? p + ws.span : ws.total;
    int s = (int)(p / ws.ltok);
    int x = (int)(p - (int64_t)s * ws.ltok);
    int r = find_range(tab, x);
    while (p < p_end) {
        const RangeEntry e = table_entry(tab, r);
        const int r_end = table_entry(tab, r + 1).pre;
        const int64_t left = p_end - p;
        const int len = left < (int64_t)(r_end - x) ? (int)left : r_end - x;
        const int t0 = e.begin + (x - e.pre);
        f(s, r, e, t0, t0 + len, x, (int64_t)blockIdx.x + (int64_t)s * tab.n_ranges + r);
        p += len;
        x += len;
        if (x == r_end) {
            if (x == ws.ltok) {  // next stream, first non-empty range
                ++s;
                x = 0;
                r = find_range(tab, 0);
            } else {
                r = find_range(tab, x);
            }
        }
    }
}

// ---- storage traits ----------------------------------------------------------------------------

// K and V are read exactly once, so their loads carry the non-temporal hint: measured on MI355X
// a pure read stream reaches about 7.1 TB/s with it against about 6.3 TB/s without.
#ifndef HG_NT_LOADS
#define HG_NT_LOADS 1
#endif

typedef unsigned int hg_u32x4 __attribute__((ext_vector_type(4)));

template <int VB>
struct RawVec;
template <>
struct RawVec<16> {
    hg_u32x4 d;
};

// storage types of q, K and V (the values of hg_dtype)
constexpr int kDtF16 = 0, kDtF32 = 1, kDtBf16 = 2;

template <int D_, int DT_>
struct Traits {
    static constexpr int D = D_;
    static constexpr int DT = DT_;
    static constexpr int ES = DT_ == kDtF32 ? 4 : 2;
    static constexpr int LPR = D_ * ES >= 256 ? 16 : 8;       // lanes per row: a lane always loads 16 bytes
    static constexpr int RPW = 64 / LPR;                      // rows per wave load instruction (4 or 8)
    static constexpr int LANE_BYTES = D_ * ES / LPR;          // bytes of a row held by one lane
    static constexpr int VB = 16;                             // bytes per load
    static constexpr int NV = LANE_BYTES / VB;                // loads per row per lane
    static constexpr int EPV = VB / ES;                       // elements per load
    static constexpr int EPL = NV * EPV;                      // elements per lane
    static constexpr int SEG = LPR * EPV;                     // elements covered by one row load of the lane group
    using Raw = RawVec<VB>;

    // element offset inside a row of lane `sub`'s vector j
    __device__ static __forceinline__ int vec_offset(int sub, int j) { return j * SEG + sub * EPV; }

    // STREAM = true for K and V (read once), false for q (re-read by every workgroup of the head)
    template <bool STREAM>
    __device__ static __forceinline__ Raw load(const char *row_ptr, int sub, int j)
    {
        Raw r;
        const char *p = row_ptr + (size_t)vec_offset(sub, j) * ES;
        using vec_t = decltype(r.d);
        if constexpr (STREAM && HG_NT_LOADS)
            r.d = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(p));
        else
            r.d = *reinterpret_cast<const vec_t *>(p);
        return r;
    }

    __device__ static __forceinline__ void widen(const Raw &r, float *out)
    {
        if constexpr (DT_ == kDtF16) {
            typedef _Float16 hvec __attribute__((ext_vector_type(EPV)));
            hvec h = __builtin_bit_cast(hvec, r.d);
#pragma unroll
            for (int i = 0; i < EPV; ++i) out[i] = (float)h[i];
        } else if constexpr (DT_ == kDtBf16) {
            // a bfloat16 is the upper half of the binary32 of the same value
            typedef uint32_t uvec __attribute__((ext_vector_type(EPV / 2)));
            uvec u = __builtin_bit_cast(uvec, r.d);
#pragma unroll
            for (int i = 0; i < EPV / 2; ++i) {
                out[2 * i] = __uint_as_float(u[i] << 16);
                out[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
            }
        } else {
            typedef float fvec __attribute__((ext_vector_type(EPV)));
            fvec f = __builtin_bit_cast(fvec, r.d);
#pragma unroll
            for (int i = 0; i < EPV; ++i) out[i] = f[i];
        }
    }
};

// The FUSED walk: workgroup blockIdx.x = stream * n_groups + group visits the group's ranges in
// order.  f as in for_each_segment (a whole range is one segment; the slot is unused: results are
// written directly); empty(stream, range index) is called for a range without tokens.
template <typename F, typename E>
__device__ __forceinline__ void for_each_range_of_group(const PartialArgs &a, F &&f, E &&empty)
{
    const int gi = (int)(blockIdx.x % (unsigned)a.fused_n_groups), s = (int)(blockIdx.x / (unsigned)a.fused_n_groups);
    const int r0 = a.fused_groups[gi], r1 = a.fused_groups[gi + 1];
    for (int r = r0; r < r1; ++r) {
        const RangeEntry e = table_entry(a.tab, r);
        if (e.end == e.begin)
            empty(s, r);
        else
            f(s, r, e, e.begin, e.end, e.pre, (int64_t)0);
    }
}

// Result of one segment for one (head, channel): a record for the reduce kernel, or, in direct
// mode, the caller's triple / normalised output itself.  mx in log2 units.
template <int D>
__device__ __forceinline__ void write_segment_result(const PartialArgs &a, int64_t rec, int r_idx, int head, int c, float mx,
                                                     float lt, float ot)
{
    if (!a.direct) {
        a.ws_o[rec * D + c] = ot;
        if (c == 0) {
            a.ws_m[rec] = mx;
            a.ws_l[rec] = lt;
        }
        return;
    }
    const int64_t rh = (int64_t)r_idx * a.ws.n_q_heads + head;
    if (a.normalise) {
        a.out_o[rh * D + c] = ot / lt;  // a segment is never empty
        if (c == 0 && a.out_m) a.out_m[rh] = mx * kLn2 + logf(lt);
    } else {
        a.out_o[rh * D + c] = ot;
        if (c == 0) {
            a.out_m[rh] = mx * kLn2;
            a.out_l[rh] = lt;
        }
    }
}

}  // namespace hg
