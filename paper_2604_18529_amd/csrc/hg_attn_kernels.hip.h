// Device code of the partitioned decode-attention library (gfx950, wave64).
//
// Three kernels:
//   hg_partial_kernel      streams the K and V rows of a span of tokens once and folds them into
//                          softmax statistics (m, l, O) per query head (paper Section 4.2: the
//                          per-token logit stage, run here per positional range).
//   hg_segment_reduce_kernel  merges the segment records of a range into the range's triple, or,
//                          for the unsplit path, into the normalised output.
//   hg_merge_kernel        exact recombination of range triples (Section 4.2.3, Token
//                          Concatenator, in statistics form).
//
// Work distribution.  The tokens of all ranges, repeated for every stream (KV head x chunk of
// query heads), form one linear space of `total` positions: position p = s * ltok + x, where
// x runs over the concatenated ranges.  Workgroup w owns positions [w * span, (w+1) * span), so
// every workgroup streams the same number of bytes whatever the shape of the partition table,
// and the launch is sized to the chip (one workgroup per compute unit for long inputs).  A
// workgroup's span is cut into segments at range and stream boundaries; each segment yields one
// (m, l, O) record in slot  w + s * n_ranges + r  (strictly increasing along the linear order,
// hence unique), and the records of a (range, stream) pair occupy a contiguous run of slots.
//
// Lane layout of the streaming kernel.  One K or V row (head_dim elements, 128..512 bytes) is
// spread over the 16 lanes of a DPP row, each lane holding 8..32 contiguous bytes per 256-byte
// segment, so one wave load instruction fetches four whole rows (1 KiB, fully coalesced).  A
// lane keeps the matching channels of q (pre-multiplied by scale*log2 e) and of the O
// accumulator, so P.V is lane-local and the only cross-lane work is the 16-lane sum of the dot
// product (four DPP adds).  The four 16-lane groups of a wave and the four waves of a
// workgroup run independent online-softmax streams that are merged once per segment.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hg {

constexpr int kInlineRanges = 64;   // range-table entries carried inside the kernel arguments
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

// pre = number of tokens in the ranges before this one (prefix sum of the range lengths);
// grp = the concatenation group the range belongs to (used by the concat path only).
struct RangeEntry {
    int32_t seq, begin, end, pre, grp;
};

// What a streaming kernel instance does with the rows it reads.
constexpr int kModeStats = 0;   // K and V -> (m, l, O) records                     (hg_attn_partial / hg_attn_full)
constexpr int kModeLogits = 1;  // K only  -> raw scaled logits                     (hg_attn_logits)
constexpr int kModeConcat = 2;  // V and given logits + group softmax stats -> sum p.v records  (hg_attn_concat)
constexpr int kConcatSlices = 32;  // partial (max, sum) records per (group, head) of the concat path

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
    const float *gs_m, *gs_l;              // concat mode: [n_groups][Hq][kConcatSlices] partial (max in log2 units, sum)
    WorkSplit ws;
    RangeTable tab;
};

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
};

struct ConcatStatsArgs {
    const float *logits;  // [Hq][ltok], natural-log units
    float *gs_m, *gs_l;   // [n_groups][Hq][kConcatSlices]
    int32_t ltok, n_q_heads;
    GroupTable groups;    // CSR over ranges
    RangeTable tab;
};

struct ConcatReduceArgs {
    const float *ws_o;        // segment records [slot][gt][D]: sums of p.v
    const float *gs_m, *gs_l;
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
    GroupTable groups;
    RangeTable tab;
};

constexpr int kSelectDirect = 0;      // one workgroup selects from the group's logits row
constexpr int kSelectCandidates = 1;  // stage 1: per part, write its top_k candidates
constexpr int kSelectFromCands = 2;   // stage 2: select among the parts' candidates

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
typedef unsigned int hg_u32x2 __attribute__((ext_vector_type(2)));

template <int VB>
struct RawVec;
template <>
struct RawVec<16> {
    hg_u32x4 d;
};
template <>
struct RawVec<8> {
    hg_u32x2 d;
};

template <int D_, bool F16_>
struct Traits {
    static constexpr int D = D_;
    static constexpr bool F16 = F16_;
    static constexpr int ES = F16_ ? 2 : 4;
    static constexpr int LANE_BYTES = D_ * ES / 16;           // bytes of a row held by one lane
    static constexpr int VB = LANE_BYTES >= 16 ? 16 : 8;      // bytes per load
    static constexpr int NV = LANE_BYTES / VB;                // loads per row per lane
    static constexpr int EPV = VB / ES;                       // elements per load
    static constexpr int EPL = NV * EPV;                      // elements per lane
    static constexpr int SEG = 16 * EPV;                      // elements covered by one wave-row load
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
        if constexpr (F16_) {
            typedef _Float16 hvec __attribute__((ext_vector_type(EPV)));
            hvec h = __builtin_bit_cast(hvec, r.d);
#pragma unroll
            for (int i = 0; i < EPV; ++i) out[i] = (float)h[i];
        } else {
            typedef float fvec __attribute__((ext_vector_type(EPV)));
            fvec f = __builtin_bit_cast(fvec, r.d);
#pragma unroll
            for (int i = 0; i < EPV; ++i) out[i] = f[i];
        }
    }
};

// ---- streaming kernel --------------------------------------------------------------------------

// Merge (m_b, l_b, acc_b) into (m, l, acc); all maxima in log2 units, kNegBig = empty.
template <int N>
__device__ __forceinline__ void merge_state(float &m, float &l, float *acc, float m_b, float l_b, const float *acc_b)
{
    float mx = fmaxf(m, m_b);
    float wa = fast_exp2(m - mx), wb = fast_exp2(m_b - mx);
    m = mx;
    l = l * wa + l_b * wb;
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = acc[i] * wa + acc_b[i] * wb;
}

// Global softmax maximum (log2 units) of (concat group, query head) from the kConcatSlices
// partial records.  Computed by one wave cooperatively.
__device__ __forceinline__ float group_softmax_max(const float *gs_m, int64_t base, int lane)
{
    float m = lane < kConcatSlices ? gs_m[base + lane] : kNegBig;
#pragma unroll
    for (int step = 32; step >= 1; step >>= 1) m = fmaxf(m, __shfl_xor(m, step, 64));
    return m;
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

// (One workgroup per compute unit is launched on long inputs, so the register allocator is told
// that two waves per SIMD is all the occupancy this kernel wants.)
template <typename TR, int GT, int U, int MODE, bool PAGED>
__global__ __launch_bounds__(kValuBlock) __attribute__((amdgpu_waves_per_eu(1, 2))) void hg_partial_kernel(const PartialArgs a)
{
    constexpr int D = TR::D, EPL = TR::EPL, NV = TR::NV, EPV = TR::EPV, ES = TR::ES;
    constexpr int CH = 4 * U;  // tokens one wave takes per iteration

    __shared__ float sm[kValuWaves][GT][D + 2];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 15, grp = lane >> 4;

    for_each_segment(a.ws, a.tab, [&](int stream, int r_idx, const RangeEntry &e, int t0, int t1, int col0, int64_t slot) __attribute__((always_inline)) {
    const int seq = e.seq;
    const int hk = stream / a.ws.n_chunks;
    const int chunk = stream - hk * a.ws.n_chunks;
    const int g0 = chunk * GT;                              // first head of this chunk inside its group
    const int nh = min(GT, a.ws.group - g0);                // valid heads in this chunk
    const int h0 = hk * a.ws.group + g0;                    // first query head

    // q fragments, scaled into the log2 domain (natural-log domain when exporting logits)
    float qf[GT][EPL];
    if constexpr (MODE != kModeConcat) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const int h = h0 + (g < nh ? g : 0);
            const char *qrow = static_cast<const char *>(a.q) + ((int64_t)seq * a.ws.n_q_heads + h) * (int64_t)(D * ES);
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                typename TR::Raw raw = TR::template load<false>(qrow, sub, j);
                TR::widen(raw, &qf[g][j * EPV]);
            }
#pragma unroll
            for (int i = 0; i < EPL; ++i) qf[g][i] *= a.qscale;
        }
    }

    // concat mode: the group's global softmax maximum per head (the division by the global sum
    // happens once, in the reduce kernel), and the logits rows
    float gmax[GT];
    const float *lrow[GT];
    if constexpr (MODE == kModeConcat) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const int h = h0 + (g < nh ? g : 0);
            gmax[g] = group_softmax_max(a.gs_m, ((int64_t)e.grp * a.ws.n_q_heads + h) * kConcatSlices, lane);
            lrow[g] = a.logits + (int64_t)h * a.ws.ltok + (col0 - t0);  // lrow[g][tok] is the logit of token tok
        }
    }

    float m[GT], l[GT], acc[GT][EPL];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        m[g] = MODE == kModeConcat ? 0.f : kNegBig;  // concat records are plain sums: equal maxima, weight 1
        l[g] = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[g][i] = 0.f;
    }

    // contiguous cache: one slab per (sequence, KV head); paged cache: the head's offset inside a
    // block, the block comes from the table
    const int64_t slab = (PAGED ? 0 : (int64_t)seq * a.stride_b) + (int64_t)hk * a.stride_h;
    const char *kbase = static_cast<const char *>(a.k) + slab * ES;
    const char *vbase = static_cast<const char *>(a.v) + slab * ES;
    const int64_t row_bytes = a.stride_t * ES;
    const int64_t block_bytes = a.stride_b * ES;
    const int32_t *table = PAGED ? a.pages.table + (int64_t)seq * a.pages.max_blocks : nullptr;

    // physical blocks of the U tokens this lane group takes in the iteration starting at tbb;
    // they are looked up one iteration ahead so that the row loads never wait for the table
    int pg[U], pg_next[U];
    auto lookup = [&](int tbb, int(&out)[U]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int tok = tbb + 4 * u + grp;
            out[u] = table[(tok < t1 ? tok : t1 - 1) >> a.pages.shift];
        }
    };
    if constexpr (PAGED) {
        if (t0 + wave * CH < t1) lookup(t0 + wave * CH, pg);
    }

    for (int tb = t0 + wave * CH; tb < t1; tb += kValuWaves * CH) {
        typename TR::Raw kraw[U][NV], vraw[U][NV];
        bool valid[U];
        int tokc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int tok = tb + 4 * u + grp;
            valid[u] = tok < t1;
            tokc[u] = valid[u] ? tok : t1 - 1;  // clamp: never read past the segment
            const int64_t off = PAGED ? (int64_t)pg[u] * block_bytes + (int64_t)(tokc[u] & a.pages.mask) * row_bytes
                                      : (int64_t)tokc[u] * row_bytes;
            if constexpr (MODE != kModeConcat) {
#pragma unroll
                for (int j = 0; j < NV; ++j) kraw[u][j] = TR::template load<true>(kbase + off, sub, j);
            }
            if constexpr (MODE != kModeLogits) {
#pragma unroll
                for (int j = 0; j < NV; ++j) vraw[u][j] = TR::template load<true>(vbase + off, sub, j);
            }
        }

        if constexpr (PAGED) {
            if (tb + kValuWaves * CH < t1) lookup(tb + kValuWaves * CH, pg_next);
        }
        // Every load of this iteration is issued before any of its arithmetic: the bytes in
        // flight per wave are what the kernel's bandwidth rests on, and without this fence the
        // instruction scheduler is free to trade them for a lower register count.
        __builtin_amdgcn_sched_barrier(0);

        // logits of the U tokens of this lane group, for every head of the chunk
        float s[GT][U];
        if constexpr (MODE != kModeConcat) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float kf[EPL];
#pragma unroll
                for (int j = 0; j < NV; ++j) TR::widen(kraw[u][j], &kf[j * EPV]);
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    float d = 0.f;
#pragma unroll
                    for (int i = 0; i < EPL; ++i) d = fmaf(qf[g][i], kf[i], d);
                    d = row16_sum(d);
                    s[g][u] = valid[u] ? d : -INFINITY;
                }
            }
        }

        if constexpr (MODE == kModeLogits) {
            // lane `g` of each 16-lane group stores head g's logit of that group's token
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int g = 0; g < GT; ++g)
                    if (sub == g && g < nh && valid[u])
                        a.logits[(int64_t)(h0 + g) * a.ws.ltok + col0 + (tokc[u] - t0)] = s[g][u];
        }

        if constexpr (MODE != kModeLogits) {
        float p[GT][U];
        if constexpr (MODE == kModeStats) {
            // online softmax update
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                float mx = m[g];
#pragma unroll
                for (int u = 0; u < U; ++u) mx = fmaxf(mx, s[g][u]);
                const float alpha = fast_exp2(m[g] - mx);
                m[g] = mx;
                float ls = 0.f;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    p[g][u] = fast_exp2(s[g][u] - mx);
                    ls += p[g][u];
                }
                l[g] = l[g] * alpha + ls;
#pragma unroll
                for (int i = 0; i < EPL; ++i) acc[g][i] *= alpha;
            }
        } else {
            // numerators exp(s - M) of the ONE softmax over the concatenated logits of the group
            // (the mask is applied as a product so that every logit load stays unconditional and
            // all of them are issued together with the V loads)
            float sv[GT][U];
#pragma unroll
            for (int g = 0; g < GT; ++g)
#pragma unroll
                for (int u = 0; u < U; ++u) sv[g][u] = lrow[g][tokc[u]];
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                float ls = 0.f;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    p[g][u] = fast_exp2(sv[g][u] * kLog2e - gmax[g]) * (valid[u] ? 1.f : 0.f);
                    ls += p[g][u];
                }
                l[g] += ls;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float vf[EPL];
#pragma unroll
            for (int j = 0; j < NV; ++j) TR::widen(vraw[u][j], &vf[j * EPV]);
#pragma unroll
            for (int g = 0; g < GT; ++g)
#pragma unroll
                for (int i = 0; i < EPL; ++i) acc[g][i] = fmaf(p[g][u], vf[i], acc[g][i]);
        }
        }  // MODE != kModeLogits
        if constexpr (PAGED) {
#pragma unroll
            for (int u = 0; u < U; ++u) pg[u] = pg_next[u];
        }
    }
    if constexpr (MODE == kModeLogits) return;  // nothing to merge or record

    // merge the four lane groups of the wave (lanes xor 16, xor 32)
#pragma unroll
    for (int g = 0; g < GT; ++g) {
#pragma unroll
        for (int step = 16; step <= 32; step <<= 1) {
            float m_b = __shfl_xor(m[g], step, 64);
            float l_b = __shfl_xor(l[g], step, 64);
            float acc_b[EPL];
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc_b[i] = __shfl_xor(acc[g][i], step, 64);
            merge_state<EPL>(m[g], l[g], acc[g], m_b, l_b, acc_b);
        }
        if (grp == 0) {
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int i = 0; i < EPV; ++i) sm[wave][g][TR::vec_offset(sub, j) + i] = acc[g][j * EPV + i];
            if (sub == 0) {
                sm[wave][g][D] = m[g];
                sm[wave][g][D + 1] = l[g];
            }
        }
    }
    __syncthreads();

    // merge the waves; one thread per (head, channel)
    for (int idx = threadIdx.x; idx < GT * D; idx += kValuBlock) {
        const int g = idx / D, c = idx - g * D;
        if (g >= nh) continue;
        float mx = kNegBig;
#pragma unroll
        for (int w = 0; w < kValuWaves; ++w) mx = fmaxf(mx, sm[w][g][D]);
        float lt = 0.f, ot = 0.f;
#pragma unroll
        for (int w = 0; w < kValuWaves; ++w) {
            const float wt = fast_exp2(sm[w][g][D] - mx);
            lt += wt * sm[w][g][D + 1];
            ot += wt * sm[w][g][c];
        }
        write_segment_result<D>(a, slot * GT + g, r_idx, h0 + g, c, mx, lt, ot);
    }
    __syncthreads();  // the next segment reuses sm
    });
}

// ---- streaming kernel for grouped-query attention (fp16, head_dim 128) on the matrix cores -----
//
// With G query heads sharing one KV head, every K and V byte feeds G dot products; on the
// vector ALU that makes the scan arithmetic-bound from G = 4 upwards.  Here up to 16 query heads
// of a KV head form the M dimension of v_mfma_f32_16x16x32_f16, so the arithmetic is a few
// percent of the matrix cores and the kernel is bandwidth-bound again.
//
// Per wave and per block of 32 tokens:
//   K   8 coalesced 16-byte loads per lane (4 whole rows per instruction) -> wave-private LDS
//       (rows padded to 272 bytes) -> read back "token per lane": lane l gets token l%16,
//       channels 8*(4kk + l/16)..+7, which IS the B operand of MFMA kk (the contraction runs
//       over channels, and Q is laid out with the same channel grouping as A operand).
//       S = Q.K^T lands as: lane (n = l%16, rg = l/16) holds heads 4rg..4rg+3 of token n.
//   softmax  row max over the 16 token lanes by DPP, running (m, l) per head, P = exp2(S - m).
//       P is split into an fp16 head and an fp16 remainder (p = ph + pl to ~22 bits), so the
//       fp16 MFMA does not cost precision in the weights.
//   P   goes through 2 KiB of LDS to become the A operand (lane l: head l%16, tokens of group l/16).
//   V   8 coalesced 16-byte loads per lane; the contraction now runs over tokens, which sit in a
//       lane's own registers (8 tokens x 8 channels), so an in-lane 8x8 transpose of halves
//       (32 v_perm_b32) yields the B operands: no LDS, no cross-lane traffic.  Token j of lane
//       group g is block token 16*(j%2) + 4*(j/2) + g, so that each load instruction still
//       fetches 4 adjacent rows and the two halves of a P word come from one lane.
//       O[nb] (nb = 0..7) holds out[head 4rg + r][channel 8n + nb].

constexpr int kGqaHeads = 16;            // query heads per workgroup (M of the MFMA)
constexpr int kGqaBlockTokens = 32;      // tokens per wave iteration (K of the P.V MFMA)
constexpr int kGqaKRow = 272;            // padded LDS row: 256 bytes + 16 so that 16 rows spread over all banks
constexpr int kGqaKBytes = kGqaBlockTokens * kGqaKRow;
constexpr int kGqaPBytes = kGqaHeads * kGqaBlockTokens * 2;
constexpr int kGqaWaveBytes = kGqaKBytes + 2 * kGqaPBytes;

typedef _Float16 hg_h8 __attribute__((ext_vector_type(8)));
typedef float hg_f4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float row16_max(float x)
{
    x = fmaxf(x, dpp_move<0xB1>(x));
    x = fmaxf(x, dpp_move<0x4E>(x));
    x = fmaxf(x, dpp_move<0x141>(x));
    x = fmaxf(x, dpp_move<0x140>(x));
    return x;
}

// LDS traffic between the lanes of ONE wave: the hardware keeps a wave's LDS operations in
// order; this only stops the compiler from moving accesses across the hand-over point.
__device__ __forceinline__ void wave_lds_handover()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int MODE, bool PAGED>
__global__ __launch_bounds__(kGqaBlock, kGqaWaves <= 4 ? 2 : 1) void hg_partial_gqa_kernel(const PartialArgs a)
{
    static_assert(!PAGED || MODE == kModeStats, "paged caches are only wired into the statistics mode");
    constexpr int D = 128;
    constexpr int kMergeBytes = kGqaWaves * kGqaHeads * (D + 2) * 4;
    constexpr int kSmemBytes = kGqaWaves * kGqaWaveBytes > kMergeBytes ? kGqaWaves * kGqaWaveBytes : kMergeBytes;
    __shared__ __align__(16) char smem[kSmemBytes];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, rg = lane >> 4;

    char *kls = smem + wave * kGqaWaveBytes;
    char *pls = kls + kGqaKBytes;

    for_each_segment(a.ws, a.tab, [&](int stream, int r_idx, const RangeEntry &e, int t0, int t1, int col0, int64_t slot) __attribute__((always_inline)) {
    const int seq = e.seq;
    const int hk = stream / a.ws.n_chunks;
    const int chunk = stream - hk * a.ws.n_chunks;
    const int g0 = chunk * kGqaHeads;
    const int nh = min(kGqaHeads, a.ws.group - g0);
    const int h0 = hk * a.ws.group + g0;

    // Q as A operand: lane l holds head l%16, channels 8*(4kk + l/16)..+7 for kk = 0..3
    hg_h8 qa[4];
    if constexpr (MODE != kModeConcat) {
        const _Float16 *qrow = static_cast<const _Float16 *>(a.q) + ((int64_t)seq * a.ws.n_q_heads + h0 + (n < nh ? n : 0)) * D;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            hg_u32x4 raw = *reinterpret_cast<const hg_u32x4 *>(qrow + 8 * (4 * kk + rg));
            if (n >= nh) raw = hg_u32x4{0u, 0u, 0u, 0u};
            qa[kk] = __builtin_bit_cast(hg_h8, raw);
        }
    }

    // concat mode: global softmax maximum (log2 units) of this lane's head n, and its logits
    // row (lrow[tok] is the logit of token tok)
    float gmax = 0.f;
    const float *lrow = nullptr;
    if constexpr (MODE == kModeConcat) {
        const int h = h0 + (n < nh ? n : 0);
        const int64_t base = ((int64_t)e.grp * a.ws.n_q_heads + h) * kConcatSlices;
        gmax = kNegBig;
        for (int z = 0; z < kConcatSlices; ++z) gmax = fmaxf(gmax, a.gs_m[base + z]);
        lrow = a.logits + (int64_t)h * a.ws.ltok + (col0 - t0);
    }

    float m[4], lsum[4];
    hg_f4 o[8];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        m[r] = MODE == kModeConcat ? 0.f : kNegBig;  // concat records are plain sums
        lsum[r] = 0.f;
    }
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) o[nb] = hg_f4{0.f, 0.f, 0.f, 0.f};

    const int64_t slab = (PAGED ? 0 : (int64_t)seq * a.stride_b) + (int64_t)hk * a.stride_h;
    const char *kbase = static_cast<const char *>(a.k) + slab * 2 + n * 16;
    const char *vbase = static_cast<const char *>(a.v) + slab * 2 + n * 16;
    const int64_t row_bytes = a.stride_t * 2;
    const int64_t block_bytes = a.stride_b * 2;
    const int32_t *table = PAGED ? a.pages.table + (int64_t)seq * a.pages.max_blocks : nullptr;

    // Paged cache: physical blocks of the 8 tokens tb + 4x + rg (x = 0..7) a lane touches in a
    // block; K load i uses x = i, V load j uses x = 4*(j&1) + (j>>1), the same 8 tokens.
    auto lookup = [&](int tb, int(&pg)[8]) __attribute__((always_inline)) {
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int tok = tb + 4 * x + rg;
            pg[x] = table[(tok < t1 ? tok : t1 - 1) >> a.pages.shift];
        }
    };
    auto row_offset = [&](int tok, int page) __attribute__((always_inline)) -> int64_t {
        return PAGED ? (int64_t)page * block_bytes + (int64_t)(tok & a.pages.mask) * row_bytes : (int64_t)tok * row_bytes;
    };

    // The 8 K-row loads and the 8 V-row loads of one 32-token block (8 KiB each per wave).
    auto load_k = [&](int tb, hg_u32x4(&kreg)[8], const int(&pg)[8]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int tok = tb + 4 * i + rg;
            tok = tok < t1 ? tok : t1 - 1;  // clamp: never read past the segment
            kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const hg_u32x4 *>(kbase + row_offset(tok, pg[i])));
        }
    };
    auto load_v = [&](int tb, hg_u32x4(&vreg)[8], const int(&pg)[8]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // token j of lane group rg: interleaved so that S halves pair up (stats mode), or the
            // 8 consecutive tokens whose logits this lane reads (concat mode)
            int tok = MODE == kModeConcat ? tb + 8 * rg + j : tb + 16 * (j & 1) + 4 * (j >> 1) + rg;
            tok = tok < t1 ? tok : t1 - 1;
            vreg[j] = __builtin_nontemporal_load(
                reinterpret_cast<const hg_u32x4 *>(vbase + row_offset(tok, pg[4 * (j & 1) + (j >> 1)])));
        }
    };
    // pages of the next block (pg1) and of the one after (pg2, in flight); unused when not paged
    int pg1[8] = {0, 0, 0, 0, 0, 0, 0, 0}, pg2[8] = {0, 0, 0, 0, 0, 0, 0, 0};

    // One block.  Software pipeline with a single register buffer: the K rows of the next block
    // are requested as soon as this block's K sits in LDS, its V rows as soon as this block's V
    // has been consumed, so a wave always has 8-16 KiB in flight while it computes.
    auto compute_block = [&](int tb, int tb_next, hg_u32x4(&kreg)[8], hg_u32x4(&vreg)[8]) __attribute__((always_inline)) {
        // K: registers -> LDS (row per token) -> B operands (token per lane)
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<hg_u32x4 *>(kls + (4 * i + rg) * kGqaKRow + n * 16) = kreg[i];
        wave_lds_handover();
        if (tb_next < t1) load_k(tb_next, kreg, pg1);
        hg_f4 s[2];
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            s[hf] = hg_f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                hg_u32x4 raw = *reinterpret_cast<const hg_u32x4 *>(kls + (16 * hf + n) * kGqaKRow + (4 * kk + rg) * 16);
                s[hf] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[kk], __builtin_bit_cast(hg_h8, raw), s[hf], 0, 0, 0);
            }
        }

        const bool ok0 = tb + n < t1, ok1 = tb + 16 + n < t1;
        if constexpr (MODE == kModeLogits) {
            // export: lane (n, rg) holds heads 4rg..4rg+3 of tokens tb + n and tb + 16 + n
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (4 * rg + r >= nh) continue;
                float *row = a.logits + (int64_t)(h0 + 4 * rg + r) * a.ws.ltok + col0 + (tb - t0);
                if (ok0) row[n] = s[0][r] * a.qscale;
                if (ok1) row[16 + n] = s[1][r] * a.qscale;
            }
            wave_lds_handover();  // the next block overwrites the K staging area
            return;
        }

        // online softmax on S (lane: token n of each half, heads 4rg..4rg+3)
        float alpha[4];
        uint32_t ph[4], pl[4];  // packed (half 0, half 1) weights: fp16 head and fp16 remainder
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float s0 = ok0 ? s[0][r] * a.qscale : -INFINITY;
            const float s1 = ok1 ? s[1][r] * a.qscale : -INFINITY;
            const float mx = fmaxf(m[r], row16_max(fmaxf(s0, s1)));
            alpha[r] = fast_exp2(m[r] - mx);
            m[r] = mx;
            const float p0 = fast_exp2(s0 - mx), p1 = fast_exp2(s1 - mx);
            lsum[r] = lsum[r] * alpha[r] + (p0 + p1);
            const _Float16 h0f = (_Float16)p0, h1f = (_Float16)p1;
            const _Float16 l0f = (_Float16)(p0 - (float)h0f), l1f = (_Float16)(p1 - (float)h1f);
            typedef _Float16 h2 __attribute__((ext_vector_type(2)));
            ph[r] = __builtin_bit_cast(uint32_t, h2{h0f, h1f});
            pl[r] = __builtin_bit_cast(uint32_t, h2{l0f, l1f});
        }
        // P -> LDS as [head][group g = n%4][j = 2*(n/4) + half], then read as A operand
        {
            const int col = (n & 3) * 16 + (n >> 2) * 4;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                *reinterpret_cast<uint32_t *>(pls + (4 * rg + r) * 64 + col) = ph[r];
                *reinterpret_cast<uint32_t *>(pls + kGqaPBytes + (4 * rg + r) * 64 + col) = pl[r];
            }
        }
        wave_lds_handover();
        const hg_h8 pa_hi = __builtin_bit_cast(hg_h8, *reinterpret_cast<const hg_u32x4 *>(pls + n * 64 + rg * 16));
        const hg_h8 pa_lo =
            __builtin_bit_cast(hg_h8, *reinterpret_cast<const hg_u32x4 *>(pls + kGqaPBytes + n * 64 + rg * 16));

        // V: in-lane transpose of halves, then O[nb] = alpha * O[nb] + P . V[:, channel 8n + nb]
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
            const uint32_t sel = (nb & 1) ? 0x07060302u : 0x05040100u;
            hg_u32x4 braw;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                braw[jj] = __builtin_amdgcn_perm(vreg[2 * jj + 1][nb >> 1], vreg[2 * jj][nb >> 1], sel);
            const hg_h8 b = __builtin_bit_cast(hg_h8, braw);
#pragma unroll
            for (int r = 0; r < 4; ++r) o[nb][r] *= alpha[r];
            o[nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa_hi, b, o[nb], 0, 0, 0);
            o[nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa_lo, b, o[nb], 0, 0, 0);
        }
        if (tb_next < t1) {
            if constexpr (PAGED) {
                // table look-up for the block after next goes out BEFORE the V loads: the K loads
                // of that block then only wait for what was issued earlier (loads return in order)
                const int tb_nn = tb_next + (tb_next - tb);
                if (tb_nn < t1) lookup(tb_nn, pg2);
            }
            load_v(tb_next, vreg, pg1);
            if constexpr (PAGED) {
#pragma unroll
                for (int x = 0; x < 8; ++x) pg1[x] = pg2[x];
            }
        }
        wave_lds_handover();  // the next block overwrites the K and P staging areas
    };

    // Concat mode block: the numerators exp(s - M) of the ONE softmax over the group's concatenated
    // logits come straight from memory in A-operand order (lane: head n, tokens tb + 8rg .. + 7);
    // they lie in (0, 1], so the fp16 head + remainder keeps them to ~22 bits.  The division by the
    // global sum happens once, in the reduce kernel.
    auto concat_block = [&](int tb, int tb_next, hg_u32x4(&vreg)[8]) __attribute__((always_inline)) {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        hg_u32x4 hi_raw, lo_raw;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            float pj[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int tok = tb + 8 * rg + 2 * jj + x;
                const float sv = lrow[tok < t1 ? tok : t1 - 1];  // unconditional load; masked by a product
                pj[x] = fast_exp2(sv * kLog2e - gmax) * ((tok < t1 && n < nh) ? 1.f : 0.f);
            }
            const _Float16 h0f = (_Float16)pj[0], h1f = (_Float16)pj[1];
            const _Float16 l0f = (_Float16)(pj[0] - (float)h0f), l1f = (_Float16)(pj[1] - (float)h1f);
            hi_raw[jj] = __builtin_bit_cast(uint32_t, h2{h0f, h1f});
            lo_raw[jj] = __builtin_bit_cast(uint32_t, h2{l0f, l1f});
        }
        const hg_h8 pa_hi = __builtin_bit_cast(hg_h8, hi_raw), pa_lo = __builtin_bit_cast(hg_h8, lo_raw);
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
            const uint32_t sel = (nb & 1) ? 0x07060302u : 0x05040100u;
            hg_u32x4 braw;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                braw[jj] = __builtin_amdgcn_perm(vreg[2 * jj + 1][nb >> 1], vreg[2 * jj][nb >> 1], sel);
            const hg_h8 b = __builtin_bit_cast(hg_h8, braw);
            o[nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa_hi, b, o[nb], 0, 0, 0);
            o[nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa_lo, b, o[nb], 0, 0, 0);
        }
        if (tb_next < t1) load_v(tb_next, vreg, pg1);
    };

    {
        constexpr int kStride = kGqaWaves * kGqaBlockTokens;
        int tb = t0 + wave * kGqaBlockTokens;
        if constexpr (MODE == kModeStats) {
            hg_u32x4 kreg[8], vreg[8];
            if (tb < t1) {
                if constexpr (PAGED) {
                    lookup(tb, pg2);
                    if (tb + kStride < t1) lookup(tb + kStride, pg1);
                }
                load_k(tb, kreg, pg2);
                load_v(tb, vreg, pg2);
            }
            while (tb < t1) {
                compute_block(tb, tb + kStride, kreg, vreg);
                tb += kStride;
            }
        } else {
            // Only K (logits) or only V (concat) is read: two register buffers, so that two
            // blocks (16 KiB per wave) are in flight as in the statistics mode.
            hg_u32x4 ra[8], rb[8];
            auto load_one = [&](int t, hg_u32x4(&reg)[8]) __attribute__((always_inline)) {
                if constexpr (MODE == kModeLogits)
                    load_k(t, reg, pg1);
                else
                    load_v(t, reg, pg1);
            };
            auto compute_one = [&](int t, hg_u32x4(&reg)[8]) __attribute__((always_inline)) {
                if constexpr (MODE == kModeLogits)
                    compute_block(t, t + 2 * kStride, reg, reg);
                else
                    concat_block(t, t + 2 * kStride, reg);
            };
            if (tb < t1) load_one(tb, ra);
            if (tb + kStride < t1) load_one(tb + kStride, rb);
            while (tb < t1) {
                compute_one(tb, ra);
                tb += kStride;
                if (tb >= t1) break;
                compute_one(tb, rb);
                tb += kStride;
            }
        }
    }
    if constexpr (MODE == kModeLogits) return;  // nothing to merge or record

    // per-wave state -> LDS (staging areas are dead now), then merge the four waves
    __syncthreads();
    float(*sm)[kGqaHeads][D + 2] = reinterpret_cast<float(*)[kGqaHeads][D + 2]>(smem);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float lrow = row16_sum(lsum[r]);
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) sm[wave][4 * rg + r][8 * n + nb] = o[nb][r];
        if (n == 0) {
            sm[wave][4 * rg + r][D] = m[r];
            sm[wave][4 * rg + r][D + 1] = lrow;
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < kGqaHeads * D; idx += kGqaBlock) {
        const int g = idx / D, c = idx - g * D;
        if (g >= nh) continue;
        float mx = kNegBig;
#pragma unroll
        for (int w = 0; w < kGqaWaves; ++w) mx = fmaxf(mx, sm[w][g][D]);
        float lt = 0.f, ot = 0.f;
#pragma unroll
        for (int w = 0; w < kGqaWaves; ++w) {
            const float wt = fast_exp2(sm[w][g][D] - mx);
            lt += wt * sm[w][g][D + 1];
            ot += wt * sm[w][g][c];
        }
        write_segment_result<D>(a, slot * kGqaHeads + g, r_idx, h0 + g, c, mx, lt, ot);
    }
    __syncthreads();  // the next segment reuses the staging areas
    });
}

// ---- segment records -> range triple (or normalised output) -----------------------------------

constexpr int kReduceBlock = 512;

// Shared tail of the two combining kernels.  Each of the S = kReduceBlock / D slices has folded
// its share of the records into a running (mx, lt, ot) in ONE pass (independent loads, no
// max pre-pass, so the kernel costs a single memory round trip); the slices are merged here.
// Returns true in the threads of slice 0, which then hold the total (mx, lt, ot[c]).
template <int D>
__device__ __forceinline__ bool combine_slices(float &mx, float &lt, float &ot, int c, int sl)
{
    constexpr int S = kReduceBlock / D;
    __shared__ float s_o[S][D];
    __shared__ float s_m[S], s_l[S];
    s_o[sl][c] = ot;
    if (c == 0) {
        s_m[sl] = mx;
        s_l[sl] = lt;
    }
    __syncthreads();
    if (sl != 0) return false;
    float M = s_m[0];
#pragma unroll
    for (int i = 1; i < S; ++i) M = fmaxf(M, s_m[i]);
    lt = 0.f;
    ot = 0.f;
#pragma unroll
    for (int i = 0; i < S; ++i) {
        const float wt = fast_exp2(s_m[i] - M);
        lt += wt * s_l[i];
        ot += wt * s_o[i][c];
    }
    mx = M;
    return true;
}

// One workgroup per (range, query head).  The segment records of the range are dealt round-robin
// to kReduceBlock / D slices of D threads (one thread per channel), so that a range cut into
// hundreds of segments is not one long chain of dependent loads.
template <int D>
__global__ __launch_bounds__(kReduceBlock) void hg_segment_reduce_kernel(const ReduceArgs a)
{
    constexpr int S = kReduceBlock / D;
    const int r = blockIdx.x, h = blockIdx.y;
    const int c = threadIdx.x % D, sl = threadIdx.x / D;

    // the records of (range r, stream of head h) sit in slots w + stream * n_ranges + r for the
    // workgroups w whose span overlaps the pair's positions [p0, p1)
    const int hk = h / a.ws.group, gi = h - hk * a.ws.group;
    const int chunk = gi / a.ws.gt, gl = gi - chunk * a.ws.gt;
    const int stream = hk * a.ws.n_chunks + chunk;
    const int pre0 = table_entry(a.tab, r).pre, pre1 = table_entry(a.tab, r + 1).pre;
    const int64_t p0 = (int64_t)stream * a.ws.ltok + pre0, p1 = (int64_t)stream * a.ws.ltok + pre1;
    const int64_t w0 = pre1 > pre0 ? p0 / a.ws.span : 0;
    const int n_rec = pre1 > pre0 ? (int)((p1 - 1) / a.ws.span - w0) + 1 : 0;
    const int64_t rec0 = (w0 + (int64_t)stream * a.tab.n_ranges + r) * a.ws.gt + gl;  // record i at rec0 + i * gt

    float mx = kNegBig, lt = 0.f, ot = 0.f;  // log2 units
#pragma unroll 4
    for (int i = sl; i < n_rec; i += S) {
        const int64_t th = rec0 + (int64_t)i * a.ws.gt;
        const float mi = a.ws_m[th], li = a.ws_l[th], oi = a.ws_o[th * D + c];
        const float mn = fmaxf(mx, mi);
        const float wa = fast_exp2(mx - mn), wb = fast_exp2(mi - mn);
        lt = lt * wa + li * wb;
        ot = ot * wa + oi * wb;
        mx = mn;
    }
    if (!combine_slices<D>(mx, lt, ot, c, sl)) return;

    const int64_t rh = (int64_t)r * a.ws.n_q_heads + h;
    const bool empty = !(lt > 0.f);
    if (a.normalise) {
        a.o_out[rh * D + c] = empty ? 0.f : ot / lt;
        if (c == 0 && a.m_out) a.m_out[rh] = empty ? -INFINITY : mx * kLn2 + logf(lt);
    } else {
        a.o_out[rh * D + c] = empty ? 0.f : ot;
        if (c == 0) {
            a.m_out[rh] = empty ? -INFINITY : mx * kLn2;
            a.l_out[rh] = empty ? 0.f : lt;
        }
    }
}

// ---- exact merge of range triples ---------------------------------------------------------------

// One workgroup per (group, query head); the group's triples are dealt to the slices as above.
// Triples arrive in natural-log units and are folded in log2 units.
template <int D>
__global__ __launch_bounds__(kReduceBlock) void hg_merge_kernel(const MergeArgs a)
{
    constexpr int S = kReduceBlock / D;
    const int gidx = blockIdx.x, h = blockIdx.y;
    const int c = threadIdx.x % D, sl = threadIdx.x / D;
    const int ts = a.tab.ext ? a.tab.ext[gidx] : a.tab.inl[gidx];
    const int te = a.tab.ext ? a.tab.ext[gidx + 1] : a.tab.inl[gidx + 1];

    float mx = kNegBig, lt = 0.f, ot = 0.f;
#pragma unroll 4
    for (int t = ts + sl; t < te; t += S) {
        const int64_t th = (int64_t)t * a.n_q_heads + h;
        const float li = a.l[th], oi = a.o[th * D + c];
        const float mi = li != 0.f ? a.m[th] * kLog2e : kNegBig;  // identity element: ignored
        const float mn = fmaxf(mx, mi);
        const float wa = fast_exp2(mx - mn), wb = li != 0.f ? fast_exp2(mi - mn) : 0.f;
        lt = lt * wa + li * wb;
        ot = ot * wa + oi * wb;
        mx = mn;
    }
    if (!combine_slices<D>(mx, lt, ot, c, sl)) return;

    const int64_t gh = (int64_t)gidx * a.n_q_heads + h;
    const bool empty = !(lt > 0.f);
    a.out[gh * D + c] = empty ? 0.f : ot / lt;
    if (c == 0 && a.lse) a.lse[gh] = empty ? -INFINITY : mx * kLn2 + logf(lt);
}

// ---- concat path: one softmax over the concatenated logits of a group --------------------------

__device__ __forceinline__ int group_entry(const GroupTable &g, int i) { return g.ext ? g.ext[i] : g.inl[i]; }

// Partial (max, sum of exp) of one slice of a group's logits row.  The ranges of a group are
// consecutive table entries, so their logits are one contiguous piece [c0, c1) of the row: the
// concatenation the paper describes is already how the logits are stored.
// Grid (kConcatSlices, n_q_heads, n_groups), 256 threads.
__global__ __launch_bounds__(256) void hg_concat_stats_kernel(const ConcatStatsArgs a)
{
    __shared__ float s_red[4];
    const int z = blockIdx.x, h = blockIdx.y, gi = blockIdx.z;
    const int c0 = table_entry(a.tab, group_entry(a.groups, gi)).pre;
    const int c1 = table_entry(a.tab, group_entry(a.groups, gi + 1)).pre;
    const int per = (c1 - c0 + kConcatSlices - 1) / kConcatSlices;
    const int b = c0 + z * per < c1 ? c0 + z * per : c1;
    const int e = b + per < c1 ? b + per : c1;
    const float *row = a.logits + (int64_t)h * a.ltok;

    // one pass: every thread folds groups of four logits into a running (max, sum) pair
    float mx = kNegBig, lt = 0.f;
    for (int i = b + 4 * (int)threadIdx.x; i < e; i += 4 * 256) {
        float x[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = row[i + j < e ? i + j : e - 1] * kLog2e * 1.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = i + j < e ? x[j] : kNegBig;
        const float mn = fmaxf(fmaxf(mx, fmaxf(x[0], x[1])), fmaxf(x[2], x[3]));
        lt = lt * fast_exp2(mx - mn) + ((fast_exp2(x[0] - mn) + fast_exp2(x[1] - mn)) + (fast_exp2(x[2] - mn) + fast_exp2(x[3] - mn)));
        mx = mn;
    }
#pragma unroll
    for (int step = 32; step >= 1; step >>= 1) {
        const float mo = __shfl_xor(mx, step, 64), lo = __shfl_xor(lt, step, 64);
        const float mn = fmaxf(mx, mo);
        lt = lt * fast_exp2(mx - mn) + lo * fast_exp2(mo - mn);
        mx = mn;
    }
    __shared__ float s_l[4];
    if ((threadIdx.x & 63) == 0) {
        s_red[threadIdx.x >> 6] = mx;
        s_l[threadIdx.x >> 6] = lt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const float M = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) L += s_l[w] * fast_exp2(s_red[w] - M);
        const int64_t idx = ((int64_t)gi * a.n_q_heads + h) * kConcatSlices + z;
        a.gs_m[idx] = M;
        a.gs_l[idx] = L;
    }
}

// out[group][head] = (sum of the exp(s - M).v records of all segments of the group's ranges) / L,
// lse = M + log L, with (M, L) the group's global softmax statistics.  Grid (n_groups, n_q_heads).
template <int D>
__global__ __launch_bounds__(kReduceBlock) void hg_concat_reduce_kernel(const ConcatReduceArgs a)
{
    constexpr int S = kReduceBlock / D;
    __shared__ float s_o[S][D];
    const int gi = blockIdx.x, h = blockIdx.y;
    const int c = threadIdx.x % D, sl = threadIdx.x / D;
    const int hk = h / a.ws.group, gidx = h - hk * a.ws.group;
    const int chunk = gidx / a.ws.gt, gl = gidx - chunk * a.ws.gt;
    const int stream = hk * a.ws.n_chunks + chunk;
    const int r0 = group_entry(a.groups, gi), r1 = group_entry(a.groups, gi + 1);

    float ot = 0.f;
    for (int r = r0; r < r1; ++r) {
        const int pre0 = table_entry(a.tab, r).pre, pre1 = table_entry(a.tab, r + 1).pre;
        if (pre1 == pre0) continue;
        const int64_t p0 = (int64_t)stream * a.ws.ltok + pre0, p1 = (int64_t)stream * a.ws.ltok + pre1;
        const int64_t w0 = p0 / a.ws.span;
        const int n_rec = (int)((p1 - 1) / a.ws.span - w0) + 1;
        const int64_t rec0 = (w0 + (int64_t)stream * a.tab.n_ranges + r) * a.ws.gt + gl;
#pragma unroll 4
        for (int i = sl; i < n_rec; i += S) ot += a.ws_o[(rec0 + (int64_t)i * a.ws.gt) * D + c];
    }
    s_o[sl][c] = ot;
    __syncthreads();
    if (sl != 0) return;
    ot = 0.f;
#pragma unroll
    for (int i = 0; i < S; ++i) ot += s_o[i][c];
    const int64_t gh = (int64_t)gi * a.ws.n_q_heads + h;
    float mx = kNegBig, lt = 0.f;  // the group's global maximum and sum of exp
    for (int z = 0; z < kConcatSlices; ++z) {
        const float mi = a.gs_m[gh * kConcatSlices + z], li = a.gs_l[gh * kConcatSlices + z];
        const float mn = fmaxf(mx, mi);
        lt = lt * fast_exp2(mx - mn) + li * fast_exp2(mi - mn);
        mx = mn;
    }
    a.out[gh * D + c] = lt > 0.f ? ot / lt : 0.f;
    if (c == 0 && a.lse) a.lse[gh] = lt > 0.f ? mx * kLn2 + logf(lt) : -INFINITY;
}

// ---- Post-QK^T selection: top-k logits of a group, folded with their V rows into (m, l, O) ------
//
// One workgroup of 16 waves per (group, query head).
//   1. radix select on order-preserving integer keys of the fp32 logits: four 8-bit passes, each
//      a histogram over the elements that still match the prefix, find the key T of the k-th
//      largest logit and how many elements equal to T are to be kept (ties go to lower columns);
//   2. one ordered sweep compacts the kept columns into LDS in ascending (token) order: a kept
//      element's slot is (#greater before it) + min(#equal before it, k_eq), which a single
//      packed block scan provides;
//   3. the kept logits give m and the weights exp(s - m); the 16 waves gather the kept V rows
//      (four rows per wave load, 16 lanes per row as in the streaming kernel) and sum p.v.
// A group of a million tokens would keep one compute unit busy for a millisecond, so long groups
// are cut into parts: stage 1 runs steps 1-2 per part and writes the part's top_k candidates
// (the global top_k is a subset of their union, and candidates stay in ascending column order),
// stage 2 runs steps 1-3 over the candidates.

__device__ __forceinline__ uint32_t order_key(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // larger float <=> larger key
}

// Exclusive scan of v over the 1024 threads of the workgroup; total receives the sum.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *s_wave, uint32_t &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(inc, d, 64);
        if (lane >= d) inc += t;
    }
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kSelectBlock / 64; ++w) {
        const uint32_t t = s_wave[w];
        before += w < wave ? t : 0u;
        all += t;
    }
    __syncthreads();  // s_wave is reused by the next call
    total = all;
    return before + inc - v;
}

template <typename TR, int STAGE>
__global__ __launch_bounds__(kSelectBlock) void hg_select_kernel(const SelectArgs a)
{
    constexpr int D = TR::D, EPL = TR::EPL, NV = TR::NV, EPV = TR::EPV, ES = TR::ES;
    constexpr int NW = kSelectBlock / 64;
    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_wave[NW];
    __shared__ uint32_t s_prefix, s_krem;
    __shared__ int32_t s_cols[kMaxTopK];   // kept columns, later their token positions
    __shared__ float s_vals[kMaxTopK];     // kept logits, later their weights
    __shared__ float s_red[NW];
    __shared__ float s_acc[NW][D];

    const int tid = threadIdx.x, h = blockIdx.y;
    const int gi = STAGE == kSelectCandidates ? blockIdx.x / a.parts : blockIdx.x;
    const int part = STAGE == kSelectCandidates ? blockIdx.x - gi * a.parts : 0;
    const int lane = tid & 63, wave = tid >> 6;
    const int r0 = group_entry(a.groups, gi), r1 = group_entry(a.groups, gi + 1);
    const int c0 = table_entry(a.tab, r0).pre, c1 = table_entry(a.tab, r1).pre;
    const int64_t gh = (int64_t)gi * a.n_q_heads + h;

    // the values this workgroup selects from: row[0..n), element i being logits column
    // col_map ? col_map[i] : col_base + i
    const float *row;
    const int32_t *col_map = nullptr;
    int n, col_base = 0, keep;
    if constexpr (STAGE == kSelectDirect) {
        row = a.logits + (int64_t)h * a.ltok + c0;
        n = c1 - c0;
        col_base = c0;
        keep = n < a.top_k ? n : a.top_k;
    } else if constexpr (STAGE == kSelectCandidates) {
        const int per = (c1 - c0 + a.parts - 1) / a.parts;
        const int b = c0 + part * per < c1 ? c0 + part * per : c1;
        const int e = b + per < c1 ? b + per : c1;
        row = a.logits + (int64_t)h * a.ltok + b;
        n = e - b;
        col_base = b;
        keep = n < a.top_k ? n : a.top_k;
    } else {
        const int64_t base = gh * a.parts * (int64_t)a.top_k;
        row = a.cand_val + base;
        col_map = a.cand_col + base;
        n = c1 > c0 ? a.parts * a.top_k : 0;  // padded with -inf entries, which sort below every logit
        keep = c1 - c0 < a.top_k ? c1 - c0 : a.top_k;
    }

    if constexpr (STAGE == kSelectCandidates) {
        // pad the part's candidate slots; the kept ones are overwritten below
        const int64_t base = (gh * a.parts + part) * (int64_t)a.top_k;
        for (int j = tid + keep; j < a.top_k; j += kSelectBlock) {
            a.cand_val[base + j] = -INFINITY;
            a.cand_col[base + j] = 0;
        }
        if (n == 0) return;
    } else {
        if (a.sel)
            for (int j = tid + keep; j < a.top_k; j += kSelectBlock) a.sel[gh * a.top_k + j] = -1;
        if (n == 0) {
            if (tid < D) a.o[gh * D + tid] = 0.f;
            if (tid == 0) {
                a.m[gh] = -INFINITY;
                a.l[gh] = 0.f;
            }
            return;
        }
    }

    // 1. radix select
    uint32_t prefix = 0, mask = 0, krem = (uint32_t)keep;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) s_hist[tid] = 0;
        __syncthreads();
        for (int i0 = 0; i0 < n; i0 += 8 * kSelectBlock) {  // eight loads in flight per thread
            float x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = i0 + j * kSelectBlock + tid;
                x[j] = row[i < n ? i : n - 1];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t u = order_key(x[j]);
                if (i0 + j * kSelectBlock + tid < n && (u & mask) == prefix) atomicAdd(&s_hist[(u >> shift) & 255u], 1u);
            }
        }
        __syncthreads();
        // the digit d with  #(digits > d) < krem <= #(digits >= d):  scan the bins from the top
        {
            const uint32_t cnt = tid < 256 ? s_hist[255 - tid] : 0u;
            uint32_t total;
            const uint32_t above = block_exclusive_scan(cnt, s_wave, total);
            if (tid < 256 && above < krem && above + cnt >= krem) {
                s_prefix = prefix | ((uint32_t)(255 - tid) << shift);
                s_krem = krem - above;
            }
        }
        __syncthreads();
        prefix = s_prefix;
        krem = s_krem;
        mask |= 0xffu << shift;
    }
    const uint32_t T = prefix, k_eq = krem;  // keep every key > T and the first k_eq keys == T

    // 2. ordered compaction of the kept columns; every thread owns kRun consecutive columns of a
    //    chunk, so one block scan serves kRun * 1024 elements
    constexpr int kRun = 8;
    uint32_t run_gt = 0, run_eq = 0;
    for (int base = 0; base < n; base += kRun * kSelectBlock) {
        const int i0 = base + kRun * tid;
        float x[kRun];
        uint32_t cnt = 0;  // low half: keys > T, high half: keys == T
#pragma unroll
        for (int j = 0; j < kRun; ++j) {
            x[j] = row[i0 + j < n ? i0 + j : n - 1];
            const uint32_t u = order_key(x[j]);
            if (i0 + j < n) cnt += (u > T ? 1u : 0u) + (u == T ? 0x10000u : 0u);
        }
        uint32_t total;
        const uint32_t scan = block_exclusive_scan(cnt, s_wave, total);
        uint32_t gt_before = run_gt + (scan & 0xffffu), eq_before = run_eq + (scan >> 16);
#pragma unroll
        for (int j = 0; j < kRun; ++j) {
            const uint32_t u = order_key(x[j]);
            const bool in = i0 + j < n, gt = in && u > T, eq = in && u == T;
            if (gt || (eq && eq_before < k_eq)) {
                const uint32_t pos = gt_before + (eq_before < k_eq ? eq_before : k_eq);
                s_cols[pos] = col_map ? col_map[i0 + j] : col_base + i0 + j;
                s_vals[pos] = x[j];
            }
            gt_before += gt ? 1u : 0u;
            eq_before += eq ? 1u : 0u;
        }
        run_gt += total & 0xffffu;
        run_eq += total >> 16;
    }
    __syncthreads();

    if constexpr (STAGE == kSelectCandidates) {
        const int64_t base = (gh * a.parts + part) * (int64_t)a.top_k;
        for (int j = tid; j < keep; j += kSelectBlock) {
            a.cand_val[base + j] = s_vals[j];
            a.cand_col[base + j] = s_cols[j];
        }
        return;
    }

    // 3a. m = max kept logit; weights; l
    float mx = -INFINITY;
    for (int j = tid; j < keep; j += kSelectBlock) mx = fmaxf(mx, s_vals[j]);
#pragma unroll
    for (int step = 32; step >= 1; step >>= 1) mx = fmaxf(mx, __shfl_xor(mx, step, 64));
    if (lane == 0) s_red[wave] = mx;
    __syncthreads();
    mx = s_red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) mx = fmaxf(mx, s_red[w]);
    __syncthreads();
    float lt = 0.f;
    const int seq = table_entry(a.tab, r0).seq;
    for (int j = tid; j < keep; j += kSelectBlock) {
        const float w = fast_exp2((s_vals[j] - mx) * kLog2e);
        lt += w;
        // column -> token position: the range of the group that holds the column
        const int col = s_cols[j];
        int lo = r0, hi = r1;  // pre[lo] <= col < pre[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (table_entry(a.tab, mid).pre <= col)
                lo = mid;
            else
                hi = mid;
        }
        const RangeEntry e = table_entry(a.tab, lo);
        const int tok = e.begin + (col - e.pre);
        s_cols[j] = tok;
        s_vals[j] = w;
        if (a.sel) a.sel[gh * a.top_k + j] = tok;
    }
#pragma unroll
    for (int step = 32; step >= 1; step >>= 1) lt += __shfl_xor(lt, step, 64);
    if (lane == 0) s_red[wave] = lt;
    __syncthreads();
    lt = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) lt += s_red[w];

    // 3b. gather the kept V rows: lane group grp of wave `wave` takes kept entries
    //     4*wave + grp, + 64, + 128, ...
    const int sub = lane & 15, grp = lane >> 4;
    const int hk = h / a.group;
    const char *vbase = static_cast<const char *>(a.v) + ((int64_t)seq * a.stride_b + (int64_t)hk * a.stride_h) * ES;
    const int64_t row_bytes = a.stride_t * ES;
    float acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;
    for (int j = 4 * wave + grp; j < keep; j += 4 * NW) {
        const float w = s_vals[j];
        const char *vrow = vbase + (int64_t)s_cols[j] * row_bytes;
        float vf[EPL];
#pragma unroll
        for (int jj = 0; jj < NV; ++jj) {
            typename TR::Raw raw = TR::template load<false>(vrow, sub, jj);
            TR::widen(raw, &vf[jj * EPV]);
        }
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] = fmaf(w, vf[i], acc[i]);
    }
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        acc[i] += __shfl_xor(acc[i], 16, 64);
        acc[i] += __shfl_xor(acc[i], 32, 64);
    }
    if (grp == 0) {
#pragma unroll
        for (int jj = 0; jj < NV; ++jj)
#pragma unroll
            for (int i = 0; i < EPV; ++i) s_acc[wave][TR::vec_offset(sub, jj) + i] = acc[jj * EPV + i];
    }
    __syncthreads();
    if (tid < D) {
        float ot = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) ot += s_acc[w][tid];
        a.o[gh * D + tid] = ot;
    }
    if (tid == 0) {
        a.m[gh] = mx;
        a.l[gh] = lt;
    }
}

// ---- table upload (host tables reach the device through kernel arguments only) ----------------

__global__ void hg_upload_ranges_kernel(RangeEntry *dst, int count, const RangeChunk chunk)
{
    const int i = threadIdx.x;
    if (i < count) dst[i] = chunk.e[i];
}

__global__ void hg_upload_ints_kernel(int32_t *dst, int count, const IntChunk chunk)
{
    const int i = threadIdx.x;
    if (i < count) dst[i] = chunk.e[i];
}

// Plain copy of known traffic (n bytes read, n bytes written): the yardstick that profiler byte
// counters are scaled by.
__global__ __launch_bounds__(256) void hg_calibration_copy_kernel(hg_u32x4 *dst, const hg_u32x4 *src, size_t n_vec)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

}  // namespace hg
