// Post-QK^T selection kernel.
#pragma once

#include "hg_common.hip.h"
#include "hg_combine.hip.h"

namespace hg {

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
//
// Fast path (FAST variants: workgroups of 8 waves, at most 32 x 512 elements each, top_k <= 256)
// replacing steps 1-2.
// The radix passes above pay for LDS atomics that nearly all land in the few bins of the common
// exponents, and read the row five times.  Here the elements are read once into registers
// (element e of thread t is column e*512 + t) and a cheap lower bound discards nearly all of them:
//   a. every thread takes the maximum of its elements.  With j = ceil(keep / 8), each wave finds
//      by bisection on the key bits (ballots only) the largest Tw that j of its 64 maxima reach;
//      the smallest Tw of the 8 waves is reached by 8*j >= keep maxima, i.e. by at least `keep`
//      distinct elements, so it is a lower bound of the keep-th largest element;
//   b. the elements at or above the bound (a few hundred for unordered data) are written to LDS as
//      64-bit words (key, ~index), whose order is "larger logit first, lower column first";
//   c. the rank of a candidate is the number of candidates above it, counted by comparison, the
//      list being split over as many threads per candidate as the workgroup has; ranks below
//      `keep` are the kept set, which a second count puts in ascending column order.
// Inputs that defeat the bound (sorted rows, masked rows full of -inf, too many candidates) fall
// back to the radix passes; the result is the same either way.

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

constexpr int kSelectFastBlock = 512;                             // threads of the FAST variants (8 waves)
constexpr int kSelectRegs = 32;                                   // elements per thread of the fast path
constexpr int kSelectRegTokens = kSelectRegs * kSelectFastBlock;  // 16384
constexpr int kSelectFastKeep = 256;                              // largest top_k of the fast path
constexpr int kSelectCandCap = 1024;                              // most candidates the fast path ranks

// Exclusive scan of v over the BLOCK threads of the workgroup; total receives the sum.
template <int BLOCK>
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
    for (int w = 0; w < BLOCK / 64; ++w) {
        const uint32_t t = s_wave[w];
        before += w < wave ? t : 0u;
        all += t;
    }
    __syncthreads();  // s_wave is reused by the next call
    total = all;
    return before + inc - v;
}

// Fast path of steps 1-2 (see the top of the file).  row[0..n) with n <= kSelectRegTokens and
// keep <= kSelectFastKeep.  On success the kept columns (ascending) and logits are in s_cols /
// s_vals and the function returns true; otherwise nothing has been decided and the caller runs
// the radix passes.  The return value is uniform; every thread of the workgroup must call it.
struct SelectFastLds {
    unsigned long long cand[kSelectCandCap + 2];  // (key << 32) | ~index; zero words never outrank anything
    unsigned long long kept[kSelectFastKeep + 2];  // the kept words by rank; read in pairs
    uint32_t rank[kSelectCandCap];
    uint32_t bound[kSelectFastBlock / 64];
    uint32_t count;
};

__device__ __forceinline__ bool select_fast(const float *__restrict__ row, int n, int keep, const int32_t *col_map,
                                            int col_base, SelectFastLds &f, int32_t *s_cols, float *s_vals)
{
    constexpr int NW = kSelectFastBlock / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float x[kSelectRegs];
#pragma unroll
    for (int e = 0; e < kSelectRegs; ++e) {
        const int i = e * kSelectFastBlock + tid;
        x[e] = row[i < n ? i : n - 1];
    }
    // LDS set-up while the loads are in flight
#pragma unroll
    for (int c = tid; c < kSelectCandCap; c += kSelectFastBlock) {
        f.cand[c] = 0ull;
        f.rank[c] = 0u;
    }
    if (tid < 2) f.cand[kSelectCandCap + tid] = 0ull;
    if (tid == 0) f.count = 0u;
    // Slots past the end must not count as elements: they become -inf, which no bound admits (a
    // bound at or below -inf sends the workgroup to the radix passes).  Without this the copies of
    // the last element made by the clamp above would pose as per-thread maxima of their own.
    float tm = -INFINITY;
#pragma unroll
    for (int e = 0; e < kSelectRegs; ++e) {
        if (e * kSelectFastBlock + tid >= n) x[e] = -INFINITY;
        tm = fmaxf(tm, x[e]);
    }
    // a. bound
    const uint32_t tmax = order_key(tm);
    const int need = (keep + NW - 1) / NW;
    uint32_t tw = 0u;
    for (int b = 31; b >= 12; --b) {
        const uint32_t c = tw | (1u << b);
        if (__builtin_popcountll(__builtin_amdgcn_ballot_w64(tmax >= c)) >= need) tw = c;
    }
    if (lane == 0) f.bound[wave] = tw;
    __syncthreads();
    uint32_t lower = f.bound[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) lower = f.bound[w] < lower ? f.bound[w] : lower;
    if (lower <= order_key(-INFINITY)) return false;  // masked or nearly empty rows: no useful bound
    const float lower_f = key_to_float(lower);

    // b. candidates -> LDS, any order: count, one counter bump per wave, write
    uint32_t mine = 0;
#pragma unroll
    for (int e = 0; e < kSelectRegs; ++e) mine += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(x[e] >= lower_f));
    uint32_t at = 0;
    if (lane == 0 && mine) at = atomicAdd(&f.count, mine);
    at = __builtin_amdgcn_readfirstlane(at);
    if (mine) {
        const uint64_t below = ((uint64_t)1 << lane) - 1;
#pragma unroll
        for (int e = 0; e < kSelectRegs; ++e) {
            const bool c = x[e] >= lower_f;
            const uint64_t bc = __builtin_amdgcn_ballot_w64(c);
            if (bc) {
                const uint32_t pos = at + (uint32_t)__builtin_popcountll(bc & below);
                if (c && pos < (uint32_t)kSelectCandCap)
                    f.cand[pos] = ((unsigned long long)order_key(x[e]) << 32) | (uint32_t)~(uint32_t)(e * kSelectFastBlock + tid);
                at += (uint32_t)__builtin_popcountll(bc);
            }
        }
    }
    __syncthreads();
    // At least `keep` candidates exist: the maxima that reach the bound are distinct elements.
    const int nc = (int)f.count;
    if (nc > kSelectCandCap || nc < keep) return false;  // (nc < keep: only with NaN logits)

    // c. ranks.  Few candidates: candidate c = tid % ncr is counted by split tid / ncr over its
    //    share of the list (partial counts meet in f.rank); many: one thread per candidate or two.
    {
        const int ncr = (nc + 63) & ~63;  // whole waves per split: the list reads broadcast
        if (ncr <= kSelectFastBlock) {
            const int splits = kSelectFastBlock / ncr;
            const int len = ((nc + splits - 1) / splits + 1) & ~1;  // even: two words per LDS read
            const int sp = tid / ncr, c = tid - sp * ncr;
            if (sp < splits && c < nc) {
                const unsigned long long me = f.cand[c];
                const int j0 = sp * len, j1 = j0 + len < nc ? j0 + len : nc;  // reads past nc see zero words
                uint32_t r = 0;
                for (int j = j0; j < j1; j += 2) {
                    const unsigned long long a0 = f.cand[j], a1 = f.cand[j + 1];
                    r += (a0 > me ? 1u : 0u) + (a1 > me ? 1u : 0u);
                }
                atomicAdd(&f.rank[c], r);
            }
        } else {
            for (int c = tid; c < nc; c += kSelectFastBlock) {
                const unsigned long long me = f.cand[c];
                uint32_t r = 0;
                for (int j = 0; j < nc; j += 2) {
                    const unsigned long long a0 = f.cand[j], a1 = f.cand[j + 1];
                    r += (a0 > me ? 1u : 0u) + (a1 > me ? 1u : 0u);
                }
                f.rank[c] = r;
            }
        }
    }
    __syncthreads();
    for (int c = tid; c < nc; c += kSelectFastBlock) {
        const uint32_t r = f.rank[c];
        if (r < (uint32_t)keep) f.kept[r] = f.cand[c];
    }
    __syncthreads();
    // kept set in ascending column order: position = number of kept entries with a lower index
    if (tid < keep) {
        const unsigned long long me = f.kept[tid];
        const uint32_t inv = (uint32_t)me;  // ~index: a lower index is a larger value
        uint32_t pos = 0;
        for (int j = 0; j < keep; j += 2) {
            const uint32_t i0 = (uint32_t)f.kept[j], i1 = (uint32_t)f.kept[j + 1];
            pos += (i0 > inv ? 1u : 0u) + ((j + 1 < keep && i1 > inv) ? 1u : 0u);
        }
        const int i = (int)~inv;
        s_cols[pos] = col_map ? col_map[i] : col_base + i;
        s_vals[pos] = key_to_float((uint32_t)(me >> 32));
    }
    __syncthreads();
    return true;
}

template <typename TR, int STAGE, bool FAST>
__global__ __launch_bounds__(FAST ? kSelectFastBlock : kSelectBlock) void hg_select_kernel(const SelectArgs a)
{
    constexpr int D = TR::D, EPL = TR::EPL, NV = TR::NV, EPV = TR::EPV, ES = TR::ES;
    constexpr int BLOCK = FAST ? kSelectFastBlock : kSelectBlock;
    constexpr int KEEP_CAP = FAST ? kSelectFastKeep : kMaxTopK;  // the host picks FAST variants for top_k <= kSelectFastKeep only
    constexpr int NW = BLOCK / 64;
    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_wave[NW];
    __shared__ uint32_t s_prefix, s_krem;
    __shared__ int32_t s_cols[KEEP_CAP];   // kept columns, later their token positions
    __shared__ float s_vals[KEEP_CAP];     // kept logits, later their weights
    __shared__ float s_red[NW];
    __shared__ float s_acc[NW][D];
    __shared__ __align__(16) unsigned char s_fast_raw[FAST ? sizeof(SelectFastLds) : 16];

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
        for (int j = tid + keep; j < a.top_k; j += BLOCK) {
            a.cand_val[base + j] = -INFINITY;
            a.cand_col[base + j] = 0;
        }
        if (n == 0) return;
    } else {
        if (a.sel)
            for (int j = tid + keep; j < a.top_k; j += BLOCK) a.sel[gh * a.top_k + j] = -1;
        if (n == 0) {
            if (tid < D) a.o[gh * D + tid] = 0.f;
            if (tid == 0) {
                a.m[gh] = -INFINITY;
                a.l[gh] = 0.f;
            }
            return;
        }
    }

    // the host launches a FAST variant only when every workgroup has n <= kSelectRegTokens
    bool decided = false;
    if constexpr (FAST) {
        if (keep <= kSelectFastKeep) decided = select_fast(row, n, keep, col_map, col_base, *reinterpret_cast<SelectFastLds *>(s_fast_raw), s_cols, s_vals);
    }
    if (!decided) {
        // 1. radix select
        uint32_t prefix = 0, mask = 0, krem = (uint32_t)keep;
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) s_hist[tid] = 0;
            __syncthreads();
            for (int i0 = 0; i0 < n; i0 += 8 * BLOCK) {  // eight loads in flight per thread
                float x[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int i = i0 + j * BLOCK + tid;
                    x[j] = row[i < n ? i : n - 1];
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t u = order_key(x[j]);
                    if (i0 + j * BLOCK + tid < n && (u & mask) == prefix) atomicAdd(&s_hist[(u >> shift) & 255u], 1u);
                }
            }
            __syncthreads();
            // the digit d with  #(digits > d) < krem <= #(digits >= d):  scan the bins from the top
            {
                const uint32_t cnt = tid < 256 ? s_hist[255 - tid] : 0u;
                uint32_t total;
                const uint32_t above = block_exclusive_scan<BLOCK>(cnt, s_wave, total);
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
        for (int base = 0; base < n; base += kRun * BLOCK) {
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
            const uint32_t scan = block_exclusive_scan<BLOCK>(cnt, s_wave, total);
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
    }

    if constexpr (STAGE == kSelectCandidates) {
        const int64_t base = (gh * a.parts + part) * (int64_t)a.top_k;
        for (int j = tid; j < keep; j += BLOCK) {
            a.cand_val[base + j] = s_vals[j];
            a.cand_col[base + j] = s_cols[j];
        }
        return;
    }

    // 3a. m = max kept logit; weights; l
    float mx = -INFINITY;
    for (int j = tid; j < keep; j += BLOCK) mx = fmaxf(mx, s_vals[j]);
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
    for (int j = tid; j < keep; j += BLOCK) {
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
    constexpr int LPR = TR::LPR, RPW = TR::RPW;
    const int sub = lane % LPR, grp = lane / LPR;
    const int hk = h / a.group;
    // contiguous cache: the (sequence, KV head) slab; paged cache: the head's offset inside a block
    const bool paged = a.pages.table != nullptr;
    const char *vbase = static_cast<const char *>(a.v) + ((paged ? 0 : (int64_t)seq * a.stride_b) + (int64_t)hk * a.stride_h) * ES;
    const int64_t row_bytes = a.stride_t * ES;
    const int32_t *table = paged ? a.pages.table + (int64_t)seq * a.pages.max_blocks : nullptr;
    float acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;
    for (int j = RPW * wave + grp; j < keep; j += RPW * NW) {
        const float w = s_vals[j];
        const int tok = s_cols[j];
        const char *vrow = paged ? vbase + ((int64_t)table[tok >> a.pages.shift] * a.stride_b + (int64_t)(tok & a.pages.mask) * a.stride_t) * ES
                                 : vbase + (int64_t)tok * row_bytes;
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
#pragma unroll
        for (int step = LPR; step <= 32; step <<= 1) acc[i] += __shfl_xor(acc[i], step, 64);
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

}  // namespace hg
