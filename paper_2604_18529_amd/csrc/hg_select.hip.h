// Post-QK^T selection kernels: hg_select_kernel (from logits rows, staged for long groups),
// hg_select_survivors_kernel (from the lists a filter pass leaves), hg_survivor_compact_kernel.
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
// Fast path (FAST variants: workgroups of 8 waves, at most 32 x 512 elements each, top_k <= 1024)
// replacing steps 1-2.  The radix passes above pay for LDS atomics that nearly all land in the few
// bins of the common exponents, and read the row five times.  Here the elements are read once into
// registers (element e of thread t is column e*512 + t) and a cheap lower bound discards nearly
// all of them:
//   a. every thread takes 8 maxima, each over 4 of its elements.  With j = ceil(keep / 8), each
//      wave finds by bisection on the key bits (ballots only) the largest Tw that j of its 512
//      maxima reach; the smallest Tw of the 8 waves is reached by 8*j >= keep maxima, i.e. by at
//      least `keep` distinct elements, so it is a lower bound of the keep-th largest element;
//   b. the keys of the elements at or above the bound (about keep..2*keep for unordered data) go
//      to LDS, in any order;
//   c. radix select among those few keys, and only over the digits below the common prefix of
//      the bound and the largest key: T and the number of ties to keep;
//   d. the ordered compaction works on wave ballots straight from the registers: one count per
//      (e, wave), one block scan over those 256 counts, and a kept element's slot follows from the
//      counts before its wave row plus the kept lanes below it.
// Inputs that defeat the bound (sorted rows, masked rows full of -inf, too many candidates) fall
// back to the radix passes over the row; the result is the same either way.
// In every path the kept elements' columns are looked up only after the selection, all at once,
// and the fold keeps four V rows per lane group in flight: both are memory latencies that would
// otherwise line up one behind the other.

constexpr int kSelectFastBlock = 512;                             // threads of the FAST variants (8 waves)
constexpr int kSelectRegs = 32;                                   // elements per thread of the fast path
constexpr int kSelectRegTokens = kSelectRegs * kSelectFastBlock;  // 16384
constexpr int kSelectSubMax = 8;                                  // maxima per thread that feed the lower bound
constexpr int kSelectFastKeep = 1024;                             // largest top_k of the fast path
constexpr int kSelectCandCap = 4096;                              // most candidates the fast path takes

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

// Exclusive scan of v over the 64 lanes of a wave (no LDS, no barrier).
__device__ __forceinline__ uint32_t wave_exclusive_scan(uint32_t v)
{
    const int lane = threadIdx.x & 63;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(inc, d, 64);
        if (lane >= d) inc += t;
    }
    return inc - v;
}

// Fast path of steps 1-2 (see the top of the file) with R elements per thread: a row of
// n <= R * kSelectFastBlock elements, keep <= kSelectFastKeep.  On success the kept elements'
// places in the row (ascending) and their logits are in s_cols / s_vals and the function returns
// true; otherwise nothing has been decided and the caller runs the radix passes over the row.
// The return value is uniform; every thread of the workgroup must call it.
struct SelectFastLds {
    uint32_t cand[kSelectCandCap];                           // keys of the elements at or above the bound
    uint32_t cnt[kSelectRegs * (kSelectFastBlock / 64)];     // kept elements per (e, wave), then their scan
    uint32_t hist[2][256];                                   // alternating between radix passes
    uint32_t wave[kSelectFastBlock / 64];
    uint32_t bcast[2];
    uint32_t count;
};

// The row a selection reads from: val(i) is element i.
// gather(x, n) loads the elements of the fast path's thread: x[e] = element e * BLOCK + tid, the
// row's last element in the slots past its end.
struct RowDirect {
    const float *row;
    __device__ __forceinline__ float operator()(int i) const { return row[i]; }
    template <int R, int BLOCK>
    __device__ __forceinline__ void gather(float (&x)[R], int n) const
    {
#pragma unroll
        for (int e = 0; e < R; ++e) {
            const int i = e * BLOCK + (int)threadIdx.x;
            x[e] = row[i < n ? i : n - 1];
        }
    }
};

template <int R, typename ROW>
__device__ __forceinline__ bool select_fast_r(const ROW &val, int n, int keep, SelectFastLds &f, int32_t *s_cols, float *s_vals)
{
    constexpr int BLOCK = kSelectFastBlock, NW = BLOCK / 64, G = kSelectSubMax;
    static_assert(R <= kSelectRegs && R % G == 0 && (R * NW) % 64 == 0, "elements per thread");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float x[R];
    val.template gather<R, BLOCK>(x, n);
    if (tid == 0) f.count = 0u;
    if (tid < 256) f.hist[0][tid] = 0u;
    if (tid < R * NW) f.cnt[tid] = 0u;  // most (e, wave) rows will hold nothing at or above T
    // Slots past the end must not count as elements: they become -inf, which no bound admits (a
    // bound at or below -inf sends the workgroup to the radix passes over the row).
    // G maxima per thread, each over the R / G elements e = g, g + G, ...
    float tm[G];
#pragma unroll
    for (int g = 0; g < G; ++g) tm[g] = -INFINITY;
#pragma unroll
    for (int e = 0; e < R; ++e) {
        if (e * BLOCK + tid >= n) x[e] = -INFINITY;
        tm[e % G] = fmaxf(tm[e % G], x[e]);
    }
    // a. bound: per wave, the largest Tw (upper 20 key bits) that `need` of its 64 * G maxima reach
    uint32_t tk[G], top = 0u;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        tk[g] = order_key(tm[g]);
        top = tk[g] > top ? tk[g] : top;
    }
    // (small keep: fewer, coarser maxima do -- 512 * g_use >= 4 * keep keeps the bound within the
    // upper quarter of the maxima -- and the bisection below costs g_use ballots per step)
    const int g_use = keep <= 128 ? 1 : keep <= 256 ? 2 : keep <= 512 ? 4 : 8;
    static_assert(G == 8, "the folding below is written for 8 maxima per thread");
    if (g_use <= 4) {
#pragma unroll
        for (int g = 0; g < 4; ++g) tk[g] = tk[g] > tk[g + 4] ? tk[g] : tk[g + 4];
    }
    if (g_use <= 2) {
#pragma unroll
        for (int g = 0; g < 2; ++g) tk[g] = tk[g] > tk[g + 2] ? tk[g] : tk[g + 2];
    }
    if (g_use <= 1) tk[0] = tk[0] > tk[1] ? tk[0] : tk[1];
    const int need = (keep + NW - 1) / NW;
    uint32_t tw = 0u;
    for (int b = 31; b >= 12; --b) {
        const uint32_t c = tw | (1u << b);
        int reach = 0;
#pragma unroll
        for (int g = 0; g < G; ++g)
            if (g < g_use) reach += __builtin_popcountll(__builtin_amdgcn_ballot_w64(tk[g] >= c));
        if (reach >= need) tw = c;
    }
    // the largest key of the workgroup bounds the digits the radix passes have to look at
#pragma unroll
    for (int step = 32; step >= 1; step >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)top, step, 64);
        top = o > top ? o : top;
    }
    if (lane == 0) {
        f.wave[wave] = tw;
        f.hist[1][wave] = top;  // (the second histogram is free until the second pass)
    }
    __syncthreads();
    uint32_t lower = f.wave[0], hi = f.hist[1][0];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        lower = f.wave[w] < lower ? f.wave[w] : lower;
        hi = f.hist[1][w] > hi ? f.hist[1][w] : hi;
    }
    if (lower <= order_key(-INFINITY)) return false;  // masked or nearly empty rows: no useful bound
    const float lower_f = key_to_float(lower);

    // b. keys of the candidates -> LDS, any order: count, one counter bump per wave, write
    uint32_t mine = 0;
#pragma unroll
    for (int e = 0; e < R; ++e) mine += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(x[e] >= lower_f));
    uint32_t at = 0;
    if (lane == 0 && mine) at = atomicAdd(&f.count, mine);
    at = __builtin_amdgcn_readfirstlane(at);
    const uint64_t below = ((uint64_t)1 << lane) - 1;
    if (mine) {
#pragma unroll
        for (int e = 0; e < R; ++e) {
            const bool c = x[e] >= lower_f;
            const uint64_t bc = __builtin_amdgcn_ballot_w64(c);
            if (bc) {
                const uint32_t pos = at + (uint32_t)__builtin_popcountll(bc & below);
                if (c && pos < (uint32_t)kSelectCandCap) f.cand[pos] = order_key(x[e]);
                at += (uint32_t)__builtin_popcountll(bc);
            }
        }
    }
    __syncthreads();  // (also: every thread has read f.hist[1][0..NW) before a pass clears it)
    // At least `keep` candidates exist: the maxima that reach the bound are distinct elements.
    const int nc = (int)f.count;
    if (nc > kSelectCandCap || nc < keep) return false;  // (nc < keep: only with NaN logits)

    // c. radix select among the candidates: T = key of the keep-th largest, k_eq = how many keys
    //    equal to T are kept.  Every candidate lies in [lower, hi]: the bits above the highest bit
    //    in which those two differ are common to all and need no pass.
    uint32_t T = hi, k_eq = (uint32_t)keep;
    if (hi != lower) {
        const int top_bit = 31 - __builtin_clz(hi ^ lower);
        int shift = top_bit & ~7;
        uint32_t mask = shift == 24 ? 0u : ~0u << (shift + 8);
        uint32_t prefix = hi & mask, krem = (uint32_t)keep;
        // One pass = two barriers: all add to the current histogram | wave 0 scans its 256 bins from
        // the top (4 per lane) and publishes the digit while the other waves clear the histogram
        // of the next pass | all read the digit.
        for (int cur = 0; shift >= 0; shift -= 8, cur ^= 1) {
            for (int c = tid; c < nc; c += BLOCK) {
                const uint32_t u = f.cand[c];
                if ((u & mask) == prefix) atomicAdd(&f.hist[cur][(u >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (wave == 0) {
                uint32_t c4[4], mine4 = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    c4[j] = f.hist[cur][255 - (4 * lane + j)];
                    mine4 += c4[j];
                }
                uint32_t above = wave_exclusive_scan(mine4);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (above < krem && above + c4[j] >= krem) {
                        f.bcast[0] = prefix | ((uint32_t)(255 - (4 * lane + j)) << shift);
                        f.bcast[1] = krem - above;
                    }
                    above += c4[j];
                }
            } else if (tid - 64 < 256) {
                f.hist[cur ^ 1][tid - 64] = 0u;
            }
            __syncthreads();
            prefix = f.bcast[0];
            krem = f.bcast[1];
            mask |= 0xffu << shift;
        }
        T = prefix;
        k_eq = krem;
    }

    // d. ordered compaction from the registers: kept elements per (e, wave), one scan over those
    //    counts, then a kept element's slot = kept before its wave row + kept lanes below it.
    //    Keep every x > T and the first k_eq (in column order) x == T.
    const float T_f = key_to_float(T);
#pragma unroll
    for (int e = 0; e < R; ++e) {
        if (__builtin_amdgcn_ballot_w64(x[e] >= T_f)) {
            const uint64_t bg = __builtin_amdgcn_ballot_w64(x[e] > T_f);
            const uint64_t be = __builtin_amdgcn_ballot_w64(x[e] == T_f);
            if (lane == 0) f.cnt[e * NW + wave] = (uint32_t)__builtin_popcountll(bg) | ((uint32_t)__builtin_popcountll(be) << 16);
        }
    }
    __syncthreads();
    if (wave == 0) {  // exclusive scan of the R * NW counts, PER per lane
        constexpr int PER = R * NW / 64;
        uint32_t c4[PER], mine4 = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            c4[j] = f.cnt[PER * lane + j];
            mine4 += c4[j];
        }
        uint32_t before = wave_exclusive_scan(mine4);
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            f.cnt[PER * lane + j] = before;
            before += c4[j];
        }
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < R; ++e) {
        if (__builtin_amdgcn_ballot_w64(x[e] >= T_f)) {
            const bool gt = x[e] > T_f, eq = x[e] == T_f;
            const uint64_t bg = __builtin_amdgcn_ballot_w64(gt);
            const uint64_t be = __builtin_amdgcn_ballot_w64(eq);
            const uint32_t base = f.cnt[e * NW + wave];
            const uint32_t gt_before = (base & 0xffffu) + (uint32_t)__builtin_popcountll(bg & below);
            const uint32_t eq_before = (base >> 16) + (uint32_t)__builtin_popcountll(be & below);
            if (gt || (eq && eq_before < k_eq)) {
                const uint32_t pos = gt_before + (eq_before < k_eq ? eq_before : k_eq);
                s_cols[pos] = e * BLOCK + tid;
                s_vals[pos] = x[e];
            }
        }
    }
    __syncthreads();
    return true;
}

template <typename ROW>
__device__ __forceinline__ bool select_fast(const ROW &val, int n, int keep, SelectFastLds &f, int32_t *s_cols, float *s_vals)
{
    return select_fast_r<kSelectRegs>(val, n, keep, f, s_cols, s_vals);
}

// The same with half the elements per thread for rows of at most half the capacity -- what a
// filter pass usually leaves of a million tokens: every step is a loop over a thread's elements.
template <typename ROW>
__device__ __forceinline__ bool select_fast_by_length(const ROW &val, int n, int keep, SelectFastLds &f, int32_t *s_cols, float *s_vals)
{
    if (n <= kSelectRegTokens / 2) return select_fast_r<kSelectRegs / 2>(val, n, keep, f, s_cols, s_vals);
    return select_fast_r<kSelectRegs>(val, n, keep, f, s_cols, s_vals);
}

// Steps 1-2 by radix passes over the row (any n, any keep <= kMaxTopK): the kept elements' places
// in the row (ascending) and their logits go to s_cols / s_vals.  Every thread of the workgroup
// must call it.
struct SelectRadixLds {
    uint32_t hist[256];
    uint32_t wave[kSelectBlock / 64];
    uint32_t prefix, krem;
};

template <int BLOCK, typename ROW>
__device__ __forceinline__ void select_radix(const ROW &val, int n, int keep, SelectRadixLds &rl, int32_t *s_cols, float *s_vals)
{
    const int tid = threadIdx.x;
    // 1. radix select
    uint32_t prefix = 0, mask = 0, krem = (uint32_t)keep;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) rl.hist[tid] = 0;
        __syncthreads();
        for (int i0 = 0; i0 < n; i0 += 8 * BLOCK) {  // eight loads in flight per thread
            float x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = i0 + j * BLOCK + tid;
                x[j] = val(i < n ? i : n - 1);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t u = order_key(x[j]);
                if (i0 + j * BLOCK + tid < n && (u & mask) == prefix) atomicAdd(&rl.hist[(u >> shift) & 255u], 1u);
            }
        }
        __syncthreads();
        // the digit d with  #(digits > d) < krem <= #(digits >= d):  scan the bins from the top
        {
            const uint32_t cnt = tid < 256 ? rl.hist[255 - tid] : 0u;
            uint32_t total;
            const uint32_t above = block_exclusive_scan<BLOCK>(cnt, rl.wave, total);
            if (tid < 256 && above < krem && above + cnt >= krem) {
                rl.prefix = prefix | ((uint32_t)(255 - tid) << shift);
                rl.krem = krem - above;
            }
        }
        __syncthreads();
        prefix = rl.prefix;
        krem = rl.krem;
        mask |= 0xffu << shift;
    }
    const uint32_t T = prefix, k_eq = krem;  // keep every key > T and the first k_eq keys == T

    // 2. ordered compaction of the kept elements; every thread owns kRun consecutive elements of a
    //    chunk, so one block scan serves kRun * BLOCK elements
    constexpr int kRun = 8;
    uint32_t run_gt = 0, run_eq = 0;
    for (int base = 0; base < n; base += kRun * BLOCK) {
        const int i0 = base + kRun * tid;
        float x[kRun];
        uint32_t cnt = 0;  // low half: keys > T, high half: keys == T
#pragma unroll
        for (int j = 0; j < kRun; ++j) {
            x[j] = val(i0 + j < n ? i0 + j : n - 1);
            const uint32_t u = order_key(x[j]);
            if (i0 + j < n) cnt += (u > T ? 1u : 0u) + (u == T ? 0x10000u : 0u);
        }
        uint32_t total;
        const uint32_t scan = block_exclusive_scan<BLOCK>(cnt, rl.wave, total);
        uint32_t gt_before = run_gt + (scan & 0xffffu), eq_before = run_eq + (scan >> 16);
#pragma unroll
        for (int j = 0; j < kRun; ++j) {
            const uint32_t u = order_key(x[j]);
            const bool in = i0 + j < n, gt = in && u > T, eq = in && u == T;
            if (gt || (eq && eq_before < k_eq)) {
                const uint32_t pos = gt_before + (eq_before < k_eq ? eq_before : k_eq);
                s_cols[pos] = i0 + j;
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

// Step 3: the kept logits s_vals[0..keep) with their logits columns s_cols[0..keep) (keep >= 1,
// ascending columns, every thread having written the entries j = tid, tid + BLOCK, ... itself or
// a barrier having passed since) are folded with their V rows into the triple of (group, head)
// pair gh; the kept tokens go to a.sel.  s_red: BLOCK / 64 floats, s_acc: BLOCK / 64 rows of D.
template <typename TR, int BLOCK>
__device__ __forceinline__ void fold_kept(const SelectArgs &a, int64_t gh, int h, int r0, int r1, int keep, int32_t *s_cols,
                                          float *s_vals, float *s_red, float (*s_acc)[TR::D])
{
    constexpr int D = TR::D, EPL = TR::EPL, NV = TR::NV, EPV = TR::EPV, ES = TR::ES, NW = BLOCK / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    //     RPW * wave + grp, + RPW * NW, ...
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
    // (four rows per lane group in flight: the rows are scattered over the cache, every load is a
    // full memory latency, and with top_k = 128 the 8 waves need four rounds)
    constexpr int kRowsAhead = 4;
    for (int j0 = RPW * wave + grp; j0 < keep; j0 += kRowsAhead * RPW * NW) {
        typename TR::Raw raw[kRowsAhead][NV];
        float w[kRowsAhead];
#pragma unroll
        for (int u = 0; u < kRowsAhead; ++u) {
            const int j = j0 + u * RPW * NW;
            const bool ok = j < keep;
            w[u] = ok ? s_vals[j] : -1.f;  // (an entry past the end re-reads the first row and is not added; real weights are >= 0)
            const int tok = s_cols[ok ? j : j0];
            const char *vrow = paged ? vbase + paged_row_offset(table[tok >> a.pages.shift], tok, a.pages.mask, (uint32_t)(a.stride_b * ES), (uint32_t)row_bytes)
                                     : vbase + (int64_t)tok * row_bytes;
#pragma unroll
            for (int jj = 0; jj < NV; ++jj) raw[u][jj] = TR::template load<false>(vrow, sub, jj);
        }
#pragma unroll
        for (int u = 0; u < kRowsAhead; ++u) {
            float vf[EPL];
#pragma unroll
            for (int jj = 0; jj < NV; ++jj) TR::widen(raw[u][jj], &vf[jj * EPV]);
            if (w[u] >= 0.f) {
#pragma unroll
                for (int i = 0; i < EPL; ++i) acc[i] = fmaf(w[u], vf[i], acc[i]);
            }
        }
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

// The triple of a (group, head) pair with nothing to select from, and its list of kept tokens.
template <int D, int BLOCK>
__device__ __forceinline__ void write_empty_selection(const SelectArgs &a, int64_t gh)
{
    const int tid = threadIdx.x;
    if (a.sel)
        for (int j = tid; j < a.top_k; j += BLOCK) a.sel[gh * a.top_k + j] = -1;
    if (tid < D) a.o[gh * D + tid] = 0.f;
    if (tid == 0) {
        a.m[gh] = -INFINITY;
        a.l[gh] = 0.f;
    }
}

// A pad of a candidate slot is the NaN with every bit set: its key is 0, below -inf, and it fails
// every float comparison, so no stage ever prefers it to a real logit, masked (-inf) ones included.
__device__ __forceinline__ float candidate_pad() { return __uint_as_float(0xffffffffu); }

template <typename TR, int STAGE, bool FAST>
__global__ __launch_bounds__(FAST ? kSelectFastBlock : kSelectBlock) void hg_select_kernel(const SelectArgs a)
{
    constexpr int D = TR::D;
    constexpr int BLOCK = FAST ? kSelectFastBlock : kSelectBlock;
    constexpr int KEEP_CAP = FAST ? kSelectFastKeep : kMaxTopK;  // the host picks FAST variants for top_k <= kSelectFastKeep only
    constexpr int NW = BLOCK / 64;
    __shared__ SelectRadixLds s_radix;
    __shared__ int32_t s_cols[KEEP_CAP];   // kept elements' places in the row, then their columns, then their token positions
    __shared__ float s_vals[KEEP_CAP];     // kept logits, later their weights
    __shared__ float s_red[NW];
    __shared__ float s_acc[NW][D];
    __shared__ __align__(16) unsigned char s_fast_raw[FAST ? sizeof(SelectFastLds) : 16];

    const int tid = threadIdx.x, h = blockIdx.y;
    constexpr bool kEmits = STAGE == kSelectCandidates || STAGE == kSelectMidCands;  // writes candidates, no triple
    const int n_parts = STAGE == kSelectCandidates ? a.parts : STAGE == kSelectMidCands ? a.parts2 : 1;
    const int gi = blockIdx.x / n_parts;
    const int part = blockIdx.x - gi * n_parts;
    const int r0 = group_entry(a.groups, gi), r1 = group_entry(a.groups, gi + 1);
    const int c0 = table_entry(a.tab, r0).pre, c1 = table_entry(a.tab, r1).pre;
    const int64_t gh = (int64_t)gi * a.n_q_heads + h;

    // the values this workgroup selects from: row[0..n), element i being logits column
    // col_map ? col_map[i] : col_base + i
    const float *row;
    const int32_t *col_map = nullptr;
    int n, col_base = 0, keep;
    if constexpr (STAGE == kSelectDirect || STAGE == kSelectCandidates) {
        // the group's logits row -- or, after a filter pass, the dense list of its survivors (a
        // superset of the group's top_k, in ascending column order)
        const bool dense = a.dense_cnt != nullptr;
        const int total = dense ? a.dense_cnt[gh] : c1 - c0;
        if (dense && a.direct_limit > 0 && (STAGE == kSelectDirect) != (total <= a.direct_limit)) return;  // the other launch's
        const int n_cut = STAGE == kSelectCandidates ? a.parts : 1;
        // (dense lists are usually far shorter than the rows the parts were sized for: fill the
        // parts of a fast-path launch to their capacity, the others find nothing and leave)
        const int even = (total + n_cut - 1) / n_cut;
        const int per = dense && FAST && even < kSelectRegTokens ? kSelectRegTokens : even;
        const int b = (int64_t)part * per < total ? part * per : total;
        const int e = b + per < total ? b + per : total;
        row = (dense ? a.dense_val : a.logits) + (int64_t)h * a.ltok + c0 + b;
        if (dense) col_map = a.dense_col + (int64_t)h * a.ltok + c0 + b;
        n = e - b;
        col_base = c0 + b;
        keep = n < a.top_k ? n : a.top_k;
    } else if constexpr (STAGE == kSelectMidCands) {
        if (a.dense_cnt && a.direct_limit > 0 && a.dense_cnt[gh] <= a.direct_limit) return;
        // chunk `part` of the group's parts * top_k candidates (pad entries included: they sort
        // below everything and are never kept ahead of a real entry)
        const int total = c1 > c0 ? a.parts * a.top_k : 0;
        const int per = (total + a.parts2 - 1) / a.parts2;
        const int b = part * per < total ? part * per : total;
        const int e = b + per < total ? b + per : total;
        const int64_t base = gh * a.parts * (int64_t)a.top_k + b;
        row = a.cand_val + base;
        col_map = a.cand_col + base;
        n = e - b;
        keep = n < a.top_k ? n : a.top_k;
    } else {
        if (a.dense_cnt && a.direct_limit > 0 && a.dense_cnt[gh] <= a.direct_limit) return;
        const bool mid = a.parts2 > 0;
        const int np = mid ? a.parts2 : a.parts;
        const int64_t base = gh * np * (int64_t)a.top_k;
        row = (mid ? a.cand2_val : a.cand_val) + base;
        col_map = (mid ? a.cand2_col : a.cand_col) + base;
        n = c1 > c0 ? np * a.top_k : 0;  // padded with entries that sort below every logit
        keep = c1 - c0 < a.top_k ? c1 - c0 : a.top_k;
    }

    // where a candidates stage writes
    float *const out_val = STAGE == kSelectMidCands ? a.cand2_val : a.cand_val;
    int32_t *const out_col = STAGE == kSelectMidCands ? a.cand2_col : a.cand_col;
    if constexpr (kEmits) {
        // pad the part's candidate slots; the kept ones are overwritten below
        const int64_t base = (gh * n_parts + part) * (int64_t)a.top_k;
        for (int j = tid + keep; j < a.top_k; j += BLOCK) {
            out_val[base + j] = candidate_pad();
            out_col[base + j] = 0;
        }
        if (n == 0) return;
    } else {
        if (n == 0) {
            write_empty_selection<D, BLOCK>(a, gh);
            return;
        }
        if (a.sel)
            for (int j = tid + keep; j < a.top_k; j += BLOCK) a.sel[gh * a.top_k + j] = -1;
    }

    // the host launches a FAST variant only when every workgroup has n <= kSelectRegTokens
    const RowDirect val{row};
    bool decided = false;
    if constexpr (FAST) {
        if (keep <= kSelectFastKeep) decided = select_fast(val, n, keep, *reinterpret_cast<SelectFastLds *>(s_fast_raw), s_cols, s_vals);
    }
    if (!decided) select_radix<BLOCK>(val, n, keep, s_radix, s_cols, s_vals);
    // Place in the row -> logits column, for the kept elements only and all at once (a look-up
    // where an element is found to be kept would cost one memory latency per step of that loop,
    // one after the other).  Every thread rewrites the entries it reads again below.
    for (int j = tid; j < keep; j += BLOCK) {
        const int i = s_cols[j];
        s_cols[j] = col_map ? col_map[i] : col_base + i;
    }

    if constexpr (kEmits) {
        const int64_t base = (gh * n_parts + part) * (int64_t)a.top_k;
        for (int j = tid; j < keep; j += BLOCK) {
            out_val[base + j] = s_vals[j];
            out_col[base + j] = s_cols[j];
        }
        return;
    }
    fold_kept<TR, BLOCK>(a, gh, h, r0, r1, keep, s_cols, s_vals, s_red, s_acc);
}

// ---- hg_select_survivors_kernel -------------------------------------------------------------------
//
// Selection straight from the lists a filter pass leaves (hg_attn_topk): per (group, head) the
// survivors sit in one short list per (segment, sub-span) -- an *item* -- at the sub-span's own
// columns.  In column order the items form one virtual row; an exclusive scan of their counts
// (kept in LDS: at most kSurvivorItems items, which the host checks) gives every item's place in
// it, and element i of the row is found by bisection over those places.  A row of at most
// kSelectRegTokens elements -- the rule: a filter pass lets a fraction of a per cent through -- is
// selected and folded by one workgroup.  A longer row is cut into slices of that size, dealt to the
// tail_parts workgroups of the pair; each writes its slices' top_k candidates, and the workgroup
// that finishes last (a counter in global memory that the filter pass has cleared; no workgroup
// waits for another) selects among the candidates of all and folds.  The host launches as many
// workgroups per pair as fill the device once: idle ones cost nothing then, and a row that the
// bounds failed on (ascending logits) still has the whole device working on it.
constexpr int kSurvivorItems = 2048;

typedef __attribute__((address_space(3))) const int32_t *LdsConstI32;

struct RowSurvivors {
    const float *vals;      // the head's row of surv_val
    LdsConstI32 isrc, idst; // per item: first column of its list, place in the virtual row
    int n_items, lo;        // element i of the slice is element lo + i of the virtual row
    // Where element i sits in the head's rows of surv_val / surv_col: the last item x with
    // idst[x] <= lo + i (empty items share their successor's place).  A fixed number of steps
    // without branches, so that the searches for a thread's elements run side by side.
    __device__ __forceinline__ int place(int i) const
    {
        const int pos = lo + i;
        int x = 0;
#pragma unroll
        for (int step = kSurvivorItems / 2; step >= 1; step >>= 1) {
            const int y = x + step;
            x = idst[y < n_items ? y : n_items] <= pos ? y : x;  // (idst[n_items], the total, is above every element)
        }
        return isrc[x] + (pos - idst[x]);
    }
    __device__ __forceinline__ float operator()(int i) const { return vals[place(i)]; }
    // The searches of all R elements step by step together: R independent LDS reads per step
    // instead of R chains of dependent ones.
    template <int R, int BLOCK>
    __device__ __forceinline__ void gather(float (&x)[R], int n) const
    {
        int pos[R], at[R];
#pragma unroll
        for (int e = 0; e < R; ++e) {
            const int i = e * BLOCK + (int)threadIdx.x;
            pos[e] = lo + (i < n ? i : n - 1);
            at[e] = 0;
        }
        int top = 1;  // uniform: the largest power of two below n_items
        while (2 * top < n_items) top *= 2;
        for (int step = top; step >= 1; step >>= 1) {
#pragma unroll
            for (int e = 0; e < R; ++e) {
                const int y = at[e] + step;
                at[e] = idst[y < n_items ? y : n_items] <= pos[e] ? y : at[e];
            }
        }
#pragma unroll
        for (int e = 0; e < R; ++e) x[e] = vals[isrc[at[e]] + (pos[e] - idst[at[e]])];
    }
};

// (Compiled for two workgroups per compute unit: several hundred (group, head) pairs then fit the
// device in one and a quarter passes instead of two and a half -- 52 -> 37 us at 640 pairs.)
template <typename TR>
__global__ __launch_bounds__(kSelectFastBlock, 4) void hg_select_survivors_kernel(const SelectArgs a)
{
    constexpr int D = TR::D, BLOCK = kSelectFastBlock, NW = BLOCK / 64;
    __shared__ SelectRadixLds s_radix;
    __shared__ int32_t s_cols[kSelectFastKeep];
    __shared__ float s_vals[kSelectFastKeep];
    __shared__ float s_red[NW];
    __shared__ float s_acc[NW][D];
    __shared__ SelectFastLds s_fast;
    __shared__ int32_t s_isrc[kSurvivorItems], s_idst[kSurvivorItems + 1];
    __shared__ uint32_t s_ticket;

    // Grid (pair, part): the workgroups that take a pair's first slice -- with short rows the only
    // ones with anything to do -- come first in the launch order and next to each other, so they
    // start at once and spread over the whole device.
    const int tid = threadIdx.x, part = blockIdx.y;
    const int gi = blockIdx.x / a.n_q_heads, h = blockIdx.x - gi * a.n_q_heads;
    const int r0 = group_entry(a.groups, gi), r1 = group_entry(a.groups, gi + 1);
    const int64_t gh = blockIdx.x;
    const int hk = h / a.ws.group, gl = h - hk * a.ws.group;
    const int chunk = gl / a.ws.gt, g = gl - chunk * a.ws.gt;
    const int64_t s = (int64_t)hk * a.ws.n_chunks + chunk;  // this head's stream
    const int64_t row = (int64_t)h * a.ws.ltok;

    // the items of the pair in column order: ranges of the group, workgroups of the filter pass
    // that held a segment of the range, sub-spans of the segment
    int n_items = 0;
    uint32_t running = 0;
    for (int r = r0; r < r1; ++r) {
        const int pre = table_entry(a.tab, r).pre, pre_next = table_entry(a.tab, r + 1).pre;
        if (pre_next == pre) continue;
        const int64_t p_first = s * a.ws.ltok + pre, p_last = s * a.ws.ltok + pre_next - 1;
        const int64_t w_first = p_first / a.ws.span, w_last = p_last / a.ws.span;
        const int n_it = (int)(w_last - w_first + 1) * a.n_sub;
        for (int base = 0; base < n_it; base += BLOCK) {
            const int i = base + tid;
            uint32_t c = 0;
            int src = 0;
            if (i < n_it) {
                const int64_t w = w_first + i / a.n_sub;
                const int j = i % a.n_sub;
                // the segment of workgroup w inside range r, in columns of the concatenated ranges
                const int64_t lo = w * a.ws.span - s * a.ws.ltok, hi = lo + a.ws.span;
                const int x0 = lo > pre ? (int)lo : pre, x1 = hi < pre_next ? (int)hi : pre_next;
                const int sub_len = filter_sub_len(x1 - x0, a.n_sub);
                src = x0 + (j * sub_len < x1 - x0 ? j * sub_len : x1 - x0);
                const int64_t slot = w + s * a.tab.n_ranges + r;
                c = (uint32_t)a.surv_cnt[(slot * a.n_sub + j) * a.ws.gt + g];
            }
            uint32_t total;
            const uint32_t before = block_exclusive_scan<BLOCK>(c, s_radix.wave, total);
            if (i < n_it && n_items + i < kSurvivorItems) {
                s_isrc[n_items + i] = src;
                s_idst[n_items + i] = (int32_t)(running + before);
            }
            running += total;
        }
        n_items += n_it;
    }
    if (n_items > kSurvivorItems) n_items = kSurvivorItems;  // (the host launches this kernel only when they fit)
    if (tid == 0) s_idst[n_items] = (int32_t)running;
    __syncthreads();
    // (a.parts slices hold the longest group: the host has checked that)
    const int total = running < (uint32_t)a.parts * kSelectRegTokens ? (int)running : a.parts * kSelectRegTokens;
    if (total == 0) {
        if (part == 0) write_empty_selection<D, BLOCK>(a, gh);
        return;
    }
    const int n_slices = (total + kSelectRegTokens - 1) / kSelectRegTokens;
    if (part >= n_slices) return;

    const bool single = n_slices == 1;

    RowSurvivors val{a.surv_val + row, (LdsConstI32)s_isrc, (LdsConstI32)s_idst, n_items, 0};
    const int64_t cand_base = gh * a.parts * (int64_t)a.top_k;
    int keep;
    for (int slice = part;;) {
        val.lo = slice * kSelectRegTokens;
        const int n = total - val.lo < kSelectRegTokens ? total - val.lo : kSelectRegTokens;
        keep = n < a.top_k ? n : a.top_k;
        if (!select_fast_by_length(val, n, keep, s_fast, s_cols, s_vals)) select_radix<BLOCK>(val, n, keep, s_radix, s_cols, s_vals);
        // place in the slice -> logits column (every thread rewrites the entries it reads again below)
        for (int j = tid; j < keep; j += BLOCK) s_cols[j] = a.surv_col[row + val.place(s_cols[j])];
        if (single) break;
        // this slice's candidates, padded to top_k
        for (int j = tid; j < a.top_k; j += BLOCK) {
            a.cand_val[cand_base + (int64_t)slice * a.top_k + j] = j < keep ? s_vals[j] : candidate_pad();
            a.cand_col[cand_base + (int64_t)slice * a.top_k + j] = j < keep ? s_cols[j] : 0;
        }
        __syncthreads();  // s_cols / s_vals are free again
        slice += a.tail_parts;
        if (slice >= n_slices) break;
    }
    if (!single) {
        // This workgroup's slices are done.  Its candidates become visible to the device, then it
        // takes a ticket; the workgroup that draws the last one sees the candidates of all and
        // selects among them.
        __threadfence();
        __syncthreads();
        if (tid == 0) s_ticket = atomicAdd(a.tail_cnt + gh, 1u);
        __syncthreads();
        const uint32_t active = (uint32_t)(n_slices < a.tail_parts ? n_slices : a.tail_parts);
        if (s_ticket != active - 1) return;
        __threadfence();
        const RowDirect cands{a.cand_val + cand_base};
        const int n = n_slices * a.top_k;
        keep = total < a.top_k ? total : a.top_k;
        if (!select_fast(cands, n, keep, s_fast, s_cols, s_vals)) select_radix<BLOCK>(cands, n, keep, s_radix, s_cols, s_vals);
        for (int j = tid; j < keep; j += BLOCK) s_cols[j] = a.cand_col[cand_base + s_cols[j]];
    }
    if (a.sel)
        for (int j = tid + keep; j < a.top_k; j += BLOCK) a.sel[gh * a.top_k + j] = -1;
    fold_kept<TR, BLOCK>(a, gh, h, r0, r1, keep, s_cols, s_vals, s_red, s_acc);
}

// ---- hg_survivor_compact_kernel ------------------------------------------------------------------
//
// Grid (group, query head, chunk).  The segments of the group's ranges in this head's stream, and
// the sub-spans inside each, are visited in column order; an exclusive scan of their survivor
// counts gives every sub-span's place in the dense list; the copying of the entries is shared by
// the `chunks` workgroups of the (group, head) pair (every one of them repeats the cheap scan).
__global__ __launch_bounds__(256) void hg_survivor_compact_kernel(const CompactArgs a)
{
    __shared__ uint32_t s_wave[4];
    __shared__ int32_t s_src[256], s_dst[256], s_cnt[256];
    const int tid = threadIdx.x;
    const int gi = blockIdx.x, h = blockIdx.y, z = blockIdx.z;
    const int r0 = group_entry(a.groups, gi), r1 = group_entry(a.groups, gi + 1);
    const int c0 = table_entry(a.tab, r0).pre;
    const int hk = h / a.ws.group, gl = h - hk * a.ws.group;
    const int chunk = gl / a.ws.gt, g = gl - chunk * a.ws.gt;
    const int64_t s = (int64_t)hk * a.ws.n_chunks + chunk;  // this head's stream
    const int64_t row = (int64_t)h * a.ws.ltok;
    uint32_t running = 0;  // survivors of the group before the current batch of sub-spans
    for (int r = r0; r < r1; ++r) {
        const int pre = table_entry(a.tab, r).pre, pre_next = table_entry(a.tab, r + 1).pre;
        if (pre_next == pre) continue;
        const int64_t p_first = s * a.ws.ltok + pre, p_last = s * a.ws.ltok + pre_next - 1;
        const int64_t w_first = p_first / a.ws.span, w_last = p_last / a.ws.span;
        const int64_t n_items = (w_last - w_first + 1) * a.n_sub;
        for (int64_t base = 0; base < n_items; base += 256) {
            const int64_t i = base + tid;
            uint32_t c = 0;
            int src = 0;
            if (i < n_items) {
                const int64_t w = w_first + i / a.n_sub;
                const int j = (int)(i % a.n_sub);
                // the segment of workgroup w inside range r, in columns of the concatenated ranges
                const int64_t lo = w * a.ws.span - s * a.ws.ltok, hi = lo + a.ws.span;
                const int x0 = lo > pre ? (int)lo : pre, x1 = hi < pre_next ? (int)hi : pre_next;
                const int sub_len = filter_sub_len(x1 - x0, a.n_sub);
                src = x0 + (j * sub_len < x1 - x0 ? j * sub_len : x1 - x0);
                const int64_t slot = w + s * a.tab.n_ranges + r;
                c = (uint32_t)a.surv_cnt[(slot * a.n_sub + j) * a.ws.gt + g];
            }
            uint32_t total;
            const uint32_t before = block_exclusive_scan<256>(c, s_wave, total);
            s_src[tid] = src;
            s_dst[tid] = (int32_t)(running + before);
            s_cnt[tid] = (int32_t)c;
            __syncthreads();
            // this workgroup copies the sub-spans z, z + chunks, ... of the batch, eight at a time
            // (32 threads each: a sub-span usually holds a few dozen survivors)
            const int n_here = n_items - base < 256 ? (int)(n_items - base) : 256;
            for (int it = z + (tid >> 5) * a.chunks; it < n_here; it += 8 * a.chunks) {
                const int cnt = s_cnt[it];
                const float *sv = a.surv_val + row + s_src[it];
                const int32_t *sc = a.surv_col + row + s_src[it];
                float *dv = a.dense_val + row + c0 + s_dst[it];
                int32_t *dc = a.dense_col + row + c0 + s_dst[it];
                for (int x = tid & 31; x < cnt; x += 32) {
                    dv[x] = sv[x];
                    dc[x] = sc[x];
                }
            }
            __syncthreads();
            running += total;
        }
    }
    if (z == 0 && tid == 0) a.dense_cnt[(int64_t)gi * a.ws.n_q_heads + h] = (int32_t)running;
}

}  // namespace hg
