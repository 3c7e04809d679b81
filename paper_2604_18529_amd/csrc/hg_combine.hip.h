// Small combining kernels: segment reduce, exact merge, the concat path's reduce, table uploads
// and the calibration kernels.
#pragma once

#include "hg_common.hip.h"

namespace hg {

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
    auto fold = [&](const float *pm, const float *pl, const float *po, int t0, int t1) __attribute__((always_inline)) {
#pragma unroll 4
        for (int t = t0 + sl; t < t1; t += S) {
            const int64_t th = (int64_t)t * a.n_q_heads + h;
            const float li = pl[th], oi = po[th * D + c];
            const float mi = li != 0.f ? pm[th] * kLog2e : kNegBig;  // identity element: ignored
            const float mn = fmaxf(mx, mi);
            const float wa = fast_exp2(mx - mn), wb = li != 0.f ? fast_exp2(mi - mn) : 0.f;
            lt = lt * wa + li * wb;
            ot = ot * wa + oi * wb;
            mx = mn;
        }
    };
    fold(a.m, a.l, a.o, ts, te);
    if (a.l_b) {
        const int bs = a.tab_b.ext ? a.tab_b.ext[gidx] : a.tab_b.inl[gidx];
        const int be = a.tab_b.ext ? a.tab_b.ext[gidx + 1] : a.tab_b.inl[gidx + 1];
        fold(a.m_b, a.l_b, a.o_b, bs, be);
    }
    if (!combine_slices<D>(mx, lt, ot, c, sl)) return;

    const int64_t gh = (int64_t)gidx * a.n_q_heads + h;
    const bool empty = !(lt > 0.f);
    a.out[gh * D + c] = empty ? 0.f : ot / lt;
    if (c == 0 && a.lse) a.lse[gh] = empty ? -INFINITY : mx * kLn2 + logf(lt);
}

// ---- concat path: one softmax over the concatenated logits of a group --------------------------

__device__ __forceinline__ int group_entry(const GroupTable &g, int i) { return g.ext ? g.ext[i] : g.inl[i]; }

// out[group][head] = exact merge of the (m, l, O) records of all segments of the group's ranges,
// normalised; lse = M + log L.  The ranges of a group are consecutive table entries, so their
// logits are one contiguous piece of the row: the concatenation the paper describes is how the
// logits are stored, and merging the records of its pieces is the one softmax over it.
// Grid (n_groups, n_q_heads).  A group of many ranges deals its ranges to the slices, a group of
// few ranges the records of each range.
template <int D>
__global__ __launch_bounds__(kReduceBlock) void hg_concat_reduce_kernel(const ConcatReduceArgs a)
{
    constexpr int S = kReduceBlock / D;
    const int gi = blockIdx.x, h = blockIdx.y;
    const int c = threadIdx.x % D, sl = threadIdx.x / D;
    const int hk = h / a.ws.group, gidx = h - hk * a.ws.group;
    const int chunk = gidx / a.ws.gt, gl = gidx - chunk * a.ws.gt;
    const int stream = hk * a.ws.n_chunks + chunk;
    const int r0 = group_entry(a.groups, gi), r1 = group_entry(a.groups, gi + 1);

    const bool by_range = r1 - r0 >= S;
    float mx = kNegBig, lt = 0.f, ot = 0.f;  // log2 units
    for (int r = r0 + (by_range ? sl : 0); r < r1; r += by_range ? S : 1) {
        const int pre0 = table_entry(a.tab, r).pre, pre1 = table_entry(a.tab, r + 1).pre;
        if (pre1 == pre0) continue;
        const int64_t p0 = (int64_t)stream * a.ws.ltok + pre0, p1 = (int64_t)stream * a.ws.ltok + pre1;
        const int64_t w0 = p0 / a.ws.span;
        const int n_rec = (int)((p1 - 1) / a.ws.span - w0) + 1;
        const int64_t rec0 = (w0 + (int64_t)stream * a.tab.n_ranges + r) * a.ws.gt + gl;
#pragma unroll 4
        for (int i = by_range ? 0 : sl; i < n_rec; i += by_range ? 1 : S) {
            const int64_t th = rec0 + (int64_t)i * a.ws.gt;
            const float mi = a.ws_m[th], li = a.ws_l[th], oi = a.ws_o[th * D + c];
            const float mn = fmaxf(mx, mi);
            const float wa = fast_exp2(mx - mn), wb = fast_exp2(mi - mn);
            lt = lt * wa + li * wb;
            ot = ot * wa + oi * wb;
            mx = mn;
        }
    }
    if (!combine_slices<D>(mx, lt, ot, c, sl)) return;
    const int64_t gh = (int64_t)gi * a.ws.n_q_heads + h;
    const bool empty = !(lt > 0.f);
    a.out[gh * D + c] = empty ? 0.f : ot / lt;
    if (c == 0 && a.lse) a.lse[gh] = empty ? -INFINITY : mx * kLn2 + logf(lt);
}

// ---- table upload (host tables reach the device through kernel arguments only) ----------------

// Sets n words to one value (the shared bounds of the filter pass start at 0; a kernel rather
// than a memset so that the call can be recorded into a graph).
__global__ __launch_bounds__(256) void hg_fill_kernel(uint32_t *dst, int64_t n, uint32_t value)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] = value;
}

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

// One-pass read stream, alone or next to writes: what this memory system gives the access pattern
// of the streaming kernels (one workgroup per compute unit, non-temporal 16-byte loads, 32 KiB per
// workgroup iteration, starts 32 KiB further apart than the shares are long).  With wvec > 0 every
// workgroup also writes wvec 16-byte vectors per iteration on average, issued as one contiguous
// burst of burst * wvec vectors every `burst` iterations (streaming stores if nt).
__global__ __launch_bounds__(256) void hg_calibration_stream_kernel(const hg_u32x4 *src, size_t share_vec, hg_u32x4 *dst, int wvec,
                                                                  int burst, int nt)
{
    constexpr int U = 8;
    const hg_u32x4 *base = src + (size_t)blockIdx.x * (share_vec + 2048);
    const int iters = (int)(share_vec / (256 * U));
    hg_u32x4 *out = dst + (size_t)blockIdx.x * (size_t)iters * (size_t)wvec;
    hg_u32x4 acc = {0u, 0u, 0u, 0u};
    int next_burst = burst - 1;
    for (int it = 0; it < iters; ++it) {
        hg_u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(base + (size_t)it * (256 * U) + u * 256 + threadIdx.x);
        hg_u32x4 x = v[0];
#pragma unroll
        for (int u = 1; u < U; ++u) x ^= v[u];
        acc ^= x;
        if (wvec > 0 && it == next_burst) {
            const int n = burst * wvec;
            hg_u32x4 *to = out + (size_t)(it / burst) * (size_t)n;
            for (int i = threadIdx.x; i < n; i += 256) {
                if (nt)
                    __builtin_nontemporal_store(acc, to + i);
                else
                    to[i] = acc;
            }
            next_burst += burst;
        }
    }
    // (keeps the loads alive; never true for the zero-filled source a caller passes)
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) dst[0] = acc;
}

}  // namespace hg
