// Attention over a listed set of tokens per (group, query head): the executor's side of a
// selection that was decided elsewhere (Pre-QK^T selection, or a Post-QK^T selection taken with
// another query).
#pragma once

#include "hg_common.hip.h"

namespace hg {

// ---- hg_gather_kernel: (m, l, O) over the tokens index[group][head][0..k) ----------------------
//
// One workgroup of four waves per (group, query head).  A row is spread over a lane group (16 or 8
// lanes, 16 bytes each) as in the vector streaming kernel; the lane groups of the workgroup take
// the listed tokens in turn, four per lane group at a time so that the eight row loads of a step
// are in flight together.  Negative entries are padding and are skipped; a token may be listed
// more than once and then counts as often.  Latency-bound: a few thousand scattered rows at most.
struct GatherArgs {
    const void *q, *k, *v;
    int64_t stride_b, stride_h, stride_t;  // elements
    PageMap pages;                         // table == nullptr: contiguous cache
    const int32_t *index;                  // [n_groups][Hq][max_k] token positions, < 0: none
    float *m, *l, *o;                      // [n_groups][Hq](..[D]); m in natural-log units
    int32_t max_k, n_q_heads, group;       // group = query heads per KV head
    float qscale;                          // scale * log2(e)
    GroupTable seqs;                       // seqs[g] = sequence of group g (n_groups entries)
};

template <typename TR>
__global__ __launch_bounds__(256) void hg_gather_kernel(const GatherArgs a)
{
    constexpr int D = TR::D, EPL = TR::EPL, NV = TR::NV, EPV = TR::EPV, ES = TR::ES;
    constexpr int LPR = TR::LPR, RPW = TR::RPW, NG = 4 * RPW;  // lane groups per workgroup
    constexpr int U = 4;
    __shared__ float sm[NG][D + 2];

    const int gi = blockIdx.x, h = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
    const int seq = a.seqs.ext ? a.seqs.ext[gi] : a.seqs.inl[gi];
    const int hk = h / a.group;
    const int64_t gh = (int64_t)gi * a.n_q_heads + h;
    const int32_t *idx = a.index + gh * a.max_k;

    float qf[EPL];
    {
        const char *qrow = static_cast<const char *>(a.q) + ((int64_t)seq * a.n_q_heads + h) * (int64_t)(D * ES);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            typename TR::Raw raw = TR::template load<false>(qrow, sub, j);
            TR::widen(raw, &qf[j * EPV]);
        }
#pragma unroll
        for (int i = 0; i < EPL; ++i) qf[i] *= a.qscale;
    }

    const bool paged = a.pages.table != nullptr;
    const int64_t slab = ((paged ? 0 : (int64_t)seq * a.stride_b) + (int64_t)hk * a.stride_h) * ES;
    const char *kbase = static_cast<const char *>(a.k) + slab;
    const char *vbase = static_cast<const char *>(a.v) + slab;
    const int64_t row_bytes = a.stride_t * ES;
    const int32_t *table = paged ? a.pages.table + (int64_t)seq * a.pages.max_blocks : nullptr;

    float m = kNegBig, l = 0.f, acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;

    for (int j0 = grp * U; j0 < a.max_k; j0 += NG * U) {
        int tok[U];
        typename TR::Raw kraw[U][NV], vraw[U][NV];
#pragma unroll
        for (int u = 0; u < U; ++u) tok[u] = j0 + u < a.max_k ? idx[j0 + u] : -1;
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int j = 0; j < NV; ++j) kraw[u][j] = typename TR::Raw{}, vraw[u][j] = typename TR::Raw{};
            if (tok[u] >= 0) {  // padding touches no memory at all
                const int t = tok[u];
                const int64_t off = paged ? paged_row_offset(table[t >> a.pages.shift], t, a.pages.mask, (uint32_t)(a.stride_b * ES), (uint32_t)row_bytes)
                                          : (int64_t)t * row_bytes;
#pragma unroll
                for (int j = 0; j < NV; ++j) kraw[u][j] = TR::template load<false>(kbase + off, sub, j);
#pragma unroll
                for (int j = 0; j < NV; ++j) vraw[u][j] = TR::template load<false>(vbase + off, sub, j);
            }
        }
        float s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[EPL];
#pragma unroll
            for (int j = 0; j < NV; ++j) TR::widen(kraw[u][j], &kf[j * EPV]);
            float dot = 0.f;
#pragma unroll
            for (int i = 0; i < EPL; ++i) dot = fmaf(qf[i], kf[i], dot);
            s[u] = tok[u] < 0 ? -INFINITY : lane_group_sum<LPR>(dot);
        }
        const float mn = fmaxf(fmaxf(m, fmaxf(s[0], s[1])), fmaxf(s[2], s[3]));
        const float alpha = fast_exp2(m - mn);
        m = mn;
        l *= alpha;
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float p = fast_exp2(s[u] - mn);  // 0 for padding
            l += p;
            float vf[EPL];
#pragma unroll
            for (int j = 0; j < NV; ++j) TR::widen(vraw[u][j], &vf[j * EPV]);
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] = fmaf(p, vf[i], acc[i]);
        }
    }

    // every lane group has its own (m, l, acc); all lanes of a group hold the same m and l
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int i = 0; i < EPV; ++i) sm[grp][TR::vec_offset(sub, j) + i] = acc[j * EPV + i];
    if (sub == 0) {
        sm[grp][D] = m;
        sm[grp][D + 1] = l;
    }
    __syncthreads();
    if (threadIdx.x < D) {
        const int c = threadIdx.x;
        float mx = kNegBig;
#pragma unroll
        for (int g = 0; g < NG; ++g) mx = fmaxf(mx, sm[g][D]);
        float lt = 0.f, ot = 0.f;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const float w = fast_exp2(sm[g][D] - mx);
            lt += w * sm[g][D + 1];
            ot += w * sm[g][c];
        }
        const bool empty = !(lt > 0.f);
        a.o[gh * D + c] = empty ? 0.f : ot;
        if (c == 0) {
            a.m[gh] = empty ? -INFINITY : mx * kLn2;
            a.l[gh] = empty ? 0.f : lt;
        }
    }
}

}  // namespace hg
