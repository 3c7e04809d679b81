// Streaming kernel on the vector ALU: statistics, logits-export and concat modes.
//
// Lane layout.  One K or V row (head_dim elements, 128..512 bytes) is spread over the 16 lanes of
// a DPP row, each lane holding 8..32 contiguous bytes per 256-byte segment, so one wave load
// instruction fetches four whole rows (1 KiB, fully coalesced).  A lane keeps the matching
// channels of q (pre-multiplied by scale*log2 e) and of the O accumulator, so P.V is lane-local
// and the only cross-lane work is the 16-lane sum of the dot product (four DPP adds).  The four
// 16-lane groups of a wave and the four waves of a workgroup run independent online-softmax
// streams that are merged once per segment.
#pragma once

#include "hg_common.hip.h"

namespace hg {

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

// (One workgroup per compute unit is launched on long inputs, so the register allocator is told
// that two waves per SIMD is all the occupancy this kernel wants.)
template <typename TR, int GT, int U, int MODE, bool PAGED>
__global__ __launch_bounds__(kValuBlock) __attribute__((amdgpu_waves_per_eu(1, 2))) void hg_partial_kernel(const PartialArgs a)
{
    constexpr int D = TR::D, EPL = TR::EPL, NV = TR::NV, EPV = TR::EPV, ES = TR::ES;
    constexpr int LPR = TR::LPR, RPW = TR::RPW;
    constexpr int CH = RPW * U;  // tokens one wave takes per iteration

    __shared__ float sm[kValuWaves][GT][D + 2];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPR, grp = lane / LPR;

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
            const int tok = tbb + RPW * u + grp;
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
            const int tok = tb + RPW * u + grp;
            valid[u] = tok < t1;
            tokc[u] = valid[u] ? tok : t1 - 1;  // clamp: never read past the segment
            const int64_t off = PAGED ? paged_row_offset(pg[u], tokc[u], a.pages.mask, (uint32_t)block_bytes, (uint32_t)row_bytes)
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
        // concat mode: the given logits of these tokens (unconditional loads, issued with the V loads)
        float sv[GT][U];
        if constexpr (MODE == kModeConcat) {
#pragma unroll
            for (int g = 0; g < GT; ++g)
#pragma unroll
                for (int u = 0; u < U; ++u) sv[g][u] = lrow[g][tokc[u]];
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
                    d = lane_group_sum<LPR>(d);
                    s[g][u] = valid[u] ? d : -INFINITY;
                }
            }
        }

        if constexpr (MODE == kModeLogits) {
            // Every lane of a group holds all GT*U logits of the group's U tokens.  Lane `sub`
            // stores entry (g, u) = (idx / U, idx % U), idx = pass * LPR + sub, so one store
            // instruction of the wave writes U * RPW consecutive tokens (128 bytes or more) of
            // each head instead of one token per group.
            constexpr int kPasses = (GT * U + LPR - 1) / LPR;
#pragma unroll
            for (int pass = 0; pass < kPasses; ++pass) {
                const int idx = pass * LPR + sub;
                float val = 0.f;
                bool ok = false;
                int tok = t0;
#pragma unroll
                for (int g = 0; g < GT; ++g)
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        if (g * U + u >= pass * LPR && g * U + u < (pass + 1) * LPR && idx == g * U + u) {
                            val = s[g][u];
                            ok = valid[u] && g < nh;
                            tok = tokc[u];
                        }
                if (ok) a.logits[(int64_t)(h0 + idx / U) * a.ws.ltok + col0 + (tok - t0)] = val;
            }
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
            // (the mask is applied as a product so that every logit load stays unconditional)
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

    // merge the lane groups of the wave (lanes xor 16, xor 32; xor 8 too when a group is 8 lanes)
#pragma unroll
    for (int g = 0; g < GT; ++g) {
#pragma unroll
        for (int step = LPR; step <= 32; step <<= 1) {
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

}  // namespace hg
