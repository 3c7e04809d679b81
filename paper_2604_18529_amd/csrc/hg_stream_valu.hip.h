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

// (One workgroup per compute unit is launched on long inputs, so the register allocator is told
// that two waves per SIMD is all the occupancy this kernel wants.)
// Logits mode.  Measured on MI355X, stores that trickle out next to a saturating read stream cost
// the memory system far more than their share of the bytes: the scan that wrote its 128 bytes per
// wave and iteration ran at 67 % of the HBM peak where the same scan without stores reaches 86 %,
// with no extra traffic in the byte counters; what costs is every switch between reading and
// writing, not the bytes.  So the logits are collected in LDS (a window of up to 32768 logits per
// head chunk, 128 KiB), and only when the window is full do all four waves stop reading and write
// it out together, in runs of up to 128 KiB per head with streaming stores; then they go on
// reading.  The window runs on across segment boundaries as long as the next segment's logits
// continue where the window ends in the rows of `logits` (the next range of the same stream; with
// one head per stream also the next stream), so a ragged table does not mean more write-outs.
#ifndef HG_VALU_ROUND_FLOATS
#define HG_VALU_ROUND_FLOATS 32768
#endif
constexpr int kValuRoundFloats = HG_VALU_ROUND_FLOATS;  // logits in the window, all heads of the chunk together

template <int GT, int CH>
struct ValuRound {
    static constexpr int kIterTokens = kValuWaves * CH;  // tokens of one workgroup iteration
    static constexpr int kTokens = kValuRoundFloats / GT / kIterTokens * kIterTokens;  // tokens the window holds per head
    static_assert(kTokens >= kIterTokens, "the window holds at least one workgroup iteration");
};

__device__ __forceinline__ void workgroup_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// FUSED (statistics mode, contiguous cache; hg_attn_partial_merge on small inputs): a workgroup takes
// all ranges of one (group, stream), writes their triples itself and, at the end, the group's
// merged output -- partial, segment reduce and merge in one launch.
template <typename TR, int GT, int U, int MODE, bool PAGED, bool FUSED = false>
__global__ __launch_bounds__(kValuBlock) __attribute__((amdgpu_waves_per_eu(1, 2))) void hg_partial_kernel(const PartialArgs a)
{
    static_assert(!FUSED || (MODE == kModeStats && !PAGED), "the fused walk exists for the statistics mode on a contiguous cache");
    constexpr int D = TR::D, EPL = TR::EPL, NV = TR::NV, EPV = TR::EPV, ES = TR::ES;
    constexpr int LPR = TR::LPR, RPW = TR::RPW;
    constexpr int CH = RPW * U;  // tokens one wave takes per iteration
    using Round = ValuRound<GT, CH>;
    __shared__ __align__(16) float ring[MODE == kModeLogits ? GT * Round::kTokens : 1];  // logits mode: the window, [head][token]
    // logits mode: tokens in the window, the index in `logits` of its first token for the chunk's
    // first head (row * ltok + column), and the valid heads of its chunk.  Uniform.
    int win_fill = 0, win_nh = 0;
    int64_t win_at = 0;
    // all waves write the window's win_fill tokens per head to the rows of `logits` (1 KiB per wave
    // and store instruction), between two barriers: the window is complete before anybody copies,
    // and copied before anybody overwrites it
    auto flush_window = [&]() __attribute__((always_inline)) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
        workgroup_lds_barrier();
        for (int g = 0; g < win_nh; ++g) {
            float *dst = a.logits + win_at + (int64_t)g * a.ws.ltok;
            for (int c = 4 * (int)threadIdx.x; c < win_fill; c += 4 * kValuBlock) {
                const f4 vals = *reinterpret_cast<const f4 *>(ring + g * Round::kTokens + c);
                if (c + 4 <= win_fill) {
                    const f4u out = vals;
                    __builtin_nontemporal_store(out, reinterpret_cast<f4u *>(dst + c));
                } else {
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        if (c + x < win_fill) dst[c + x] = vals[x];
                }
            }
        }
        workgroup_lds_barrier();
        win_at += win_fill;
        win_fill = 0;
    };

    __shared__ float sm[kValuWaves][GT][D + 2];
    // filter mode (one head per stream): each wave's bound, and the survivors waiting to be written out
    constexpr int kStage = 2 * CH;
    __shared__ float wmin[MODE == kModeFilter ? kValuWaves : 1];
    __shared__ float stage_val[MODE == kModeFilter ? kValuWaves * kStage : 1];
    __shared__ int32_t stage_col[MODE == kModeFilter ? kValuWaves * kStage : 1];
    static_assert(MODE != kModeFilter || (GT == 1 && U <= LPR && CH <= 64), "filter mode: one head, one lane per row of an iteration");

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPR, grp = lane / LPR;

    if constexpr (MODE == kModeFilter) {
        // the selection that follows counts its finished workgroups from zero
        if (blockIdx.x == 0)
            for (int64_t i = threadIdx.x; i < a.n_tail; i += blockDim.x) a.tail_cnt[i] = 0u;
    }
    // FUSED: the group's running merge, per (head, channel) this thread owns (log2 units, as the
    // segment results)
    constexpr int kOwn = (GT * D + kValuBlock - 1) / kValuBlock;
    float f_m[kOwn], f_l[kOwn], f_o[kOwn];
#pragma unroll
    for (int it = 0; it < kOwn; ++it) {
        f_m[it] = kNegBig;
        f_l[it] = 0.f;
        f_o[it] = 0.f;
    }
    auto segment = [&](int stream, int r_idx, const RangeEntry &e, int seg_t0, int seg_t1, int seg_col0, int64_t slot) __attribute__((always_inline)) {
    // Tokens [t0, t1) the waves share iteration by iteration and the column of t0 -- or, in filter
    // mode, this wave's own consecutive sub-span, so that what it appends is in column order.
    int t0 = seg_t0, t1 = seg_t1, col0 = seg_col0;
    const int first = MODE == kModeFilter ? 0 : wave * CH;            // this wave's first iteration, relative to t0
    constexpr int kStep = MODE == kModeFilter ? CH : kValuWaves * CH;  // from one of its iterations to the next
    if constexpr (MODE == kModeFilter) {
        const int sub_len = filter_sub_len(seg_t1 - seg_t0, kValuWaves);
        t0 = min(seg_t0 + wave * sub_len, seg_t1);
        t1 = min(t0 + sub_len, seg_t1);
        col0 = seg_col0 + (t0 - seg_t0);
    }
    const int seq = e.seq;
    const int hk = stream / a.ws.n_chunks;
    const int chunk = stream - hk * a.ws.n_chunks;
    const int g0 = chunk * GT;                              // first head of this chunk inside its group
    const int nh = min(GT, a.ws.group - g0);                // valid heads in this chunk
    const int h0 = hk * a.ws.group + g0;                    // first query head

    if constexpr (MODE == kModeLogits) {
        // does this segment go on where the window ends?  Otherwise the window is written out first.
        const int64_t seg_at = (int64_t)h0 * a.ws.ltok + seg_col0;
        if (win_fill > 0 && (seg_at != win_at + win_fill || nh != win_nh)) flush_window();
        if (win_fill == 0) {
            win_at = seg_at;
            win_nh = nh;
        }
    }

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

    // concat mode: the rows of the given logits (lrow[g][tok] is the logit of token tok)
    const float *lrow[GT];
    if constexpr (MODE == kModeConcat) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const int h = h0 + (g < nh ? g : 0);
            lrow[g] = a.logits + (int64_t)h * a.ws.ltok + (col0 - t0);
        }
    }

    float m[GT], l[GT], acc[GT][EPL];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        m[g] = kNegBig;
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
        if (t0 + first < t1) lookup(t0 + first, pg);
    }

    // Filter mode.  Lane `sub` of a lane group speaks for row `sub` of the group's U rows of an
    // iteration (sub < U) and keeps the four largest logits it has seen.  At a refresh every wave
    // finds, by bisection on the key bits with ballots, a value that ceil(top_k / waves) of the
    // logits its lanes keep reach; the smallest of the waves' values is then reached by top_k
    // distinct logits of this segment: a lower bound of the group's top_k-th largest logit, below
    // which nothing can be among the kept tokens.  (Counting among all kept logits follows the
    // true value far more closely than the smallest of the lanes' maxima would: that one sits at
    // the level of about the 700th largest logit for 128 lanes, this one near the 180th.)
    // Survivors are staged in LDS in column order and
    // written out in runs (a conditional global store in every iteration would leave the number of
    // memory operations in flight unknown at compile time and stall the row loads).
    const bool owner = sub < U;
    float top_a = -INFINITY, top_b = -INFINITY, top_c = -INFINITY, top_d = -INFINITY, tau = -INFINITY;
    uint32_t staged = 0, written = 0;
    int iter = 0, next_refresh = 1;
    auto flush_staged = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int64_t dst = (int64_t)h0 * a.ws.ltok + col0 + written;
#pragma unroll
        for (int x = 0; x < kStage; x += 64) {
            if (x + lane < (int)staged) {
                a.surv_val[dst + x + lane] = stage_val[wave * kStage + x + lane];
                a.surv_col[dst + x + lane] = stage_col[wave * kStage + x + lane];
            }
        }
        written += staged;
        staged = 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    if constexpr (MODE == kModeFilter) {
        if (lane == 0) lds_publish(&wmin[wave], -INFINITY);
        __syncthreads();
    }

    int it = 0;  // logits mode: this wave's iteration inside the segment
    for (int tb = t0 + first; tb < t1; tb += kStep) {
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
            if constexpr (MODE != kModeLogits && MODE != kModeFilter) {
#pragma unroll
                for (int j = 0; j < NV; ++j) vraw[u][j] = TR::template load<true>(vbase + off, sub, j);
            }
        }

        if constexpr (PAGED) {
            if (tb + kStep < t1) lookup(tb + kStep, pg_next);
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
        if constexpr (MODE == kModeConcat) {
            // the given logits take the place of q.k (natural-log units -> log2 units)
#pragma unroll
            for (int g = 0; g < GT; ++g)
#pragma unroll
                for (int u = 0; u < U; ++u) s[g][u] = valid[u] ? sv[g][u] * kLog2e : -INFINITY;
        }
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
            // puts entry (g, u) = (idx / U, idx % U), idx = pass * LPR + sub, into this round's
            // buffer at the token's place, so one LDS store instruction of the wave covers U * RPW
            // consecutive tokens of a head.  (Tokens past the segment's end leave their place
            // unwritten; only the segment's tokens are copied out.)
            constexpr int kPasses = (GT * U + LPR - 1) / LPR;
            // (every wave makes the same decision for the same workgroup iteration)
            if (win_fill + Round::kIterTokens > Round::kTokens) flush_window();
            float *buf = ring + win_fill + wave * CH;
#pragma unroll
            for (int pass = 0; pass < kPasses; ++pass) {
                const int idx = pass * LPR + sub;
                float val = 0.f;
                bool ok = false;
                int place = 0;
#pragma unroll
                for (int g = 0; g < GT; ++g)
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        if (g * U + u >= pass * LPR && g * U + u < (pass + 1) * LPR && idx == g * U + u) {
                            val = s[g][u];
                            ok = valid[u] && g < nh;
                            place = g * Round::kTokens + RPW * u + grp;
                        }
                if (ok) buf[place] = val;
            }
            ++it;
            win_fill += Round::kIterTokens;
        }

        if constexpr (MODE == kModeFilter) {
            // this lane's row of the iteration: logit, validity, token
            float val = -INFINITY;
            int tok = t0;
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (sub == u) {
                    val = s[0][u];  // (-inf past the end of the sub-span)
                    tok = tokc[u];
                }
            if (!owner) val = -INFINITY;
            const uint64_t pass = __builtin_amdgcn_ballot_w64(val >= tau && val > -INFINITY);
            if (pass) {
                // rows of an iteration in token order: row u of group g is token RPW * u + g
                constexpr uint64_t kEvery = LPR == 16 ? 0x0001000100010001ull : 0x0101010101010101ull;  // one lane per group
                const uint64_t rows_before = kEvery * ((1ull << sub) - 1ull);                   // rows u' < u of every group
                const uint64_t same_row = (kEvery << sub) & ((1ull << (grp * LPR)) - 1ull);      // row u of the groups before
                if (val >= tau && val > -INFINITY) {
                    const int at = wave * kStage + (int)staged + __builtin_popcountll(pass & rows_before) + __builtin_popcountll(pass & same_row);
                    stage_val[at] = val;
                    stage_col[at] = col0 + (tok - t0);
                }
                staged += (uint32_t)__builtin_popcountll(pass);
                if (staged > (uint32_t)(kStage - CH)) flush_staged();  // uniform
            }
            {   // the four largest of this lane's rows
                float x = val, hi;
                hi = fmaxf(top_a, x);
                x = fminf(top_a, x);
                top_a = hi;
                hi = fmaxf(top_b, x);
                x = fminf(top_b, x);
                top_b = hi;
                hi = fmaxf(top_c, x);
                x = fminf(top_c, x);
                top_c = hi;
                top_d = fmaxf(top_d, x);
            }
            if (iter == next_refresh) {
                next_refresh = next_refresh * 5 / 2 + 1;
                // largest key (upper 20 bits) that `need` of the wave's kept logits reach; lanes that
                // speak for no row hold -inf four times, which no useful bound admits
                const uint32_t ka = order_key(top_a), kb = order_key(top_b), kc = order_key(top_c), kd = order_key(top_d);
                const int need = (a.filter_k + kValuWaves - 1) / kValuWaves;
                uint32_t tw = 0u;
                for (int b = 31; b >= 12; --b) {
                    const uint32_t c = tw | (1u << b);
                    const int reach = __builtin_popcountll(__builtin_amdgcn_ballot_w64(ka >= c)) + __builtin_popcountll(__builtin_amdgcn_ballot_w64(kb >= c)) +
                                      __builtin_popcountll(__builtin_amdgcn_ballot_w64(kc >= c)) + __builtin_popcountll(__builtin_amdgcn_ballot_w64(kd >= c));
                    if (reach >= need) tw = c;
                }
                const float low = tw > order_key(-INFINITY) ? key_to_float(tw) : -INFINITY;
                if (lane == 0) lds_publish(&wmin[wave], low);
                // (a wave's own LDS operations complete in order; the other waves' entries may be
                // older, i.e. lower, which is still a valid bound)
                float t = lds_peek(&wmin[0]);
#pragma unroll
                for (int w = 1; w < kValuWaves; ++w) t = fminf(t, lds_peek(&wmin[w]));
                tau = fmaxf(tau, t);
            }
            ++iter;
        }

        if constexpr (MODE != kModeLogits && MODE != kModeFilter) {
        float p[GT][U];
        // online softmax update (concat mode: over the given logits; the records of all segments of a
        // group are merged exactly afterwards, which is the one softmax over the concatenated logits)
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
        }  // modes that read V
        if constexpr (PAGED) {
#pragma unroll
            for (int u = 0; u < U; ++u) pg[u] = pg_next[u];
        }
    }
    if constexpr (MODE == kModeLogits) {
        // A wave without tokens in the segment's last workgroup iteration still takes that
        // iteration's step, so that all waves agree on the window; then the part of the last
        // iteration beyond the segment's end is given back.
        const int n_iters = (seg_t1 - seg_t0 + Round::kIterTokens - 1) / Round::kIterTokens;
        if (it < n_iters) {
            if (win_fill + Round::kIterTokens > Round::kTokens) flush_window();
            win_fill += Round::kIterTokens;
        }
        win_fill -= n_iters * Round::kIterTokens - (seg_t1 - seg_t0);
        return;  // nothing to merge or record
    }
    if constexpr (MODE == kModeFilter) {
        flush_staged();
        if (lane == 0) a.surv_cnt[(slot * kValuWaves + wave) * GT] = (int32_t)written;
        __syncthreads();  // the next segment resets the waves' bounds
        return;
    }

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
    if constexpr (FUSED) {
        // the same results again, folded into the group's running merge
#pragma unroll
        for (int it = 0; it < kOwn; ++it) {
            const int idx = (int)threadIdx.x + it * kValuBlock;
            const int g = idx / D, c = idx - g * D;
            if (idx >= GT * D || g >= nh) continue;
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
            const float m_new = fmaxf(f_m[it], mx);
            const float w_old = fast_exp2(f_m[it] - m_new), w_seg = fast_exp2(mx - m_new);
            f_l[it] = f_l[it] * w_old + lt * w_seg;
            f_o[it] = f_o[it] * w_old + ot * w_seg;
            f_m[it] = m_new;
        }
    }
    __syncthreads();  // the next segment reuses sm
    };
    if constexpr (FUSED) {
        const int gi = (int)(blockIdx.x % (unsigned)a.fused_n_groups), stream = (int)(blockIdx.x / (unsigned)a.fused_n_groups);
        const int hk = stream / a.ws.n_chunks, g0 = (stream - hk * a.ws.n_chunks) * GT;
        const int nh = min(GT, a.ws.group - g0), h0 = hk * a.ws.group + g0;
        for_each_range_of_group(a, segment, [&](int, int r_idx) __attribute__((always_inline)) {
            // a range without tokens: m = -inf, l = 0, O = 0
            for (int idx = threadIdx.x; idx < GT * D; idx += kValuBlock) {
                const int g = idx / D, c = idx - g * D;
                if (g >= nh) continue;
                const int64_t rh = (int64_t)r_idx * a.ws.n_q_heads + h0 + g;
                a.out_o[rh * D + c] = 0.f;
                if (c == 0) {
                    a.out_m[rh] = -INFINITY;
                    a.out_l[rh] = 0.f;
                }
            }
        });
#pragma unroll
        for (int it = 0; it < kOwn; ++it) {
            const int idx = (int)threadIdx.x + it * kValuBlock;
            const int g = idx / D, c = idx - g * D;
            if (idx >= GT * D || g >= nh) continue;
            const int64_t gh = (int64_t)gi * a.ws.n_q_heads + h0 + g;
            const bool none = f_l[it] <= 0.f;  // a group without tokens
            a.merged_out[gh * D + c] = none ? 0.f : f_o[it] / f_l[it];
            if (c == 0 && a.merged_lse) a.merged_lse[gh] = none ? -INFINITY : f_m[it] * kLn2 + logf(f_l[it]);
        }
    } else {
        for_each_segment(a.ws, a.tab, segment);
    }
    if constexpr (MODE == kModeLogits) {
        if (win_fill > 0) flush_window();
    }
}

}  // namespace hg
