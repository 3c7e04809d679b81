// Streaming kernel for grouped-query attention on the matrix cores, fp16 with head_dim 64
// (128-byte rows).  Same structure as hg_partial_gqa_kernel (head_dim 128); what differs is the
// lane geometry, because a row is only 8 lanes wide:
//
//   loads  lane l holds chunk l%8 (8 channels) of row l/8 of a load: one load instruction fetches
//          8 whole rows, a 32-token block is 4 K loads + 4 V loads per lane (4 KiB each per wave).
//   K      staged in wave-private LDS with 144-byte rows (conflict-free 16-byte reads), read back
//          token-per-lane: lane (n = l%16, rg = l/16) takes token n of each half, channel chunk
//          4kk + rg for kk = 0, 1 -> two MFMAs (K = 64 channels) per half.
//   V      a lane owns 4 tokens of the block (rows l/8 of the 4 loads): the even tokens 8j + 2rg for
//          lanes n < 8, the odd tokens 8j + 2rg + 1 for lanes n >= 8, always chunk n%8.  The P.V
//          MFMA takes 8 contraction slots per lane, so lanes n < 8 fill slots 0..3 and leave
//          4..7 zero, lanes n >= 8 the other way round; columns n and n^8 of the result are two
//          partial sums of the same channel 8*(n%8) + nb and are added once per segment.
//          Slot order inside a parity is load 0, 2, 1, 3, which puts tokens t and t+16 in
//          adjacent slots, so that a lane of the S tile writes its two halves as one word of P.
#pragma once

#include "hg_common.hip.h"
#include "hg_stream_gqa.hip.h"

namespace hg {

constexpr int kGqa64KRow = 144;  // 128 bytes + 16: 16 rows land in 16 distinct bank groups
constexpr int kGqa64KBytes = kGqaBlockTokens * kGqa64KRow;
constexpr int kGqa64WaveBytes = kGqa64KBytes + 2 * kGqaPBytes;

template <int MODE, bool PAGED, bool BF16>
__global__ __launch_bounds__(kGqaBlock, kGqaWaves <= 4 ? 2 : 1) void hg_partial_gqa64_kernel(const PartialArgs a)
{
    constexpr int D = 64;
    constexpr int kMergeBytes = kGqaWaves * kGqaHeads * (D + 2) * 4;
    constexpr int kSmemBytes = kGqaWaves * kGqa64WaveBytes > kMergeBytes ? kGqaWaves * kGqa64WaveBytes : kMergeBytes;
    __shared__ __align__(16) char smem[kSmemBytes];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: block loop control stays scalar
    const int n = lane & 15, rg = lane >> 4;  // MFMA view: column / k-group
    const int c8 = lane & 7, rl = lane >> 3;  // load view: chunk of the row / row of the load
    const bool odd = n >= 8;                  // this lane's V tokens are the odd ones of its k-group

    char *kls = smem + wave * kGqa64WaveBytes;
    char *pls = kls + kGqa64KBytes;

    for_each_segment(a.ws, a.tab, [&](int stream, int r_idx, const RangeEntry &e, int t0, int t1, int col0, int64_t slot) __attribute__((always_inline)) {
    const int seq = e.seq;
    const int hk = stream / a.ws.n_chunks;
    const int chunk = stream - hk * a.ws.n_chunks;
    const int g0 = chunk * kGqaHeads;
    const int nh = min(kGqaHeads, a.ws.group - g0);
    const int h0 = hk * a.ws.group + g0;

    // Q as A operand: lane l holds head l%16, channels 8*(4kk + l/16)..+7 for kk = 0, 1
    hg_u32x4 qa[2];
    if constexpr (MODE != kModeConcat) {
        const uint16_t *qrow = static_cast<const uint16_t *>(a.q) + ((int64_t)seq * a.ws.n_q_heads + h0 + (n < nh ? n : 0)) * D;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            hg_u32x4 raw = *reinterpret_cast<const hg_u32x4 *>(qrow + 8 * (4 * kk + rg));
            if (n >= nh) raw = hg_u32x4{0u, 0u, 0u, 0u};
            qa[kk] = raw;
        }
    }

    // concat mode: the logits row of this lane's head n, and the running maximum and sum of that
    // head (log2 units) in A-operand order, as in the head_dim 128 kernel
    const float *lrow = nullptr;
    float m_a = kNegBig, l_a = 0.f;
    if constexpr (MODE == kModeConcat) {
        const int h = h0 + (n < nh ? n : 0);
        lrow = a.logits + (int64_t)h * a.ws.ltok + (col0 - t0);
    }

    float m[4], lsum[4];
    hg_f4 o[8];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        m[r] = kNegBig;
        lsum[r] = 0.f;
    }
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) o[nb] = hg_f4{0.f, 0.f, 0.f, 0.f};

    // Contiguous cache: the address of a row is a uniform 64-bit base (start of the segment) plus a
    // 32-bit byte offset, (token - t0) * row_bytes + 16 * chunk.  The host keeps a workgroup's span
    // times the row stride below 4 GiB.  Only the lane part of the offset is a vector quantity, so a
    // load costs one add and one min (the clamp to the last row, taken in offset space).
    // Paged cache: per-lane 64-bit addresses from the block table.
    const int64_t slab = PAGED ? (int64_t)hk * a.stride_h : (int64_t)seq * a.stride_b + (int64_t)hk * a.stride_h + (int64_t)t0 * a.stride_t;
    const char *kbase = static_cast<const char *>(a.k) + slab * 2 + (PAGED ? c8 * 16 : 0);
    const char *vbase = static_cast<const char *>(a.v) + slab * 2 + (PAGED ? c8 * 16 : 0);
    const int64_t row_bytes = a.stride_t * 2;
    const int64_t block_bytes = a.stride_b * 2;
    const uint32_t row_b32 = (uint32_t)row_bytes;
    const uint32_t lane_off = (uint32_t)(MODE == kModeConcat ? 4 * rl : rl) * row_b32 + (uint32_t)c8 * 16u;
    const uint32_t last_off = (uint32_t)(t1 - 1 - t0) * row_b32 + (uint32_t)c8 * 16u;
    const int32_t *table = PAGED ? a.pages.table + (int64_t)seq * a.pages.max_blocks : nullptr;

    // the 4 tokens a lane touches in a block, for K and for V alike: tb + 8i + rl (i = 0..3), or
    // tb + 4rl + (slot of load i) in concat mode
    auto lookup = [&](int tb, int(&pg)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tok = MODE == kModeConcat ? tb + 4 * rl + 2 * (i & 1) + (i >> 1) : tb + 8 * i + rl;
            pg[i] = table[(tok < t1 ? tok : t1 - 1) >> a.pages.shift];
        }
    };
    // Concat mode reads V only and wants slot j of k-group g to be token 8g + j (the logits a lane
    // reads are then consecutive): load i fetches token 4*rl + (slot of load i within the parity).
    auto load_rows = [&](const char *base, int tb, hg_u32x4(&reg)[4], const int(&pg)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (PAGED) {
                int tok = MODE == kModeConcat ? tb + 4 * rl + 2 * (i & 1) + (i >> 1) : tb + 8 * i + rl;
                tok = tok < t1 ? tok : t1 - 1;  // clamp: never read past the segment
                const int64_t off = paged_row_offset(pg[i], tok, a.pages.mask, (uint32_t)block_bytes, row_b32);
                reg[i] = __builtin_nontemporal_load(reinterpret_cast<const hg_u32x4 *>(base + off));
            } else {
                const int row = MODE == kModeConcat ? 2 * (i & 1) + (i >> 1) : 8 * i;
                uint32_t off = (uint32_t)(tb - t0 + row) * row_b32 + lane_off;
                off = off < last_off ? off : last_off;  // clamp: never read past the segment
                reg[i] = __builtin_nontemporal_load(reinterpret_cast<const hg_u32x4 *>(base + off));
            }
        }
    };
    // pages of the next block, the one after and the one after that (paged only)
    int pg1[4] = {0, 0, 0, 0}, pg2[4] = {0, 0, 0, 0}, pg3[4] = {0, 0, 0, 0};

    // B operand nb of the P.V product: the halves of channel 8*(n%8) + nb of the lane's 4 tokens go
    // to the slots of its parity, the other 4 slots are zero.  A byte selector of 0x0c makes
    // v_perm_b32 emit a zero byte, so the masking costs nothing beyond the transpose itself.
    const uint32_t sel_even_lo = odd ? 0x0c0c0c0cu : 0x05040100u, sel_even_hi = odd ? 0x05040100u : 0x0c0c0c0cu;
    const uint32_t sel_odd_lo = odd ? 0x0c0c0c0cu : 0x07060302u, sel_odd_hi = odd ? 0x07060302u : 0x0c0c0c0cu;
    auto v_operand = [&](const hg_u32x4(&vreg)[4], int nb) __attribute__((always_inline)) -> hg_u32x4 {
        const uint32_t s_lo = (nb & 1) ? sel_odd_lo : sel_even_lo, s_hi = (nb & 1) ? sel_odd_hi : sel_even_hi;
        hg_u32x4 braw;
        braw[0] = __builtin_amdgcn_perm(vreg[2][nb >> 1], vreg[0][nb >> 1], s_lo);
        braw[1] = __builtin_amdgcn_perm(vreg[3][nb >> 1], vreg[1][nb >> 1], s_lo);
        braw[2] = __builtin_amdgcn_perm(vreg[2][nb >> 1], vreg[0][nb >> 1], s_hi);
        braw[3] = __builtin_amdgcn_perm(vreg[3][nb >> 1], vreg[1][nb >> 1], s_hi);
        return braw;
    };

    auto compute_block = [&](int tb, int tb_next, hg_u32x4(&kreg)[4], hg_u32x4(&vreg)[4]) __attribute__((always_inline)) {
        // K: registers -> LDS (row per token) -> B operands (token per lane)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<hg_u32x4 *>(kls + (8 * i + rl) * kGqa64KRow + c8 * 16) = kreg[i];
        wave_lds_handover();
        if constexpr (PAGED && MODE == kModeStats) {
            // pages three blocks ahead, requested before this block's loads: see hg_partial_gqa_kernel
            const int tb_3 = tb + 3 * (tb_next - tb);
            if (tb_3 < t1) lookup(tb_3, pg3);
        }
        if (tb_next < t1) {
            load_rows(kbase, tb_next, kreg, pg1);
            if constexpr (PAGED && MODE == kModeLogits) {  // blocks are loaded in order: pages of the one after
                if (tb_next + kGqaWaves * kGqaBlockTokens < t1) lookup(tb_next + kGqaWaves * kGqaBlockTokens, pg1);
            }
        }
        hg_f4 s[2];
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            s[hf] = hg_f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                hg_u32x4 raw = *reinterpret_cast<const hg_u32x4 *>(kls + (16 * hf + n) * kGqa64KRow + (4 * kk + rg) * 16);
                s[hf] = mfma_16x16x32<BF16>(qa[kk], raw, s[hf]);
            }
        }

        if constexpr (MODE == kModeLogits) {
            // export through the idle P staging area as [head][32 tokens], four tokens per lane
            float *stile = reinterpret_cast<float *>(pls);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                stile[(4 * rg + r) * 32 + n] = s[0][r] * a.qscale;
                stile[(4 * rg + r) * 32 + 16 + n] = s[1][r] * a.qscale;
            }
            wave_lds_handover();
            typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int head = 8 * half + (lane >> 3), tq = 4 * (lane & 7);
                if (head < nh && tb + tq < t1) {
                    const hg_f4 vals = *reinterpret_cast<const hg_f4 *>(stile + head * 32 + tq);
                    float *dst = a.logits + (int64_t)(h0 + head) * a.ws.ltok + col0 + (tb - t0) + tq;
                    if (tb + tq + 4 <= t1) {
                        *reinterpret_cast<f4u *>(dst) = vals;
                    } else {
#pragma unroll
                        for (int x = 0; x < 4; ++x)
                            if (tb + tq + x < t1) dst[x] = vals[x];
                    }
                }
            }
            wave_lds_handover();
            return;
        }

        // online softmax on S (lane: token n of each half, heads 4rg..4rg+3)
        const bool ok0 = tb + n < t1, ok1 = tb + 16 + n < t1;
        // e = s - m against the running maximum.  Once a few blocks have been seen a new maximum is
        // rare, so the row-maximum reduction and the rescaling of the accumulators sit behind a
        // wave-uniform branch that is taken only when some logit of the block exceeds its m.
        float e0[4], e1[4];
        float top = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            e0[r] = ok0 ? fmaf(s[0][r], a.qscale, -m[r]) : -INFINITY;
            e1[r] = ok1 ? fmaf(s[1][r], a.qscale, -m[r]) : -INFINITY;
            top = fmaxf(fmaxf(e0[r], e1[r]), top);
        }
        const bool grow = __builtin_amdgcn_ballot_w64(top > 0.f) != 0;
        if (grow) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float s0 = ok0 ? s[0][r] * a.qscale : -INFINITY;
                const float s1 = ok1 ? s[1][r] * a.qscale : -INFINITY;
                const float mx = fmaxf(m[r], row16_max(fmaxf(s0, s1)));
                const float alpha = fast_exp2(m[r] - mx);
                m[r] = mx;
                e0[r] = s0 - mx;
                e1[r] = s1 - mx;
                lsum[r] *= alpha;
#pragma unroll
                for (int nb = 0; nb < 8; ++nb) o[nb][r] *= alpha;
            }
        }
        uint32_t ph[4], pl[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p0 = fast_exp2(e0[r]), p1 = fast_exp2(e1[r]);
            lsum[r] += p0 + p1;
            split_weights<BF16>(p0, p1, ph[r], pl[r]);
        }
        // P -> LDS as [head][k-group g][slot j]: token t = 16*half + n belongs to k-group (n%8)/2,
        // parity n%2, load 2*half + n/8, i.e. slot 4*(n%2) + 2*(n/8) + half: the two halves are one word
        {
            const int col = ((n & 7) >> 1) * 16 + (4 * (n & 1) + 2 * (n >> 3)) * 2;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                *reinterpret_cast<uint32_t *>(pls + (4 * rg + r) * 64 + col) = ph[r];
                *reinterpret_cast<uint32_t *>(pls + kGqaPBytes + (4 * rg + r) * 64 + col) = pl[r];
            }
        }
        wave_lds_handover();
        const hg_u32x4 pa_hi = *reinterpret_cast<const hg_u32x4 *>(pls + n * 64 + rg * 16);
        const hg_u32x4 pa_lo = *reinterpret_cast<const hg_u32x4 *>(pls + kGqaPBytes + n * 64 + rg * 16);

        // V: this lane's 4 tokens fill the slots of its parity in the order load 0, 2, 1, 3
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
            const hg_u32x4 b = v_operand(vreg, nb);
            o[nb] = mfma_16x16x32<BF16>(pa_hi, b, o[nb]);
            o[nb] = mfma_16x16x32<BF16>(pa_lo, b, o[nb]);
        }
        if (tb_next < t1) {
            load_rows(vbase, tb_next, vreg, pg1);
            if constexpr (PAGED) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    pg1[i] = pg2[i];
                    pg2[i] = pg3[i];
                }
            }
        }
        wave_lds_handover();  // the next block overwrites the K and P staging areas
    };

    // Concat mode block: the given logits, read in A-operand order (lane: head n, tokens
    // tb + 8rg .. + 7), take the place of q.k in an online softmax, as in the head_dim 128 kernel.
    // The 8 logits a lane needs for block tb (head n, tokens tb + 8rg .. + 7) are requested with the
    // V rows of that block, two 16-byte loads when the block is full (they need 4-byte alignment
    // only), clamped single loads in the last block of a segment.  The branch is wave-uniform, so
    // neither side has to wait for its loads before the join.
    typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
    auto load_logits = [&](int tb, float(&sv)[8]) __attribute__((always_inline)) {
        if (tb + kGqaBlockTokens <= t1) {
            const f4u lo4 = *reinterpret_cast<const f4u *>(lrow + tb + 8 * rg);
            const f4u hi4 = *reinterpret_cast<const f4u *>(lrow + tb + 8 * rg + 4);
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                sv[x] = lo4[x];
                sv[4 + x] = hi4[x];
            }
        } else {
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const int tok = tb + 8 * rg + x;
                sv[x] = lrow[tok < t1 ? tok : t1 - 1];
            }
        }
    };
    auto concat_block = [&](int tb, int tb_next, hg_u32x4(&vreg)[4], float(&sv)[8]) __attribute__((always_inline)) {
        // online softmax over the given logits (see the head_dim 128 kernel)
        float sl[8], bm = -INFINITY;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int tok = tb + 8 * rg + x;
            sl[x] = (tok < t1 && n < nh) ? sv[x] * kLog2e : -INFINITY;
            bm = fmaxf(bm, sl[x]);
        }
        if (__builtin_amdgcn_ballot_w64(bm > m_a) != 0) {
            bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
            bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
            const float m_new = fmaxf(m_a, bm);
            const float alpha = fast_exp2(m_a - m_new);
            m_a = m_new;
            l_a *= alpha;
            float *al = reinterpret_cast<float *>(pls);  // (the P staging area is idle in this mode)
            if (rg == 0) al[n] = alpha;
            wave_lds_handover();
            const hg_f4 a4 = *reinterpret_cast<const hg_f4 *>(al + 4 * rg);
#pragma unroll
            for (int nb = 0; nb < 8; ++nb)
#pragma unroll
                for (int r = 0; r < 4; ++r) o[nb][r] *= a4[r];
            wave_lds_handover();
        }
        hg_u32x4 hi_raw, lo_raw;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const float p0 = fast_exp2(sl[2 * jj] - m_a), p1 = fast_exp2(sl[2 * jj + 1] - m_a);
            l_a += p0 + p1;
            uint32_t hi_w, lo_w;
            split_weights<BF16>(p0, p1, hi_w, lo_w);
            hi_raw[jj] = hi_w;
            lo_raw[jj] = lo_w;
        }
        const hg_u32x4 pa_hi = hi_raw, pa_lo = lo_raw;
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
            const hg_u32x4 b = v_operand(vreg, nb);
            o[nb] = mfma_16x16x32<BF16>(pa_hi, b, o[nb]);
            o[nb] = mfma_16x16x32<BF16>(pa_lo, b, o[nb]);
        }
        if (tb_next < t1) {
            load_rows(vbase, tb_next, vreg, pg1);
            load_logits(tb_next, sv);
            if constexpr (PAGED) {
                if (tb_next + kGqaWaves * kGqaBlockTokens < t1) lookup(tb_next + kGqaWaves * kGqaBlockTokens, pg1);
            }
        }
    };

    {
        constexpr int kStride = kGqaWaves * kGqaBlockTokens;
        int tb = t0 + wave * kGqaBlockTokens;
        if constexpr (MODE == kModeStats) {
            hg_u32x4 kreg[4], vreg[4];
            if (tb < t1) {
                if constexpr (PAGED) {
                    lookup(tb, pg3);
                    if (tb + kStride < t1) lookup(tb + kStride, pg1);
                    if (tb + 2 * kStride < t1) lookup(tb + 2 * kStride, pg2);
                }
                load_rows(kbase, tb, kreg, pg3);
                load_rows(vbase, tb, vreg, pg3);
            }
            while (tb < t1) {
                compute_block(tb, tb + kStride, kreg, vreg);
                tb += kStride;
            }
        } else {
            // K only (logits) or V only (concat): four register buffers keep 16 KiB per wave in flight
            // Paged: pg1 always holds the pages of the next block to be loaded; the look-up for the
            // block after it goes out right behind the loads.
            hg_u32x4 r0[4], r1[4], r2[4], r3[4];
            const char *base = MODE == kModeLogits ? kbase : vbase;
            float s0[8], s1[8], s2[8], s3[8];  // concat mode: the logits that go with r0..r3
            auto load_one = [&](int t, hg_u32x4(&reg)[4], float(&sv)[8]) __attribute__((always_inline)) {
                load_rows(base, t, reg, pg1);
                if constexpr (MODE == kModeConcat) load_logits(t, sv);
                if constexpr (PAGED) {
                    if (t + kStride < t1) lookup(t + kStride, pg1);
                }
            };
            if constexpr (PAGED) {
                if (tb < t1) lookup(tb, pg1);
            }
            auto compute_one = [&](int t, hg_u32x4(&reg)[4], float(&sv)[8]) __attribute__((always_inline)) {
                if constexpr (MODE == kModeLogits)
                    compute_block(t, t + 4 * kStride, reg, reg);
                else
                    concat_block(t, t + 4 * kStride, reg, sv);
            };
            if (tb < t1) load_one(tb, r0, s0);
            if (tb + kStride < t1) load_one(tb + kStride, r1, s1);
            if (tb + 2 * kStride < t1) load_one(tb + 2 * kStride, r2, s2);
            if (tb + 3 * kStride < t1) load_one(tb + 3 * kStride, r3, s3);
            while (tb < t1) {
                compute_one(tb, r0, s0);
                tb += kStride;
                if (tb >= t1) break;
                compute_one(tb, r1, s1);
                tb += kStride;
                if (tb >= t1) break;
                compute_one(tb, r2, s2);
                tb += kStride;
                if (tb >= t1) break;
                compute_one(tb, r3, s3);
                tb += kStride;
            }
        }
    }
    if constexpr (MODE == kModeLogits) return;  // nothing to merge or record

    // per-wave state -> LDS (staging areas are dead now), then merge the waves.  Columns n and
    // n ^ 8 hold the even-token and odd-token partial sums of the same channel.
    __syncthreads();
    float(*sm)[kGqaHeads][D + 2] = reinterpret_cast<float(*)[kGqaHeads][D + 2]>(smem);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
            const float both = o[nb][r] + __shfl_xor(o[nb][r], 8, 64);
            if (!odd) sm[wave][4 * rg + r][8 * n + nb] = both;
        }
        if constexpr (MODE != kModeConcat) {
            const float lrow = row16_sum(lsum[r]);
            if (n == 0) {
                sm[wave][4 * rg + r][D] = m[r];
                sm[wave][4 * rg + r][D + 1] = lrow;
            }
        }
    }
    if constexpr (MODE == kModeConcat) {  // maximum and sum of head n sit in the four lanes of that head
        float lt = l_a + __shfl_xor(l_a, 16, 64);
        lt += __shfl_xor(lt, 32, 64);
        if (rg == 0) {
            sm[wave][n][D] = m_a;
            sm[wave][n][D + 1] = lt;
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

}  // namespace hg
