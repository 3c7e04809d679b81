// Streaming kernel for grouped-query attention on the matrix cores (fp16, head_dim 128).
#pragma once

#include "hg_common.hip.h"

namespace hg {

// ---- streaming kernel for grouped-query attention (fp16, head_dim 128) on the matrix cores -----
//
// With G query heads sharing one KV head, every K and V byte feeds G dot products; on the
// vector ALU that makes the scan arithmetic-bound from G = 4 upwards.  Here up to 16 query heads
// of a KV head form the M dimension of v_mfma_f32_16x16x32_f16, so the arithmetic is a few
// percent of the matrix cores and the kernel is bandwidth-bound again.
//
// Per wave and per block of 32 tokens:
//   K   the B operand of MFMA kk is "token per lane": lane l holds token l%16, channels
//       8*(4kk + l/16)..+7 (the contraction runs over channels, and Q is laid out with the same
//       channel grouping as A operand).  Statistics mode on a contiguous cache loads exactly
//       those 16 bytes per lane (a load instruction then covers 16 rows x 64 bytes); the other
//       modes and paged caches take 8 coalesced 16-byte loads per lane (4 whole rows per
//       instruction) -> wave-private LDS (rows padded to 288 bytes) -> read back token per lane.
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
constexpr int kGqaKRow = 288;            // padded LDS row: 256 bytes + 32 (the bank-conflict counter reads zero with it; with + 16 the
                                         // 16-byte reads of 16 rows collided in pairs -- though neither shows in the kernels' times)
constexpr int kGqaKBytes = kGqaBlockTokens * kGqaKRow;
constexpr int kGqaPBytes = kGqaHeads * kGqaBlockTokens * 2;
constexpr int kGqaWaveBytes = kGqaKBytes + 2 * kGqaPBytes;
constexpr int kWaitVmcnt0 = 0x0F70;      // s_waitcnt vmcnt(0) alone (expcnt and lgkmcnt fields at their maxima)
constexpr int kRawBufferFlags = 0x00020000;  // buffer descriptor, last word: raw buffer of 32-bit data
constexpr int kCacheSc1 = 1 << 4;            // buffer load: device-scope coherence (bypass the compute unit's cache)
constexpr int kGqaPublishLead = 2;  // filter mode: blocks between publishing and evaluating the shared bound
// filter mode: blocks after its own evaluation during which a wave still looks for the bounds the
// other waves find (their searches take 8 or 16 rounds, so the waves are up to a block or two apart)
constexpr int kGqaPickupBlocks = 6;
constexpr int kGqaSeedBlocks = 2;   // filter mode: blocks of the seed pass (even: the loop runs them in pairs)
constexpr int kGqaAfterSeed = 3;    // filter mode: first evaluation of the shared bound after a seed pass (block index)
constexpr int kGqaSetsPerHead = 64;  // filter mode: values a workgroup may publish per head (one per lane position and wave)
constexpr int kGqaMaxPeers = 32;         // filter mode: workgroups whose published values a shared bound is taken from
constexpr int kGqaStage = 64;            // filter mode: survivors staged in LDS per (wave, head) between write-outs
// Logits mode: as in the vector kernel, stores that trickle out next to the read stream cost far
// more than their bytes, so the logits are collected in an LDS window (96 KiB laid out
// [valid head][tokens + 4]: the fewer heads, the more tokens it holds) that all four waves write
// out together, between two LDS-only barriers, when it is full; it runs on across the ranges of a
// stream.  With 8 query heads per KV head the window holds 2944 tokens; the logits are then an
// eighth of all bytes moved, and what remains above the bare scan is close to what writing them in
// a phase of their own costs.
constexpr int kGqaRingFloats = 24576;
constexpr int kGqaIterTokens = HG_GQA_WAVES * kGqaBlockTokens;  // tokens of one workgroup iteration

__device__ __forceinline__ void gqa_workgroup_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

typedef _Float16 hg_h8 __attribute__((ext_vector_type(8)));
typedef __bf16 hg_b8 __attribute__((ext_vector_type(8)));
typedef float hg_f4 __attribute__((ext_vector_type(4)));

// D += A . B on the 16x16x32 matrix-core shape; the operands are eight 16-bit values per lane,
// fp16 or bf16 (same layout, same rate).
template <bool BF16>
__device__ __forceinline__ hg_f4 mfma_16x16x32(hg_u32x4 a, hg_u32x4 b, hg_f4 c)
{
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(hg_b8, a), __builtin_bit_cast(hg_b8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(hg_h8, a), __builtin_bit_cast(hg_h8, b), c, 0, 0, 0);
}

// Two softmax weights in [0, 1] as a packed pair of 16-bit heads (hi) and a packed pair of 16-bit
// remainders (lo), p = hi + lo to about 22 bits (fp16) or 16 bits (bf16): two matrix-core passes
// then carry the weights at far better than the precision of the 16-bit V they multiply.
template <bool BF16>
__device__ __forceinline__ void split_weights(float p0, float p1, uint32_t &hi, uint32_t &lo)
{
    if constexpr (BF16) {
        typedef __bf16 b2 __attribute__((ext_vector_type(2)));
        const __bf16 h0 = (__bf16)p0, h1 = (__bf16)p1;
        const __bf16 l0 = (__bf16)(p0 - (float)h0), l1 = (__bf16)(p1 - (float)h1);
        hi = __builtin_bit_cast(uint32_t, b2{h0, h1});
        lo = __builtin_bit_cast(uint32_t, b2{l0, l1});
    } else {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const _Float16 h0 = (_Float16)p0, h1 = (_Float16)p1;
        const _Float16 l0 = (_Float16)(p0 - (float)h0), l1 = (_Float16)(p1 - (float)h1);
        hi = __builtin_bit_cast(uint32_t, h2{h0, h1});
        lo = __builtin_bit_cast(uint32_t, h2{l0, l1});
    }
}

__device__ __forceinline__ float row16_min(float x)
{
    x = fminf(x, dpp_move<0xB1>(x));
    x = fminf(x, dpp_move<0x4E>(x));
    x = fminf(x, dpp_move<0x141>(x));
    x = fminf(x, dpp_move<0x140>(x));
    return x;
}

// Insert x into the descending list a >= b (>= c >= d) of the J = 2 or 4 largest values seen.
// (Separate scalars: an array indexed through a reference stayed in scratch memory.)
template <int J>
__device__ __forceinline__ void track_largest(float &a, float &b, float &c, float &d, float x)
{
    float hi = fmaxf(a, x);
    x = fminf(a, x);
    a = hi;
    hi = fmaxf(b, x);
    x = fminf(b, x);
    b = hi;
    if constexpr (J > 2) {
        hi = fmaxf(c, x);
        x = fminf(c, x);
        c = hi;
        d = fmaxf(d, x);
    }
}

// Sum over the 16 lanes of a DPP row; every lane of the row ends with the total.
__device__ __forceinline__ uint32_t row16_sum_u32(uint32_t x)
{
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x140, 0xf, 0xf, true);
    return x;
}

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

// FJ (filter mode only): logits each lane keeps for the bound, 2 (top_k <= 128) or 4 (top_k <= 256).
// The filter mode keeps more state per lane than 256 registers hold; it is compiled for one wave
// per SIMD (which is how the kernel is launched anyway), so that the rest lives in the accumulation
// registers instead of scratch memory: a scratch access inside the loop would make every wait for
// K rows a wait for all memory operations in flight.
template <int MODE, bool PAGED, bool BF16, int FJ = 2>
__global__ __launch_bounds__(kGqaBlock, kGqaWaves <= 4 && MODE != kModeFilter && MODE != kModeLogits ? 2 : 1) void hg_partial_gqa_kernel(const PartialArgs a)
{
    constexpr int D = 128;
    constexpr int kMergeBytes = kGqaWaves * kGqaHeads * (D + 2) * 4;
    constexpr int kSmemBytes = kGqaWaves * kGqaWaveBytes > kMergeBytes ? kGqaWaves * kGqaWaveBytes : kMergeBytes;
    __shared__ __align__(16) char smem[kSmemBytes];
    // filter mode: per wave and head, the smallest of the 16 lanes' rank-th largest logits
    __shared__ float wmin[MODE == kModeFilter ? kGqaWaves * kGqaHeads : 1];  // own bound: [wave][head]
    // shared bound: every lane's largest logit [wave][head][lane n]; the bounds found [head]
    __shared__ float wpub[MODE == kModeFilter ? kGqaWaves * kGqaHeads * 16 : 1];
    __shared__ float wtau[MODE == kModeFilter ? kGqaHeads : 1];
    static_assert(MODE != kModeFilter || kGqaWaves == 4, "filter mode: wave w evaluates the shared bound of heads 4w .. 4w + 3");
    // filter mode: survivors wait here, per wave and head, until a run of them is written out
    __shared__ float stage_val[MODE == kModeFilter ? kGqaWaves * kGqaHeads * kGqaStage : 1];
    __shared__ int32_t stage_col[MODE == kModeFilter ? kGqaWaves * kGqaHeads * kGqaStage : 1];

    __shared__ __align__(16) float lring[MODE == kModeLogits ? kGqaRingFloats : 1];  // logits mode: the window
    // logits mode: tokens in the window, tokens it holds and floats per head (+ 4: the four row
    // groups of an LDS store then fall on different banks), the index in `logits` of its first
    // token for the chunk's first head (row * ltok + column), the valid heads of its chunk.  Uniform.
    int win_fill = 0, win_tokens = 0, win_stride = 0, win_nh = 0;
    int64_t win_at = 0;
    auto flush_window = [&]() __attribute__((always_inline)) {
        typedef float wf4 __attribute__((ext_vector_type(4)));
        typedef float wf4u __attribute__((ext_vector_type(4), aligned(4)));
        gqa_workgroup_lds_barrier();  // the window is complete
        for (int g = 0; g < win_nh; ++g) {
            float *dst = a.logits + win_at + (int64_t)g * a.ws.ltok;
            for (int c = 4 * (int)threadIdx.x; c < win_fill; c += 4 * kGqaBlock) {
                const wf4 vals = *reinterpret_cast<const wf4 *>(lring + g * win_stride + c);
                if (c + 4 <= win_fill) {
                    const wf4u out = vals;
                    __builtin_nontemporal_store(out, reinterpret_cast<wf4u *>(dst + c));
                } else {
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        if (c + x < win_fill) dst[c + x] = vals[x];
                }
            }
        }
        gqa_workgroup_lds_barrier();  // copied: the window is free again
        win_at += win_fill;
        win_fill = 0;
    };

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: block loop control stays scalar
    const int n = lane & 15, rg = lane >> 4;

    char *kls = smem + wave * kGqaWaveBytes;
    char *pls = kls + kGqaKBytes;

    if constexpr (MODE == kModeFilter) {
        // the selection that follows counts its finished workgroups from zero
        if (blockIdx.x == 0)
            for (int64_t i = threadIdx.x; i < a.n_tail; i += blockDim.x) a.tail_cnt[i] = 0u;
    }
    for_each_segment(a.ws, a.tab, [&](int stream, int r_idx, const RangeEntry &e, int seg_t0, int seg_t1, int seg_col0, int64_t slot) __attribute__((always_inline)) {
    // Tokens [t0, t1) this wave works on and the column of t0: the whole segment, whose 32-token
    // blocks the waves take in turn -- or, in filter mode, the wave's own consecutive sub-span, so
    // that the survivors a wave appends are in ascending column order.
    int t0 = seg_t0, t1 = seg_t1, col0 = seg_col0;
    constexpr int kStride = MODE == kModeFilter ? kGqaBlockTokens : kGqaWaves * kGqaBlockTokens;
    if constexpr (MODE == kModeFilter) {
        const int sub_len = filter_sub_len(seg_t1 - seg_t0, kGqaWaves);
        t0 = min(seg_t0 + wave * sub_len, seg_t1);
        t1 = min(t0 + sub_len, seg_t1);
        col0 = seg_col0 + (t0 - seg_t0);
    }
    const int seq = e.seq;
    const int hk = stream / a.ws.n_chunks;
    const int chunk = stream - hk * a.ws.n_chunks;
    const int g0 = chunk * kGqaHeads;
    const int nh = min(kGqaHeads, a.ws.group - g0);
    const int h0 = hk * a.ws.group + g0;

    if constexpr (MODE == kModeLogits) {
        // does this segment go on where the window ends?  Otherwise the window is written out first.
        const int64_t seg_at = (int64_t)h0 * a.ws.ltok + seg_col0;
        if (win_fill > 0 && (seg_at != win_at + win_fill || nh != win_nh)) flush_window();
        if (win_fill == 0) {
            win_at = seg_at;
            win_nh = nh;
            win_tokens = (kGqaRingFloats / nh - 4) / kGqaIterTokens * kGqaIterTokens;
            win_stride = win_tokens + 4;
        }
    }

    // Q as A operand: lane l holds head l%16, channels 8*(4kk + l/16)..+7 for kk = 0..3
    hg_u32x4 qa[4];
    if constexpr (MODE != kModeConcat) {
        const uint16_t *qrow = static_cast<const uint16_t *>(a.q) + ((int64_t)seq * a.ws.n_q_heads + h0 + (n < nh ? n : 0)) * D;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            hg_u32x4 raw = *reinterpret_cast<const hg_u32x4 *>(qrow + 8 * (4 * kk + rg));
            if (n >= nh) raw = hg_u32x4{0u, 0u, 0u, 0u};
            qa[kk] = raw;
        }
    }

    // concat mode: the logits row of this lane's head n (lrow[tok] is the logit of token tok), and
    // the running maximum and sum of that head, in log2 units, kept in A-operand order (the four
    // lanes of a head hold the same maximum and each its own part of the sum)
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
    const char *kbase = static_cast<const char *>(a.k) + slab * 2 + (PAGED ? n * 16 : 0);
    const char *vbase = static_cast<const char *>(a.v) + slab * 2 + (PAGED ? n * 16 : 0);
    const int64_t row_bytes = a.stride_t * 2;
    const int64_t block_bytes = a.stride_b * 2;
    const uint32_t row_b32 = (uint32_t)row_bytes;
    const uint32_t lane_off = (uint32_t)rg * row_b32 + (uint32_t)n * 16u;  // row rg of a load
    const uint32_t lane_off_cc = (uint32_t)(8 * rg) * row_b32 + (uint32_t)n * 16u;  // concat mode: rows 8rg + j
    const uint32_t last_off = (uint32_t)(t1 - 1 - t0) * row_b32 + (uint32_t)n * 16u;
    const int32_t *table = PAGED ? a.pages.table + (int64_t)seq * a.pages.max_blocks : nullptr;

    // Paged cache: physical blocks of the 8 tokens tb + 4x + rg (x = 0..7) a lane touches in a
    // block; K load i uses x = i, V load j uses x = 4*(j&1) + (j>>1), the same 8 tokens.  In
    // concat mode a lane's V tokens are tb + 8rg + x instead.
    auto lookup = [&](int tb, int(&pg)[8]) __attribute__((always_inline)) {
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int tok = MODE == kModeConcat ? tb + 8 * rg + x : tb + 4 * x + rg;
            pg[x] = table[(tok < t1 ? tok : t1 - 1) >> a.pages.shift];
        }
    };
    auto paged_offset = [&](int tok, int page) __attribute__((always_inline)) -> int64_t {
        tok = tok < t1 ? tok : t1 - 1;  // clamp: never read past the segment
        return paged_row_offset(page, tok, a.pages.mask, (uint32_t)block_bytes, row_b32);
    };
    // row = token of the load relative to the lane's first row of the block (uniform)
    auto flat_offset = [&](int tb, int row, uint32_t lane_part) __attribute__((always_inline)) -> uint32_t {
        const uint32_t off = (uint32_t)(tb - t0 + row) * row_b32 + lane_part;
        return off < last_off ? off : last_off;  // clamp: never read past the segment
    };

    // The 8 K-row loads and the 8 V-row loads of one 32-token block (8 KiB each per wave).
    // Statistics mode on a contiguous cache: a lane's 16-byte load of token n, channel chunk
    // 4 kk + rg IS its B operand of MFMA kk, so K needs no trip through LDS (a load instruction
    // then covers 16 rows x 64 bytes instead of 4 whole rows).  Measured on the 1M-token workload
    // in one GPU session: statistics mode 618 -> 611 us; without the non-temporal hint the same
    // loads lost 10 %.  The K-only modes, which keep two blocks of K in flight, lose with it
    // (logits 442 -> 462 us, filter scan 326 -> 368 us) and keep the LDS path.
    constexpr bool kDirectK = MODE == kModeStats && !PAGED;
    const uint32_t lane_off_d = (uint32_t)n * row_b32 + (uint32_t)rg * 16u;   // direct K: token n of a half, chunk rg of a group of four
    const uint32_t last_row_off = (uint32_t)(t1 - 1 - t0) * row_b32;
    auto load_k = [&](int tb, hg_u32x4(&kreg)[8], const int(&pg)[8]) __attribute__((always_inline)) {
        if constexpr (kDirectK) {
            // every lane fetches its own B operands: token tb + 16 hf + n, channels 8 (4 kk + rg) .. + 7
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int hf = i >> 2, kk = i & 3;
                const uint32_t off = (uint32_t)(tb - t0 + 16 * hf) * row_b32 + lane_off_d + (uint32_t)kk * 64u;
                const uint32_t last = last_row_off + (uint32_t)rg * 16u + (uint32_t)kk * 64u;
                const char *src = kbase + (off < last ? off : last);
                kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const hg_u32x4 *>(src));
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const char *src = PAGED ? kbase + paged_offset(tb + 4 * i + rg, pg[i]) : kbase + flat_offset(tb, 4 * i, lane_off);
            kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const hg_u32x4 *>(src));
        }
    };
    auto load_v = [&](int tb, hg_u32x4(&vreg)[8], const int(&pg)[8]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // token j of lane group rg: interleaved so that S halves pair up (stats mode), or the
            // 8 consecutive tokens whose logits this lane reads (concat mode)
            const int row = 16 * (j & 1) + 4 * (j >> 1);
            const char *src;
            if constexpr (MODE == kModeConcat)
                src = PAGED ? vbase + paged_offset(tb + 8 * rg + j, pg[j]) : vbase + flat_offset(tb, j, lane_off_cc);
            else
                src = PAGED ? vbase + paged_offset(tb + row + rg, pg[4 * (j & 1) + (j >> 1)]) : vbase + flat_offset(tb, row, lane_off);
            vreg[j] = __builtin_nontemporal_load(reinterpret_cast<const hg_u32x4 *>(src));
        }
    };
    // pages of the next block (pg1), the one after (pg2) and the one after that (pg3, in flight);
    // unused when not paged
    int pg1[8] = {0, 0, 0, 0, 0, 0, 0, 0}, pg2[8] = {0, 0, 0, 0, 0, 0, 0, 0}, pg3[8] = {0, 0, 0, 0, 0, 0, 0, 0};

    // Filter mode.  Every lane keeps the largest logits of its own tokens (per head: tokens n and
    // 16 + n of every block of this wave), tj0[r] >= tj1[r] >= ...
    //
    // Own bound.  The smallest, over the 16 lanes of a head and the waves of the workgroup, of the
    // lanes' (rank+1)-th largest is reached by 64 * (rank + 1) >= top_k distinct logits of this
    // segment, so it is a lower bound of the segment's (hence the group's) top_k-th largest logit:
    // nothing below it can be among the kept tokens.
    //
    // Shared bound.  When several workgroups scan the same (range, stream) pair -- a long sequence
    // with few KV heads -- each sees a slice of the group only and its own bound stays far below
    // the group's.  Then every workgroup whose span begins inside the pair publishes, in global
    // memory, sixteen values per head: for every lane position n the largest logit that lane n of
    // any of its waves has seen -- the maxima of sixteen disjoint sets of its tokens.  Among the
    // 16 * P values of P such workgroups the top_k-th largest is reached by top_k distinct logits
    // of the pair, so it is a lower bound of the pair's top_k-th largest logit; it follows the true
    // value closely (the smallest of the values would sit far lower) and closes in on it as the
    // workgroups advance together.  With few such workgroups (up to eight, or fewer than
    // top_k / 8: the sets should be twice top_k) they publish the waves' values separately -- 64
    // disjoint sets per head -- and up to eight of them are read.  Only workgroups whose span begins inside the pair take part:
    // the pair is the first thing they scan, so they are under way from the start of the launch,
    // whereas the workgroup that holds the beginning of the pair reaches it only after it has
    // finished the end of the previous pair.  Nothing ever waits: a value not published yet reads
    // as the lowest key (the host clears the array before the launch), a stale one reads lower
    // than the current one, and either only makes the bound weaker.  Wave w evaluates heads
    // 4w .. 4w + 3 (its 16-lane rows take one head each, every lane the values of its own position
    // n; the count in the bisection runs over the row) and hands the bounds to the other waves
    // through LDS.
    //
    // tau[r] is the bound in use: the largest seen so far of both kinds.
    float tj0[4], tj1[4], tj2[4], tj3[4], tau[4];  // tj0[r] >= tj1[r] >= ...: largest logits of head 4rg + r
    uint32_t cnt[4] = {0u, 0u, 0u, 0u};
    int blk = 0, next_refresh = 1;
    bool published = false;       // shared bound: this round's values are out
    bool seeded = false;          // a seed pass has run: sparser schedule
    bool seed = false;            // seed pass: nothing is appended
    int pickup = 0;               // blocks during which the other waves' new bounds are still picked up
    uint32_t staged[4] = {0u, 0u, 0u, 0u};  // survivors of heads 4rg..4rg+3 waiting in LDS (cnt: already written out)
    uint32_t tw_last = 0u;        // shared bound: the 16-bit key the last evaluation found for this row's head
    int n_peers = 0;              // shared bound: workgroups that take part (0: none, own bound only)
    bool per_wave = false;        // they publish 64 values per head (every wave's lanes) rather than 16
    bool takes_part = false;      // this workgroup is one of them
    int64_t gb_first = 0;         // slot of the first of them
    if constexpr (MODE == kModeFilter) {
        const int pre_r = e.pre, pre_n = table_entry(a.tab, r_idx + 1).pre;
        const int64_t p_first = (int64_t)stream * a.ws.ltok + pre_r, p_last = (int64_t)stream * a.ws.ltok + pre_n - 1;
        // the workgroups whose span begins inside the pair: this pair is the first thing they scan
        const int64_t w_first = (p_first + a.ws.span - 1) / a.ws.span, w_last = p_last / a.ws.span;
        const int64_t n_inner = w_last - w_first + 1;
        if (n_inner > 0 && filter_valid_waves(a.ws.span, kGqaWaves) == kGqaWaves) {
            const int many = n_inner < kGqaMaxPeers ? (int)n_inner : kGqaMaxPeers;
            const int few = n_inner < kGqaMaxPeers / kGqaWaves ? (int)n_inner : kGqaMaxPeers / kGqaWaves;
            // (the top_k-th largest of S set maxima is about the -S ln(1 - top_k / S)-th largest
            // logit of the tokens they cover: S = top_k would give the smallest maximum)
            if (many > few && many * 16 >= 2 * a.filter_k) {
                n_peers = many;
            } else if (few * 16 * kGqaWaves * 3 >= 4 * a.filter_k) {
                n_peers = few;
                per_wave = true;
            }
            gb_first = w_first + (int64_t)stream * a.tab.n_ranges + r_idx;
        }
        takes_part = n_peers > 0 && (int64_t)blockIdx.x >= w_first && (int64_t)blockIdx.x < w_first + n_peers;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            tau[r] = 4 * rg + r < nh ? -INFINITY : INFINITY;  // rows of the tile beyond the group's heads pass nothing
            tj0[r] = tj1[r] = tj2[r] = tj3[r] = -INFINITY;
        }
        if (lane < kGqaHeads) {
            lds_publish(&wmin[wave * kGqaHeads + lane], -INFINITY);
            if (wave == 0) lds_publish(&wtau[lane], -INFINITY);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) lds_publish(&wpub[(wave * kGqaHeads + 4 * rg + r) * 16 + n], -INFINITY);
        __syncthreads();
    }

    // Write the staged survivors of every head of this wave behind those already written out.
    auto flush_staged = [&]() __attribute__((always_inline)) {
        wave_lds_handover();
        const int64_t ltok_here = a.ws.ltok;
#pragma unroll
        for (int hh = 0; hh < kGqaHeads; ++hh) {
            // head hh is held by row group hh / 4 as its entry hh % 4; lane 16 * (hh / 4) speaks for the group
            const int c = __builtin_amdgcn_readlane((int)staged[hh & 3], 16 * (hh >> 2));
            if (c == 0) continue;
            const int done = __builtin_amdgcn_readlane((int)cnt[hh & 3], 16 * (hh >> 2));
            const int64_t dst = (int64_t)(h0 + hh) * ltok_here + col0 + done;
            const int src = (wave * kGqaHeads + hh) * kGqaStage;
            if (lane < c) {
                a.surv_val[dst + lane] = stage_val[src + lane];
                a.surv_col[dst + lane] = stage_col[src + lane];
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            cnt[r] += staged[r];
            staged[r] = 0u;
        }
        // Let the stores retire here, on the rare path.  While a store may be in flight the
        // compiler has to treat the loads' completion order as unknown and waits for ALL of them
        // before it touches a K row, which would undo the two register buffers.
        __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
        wave_lds_handover();
    };

    // Shared bound, first half: request the peers' values of the head this 16-lane row evaluates
    // (head 4 * wave + rg, this lane's position n).  Buffer loads that go to the device-wide cache
    // (sc1), not atomic loads: those complete one by one, these are all in flight together.  The
    // buffer is the peers' part of the array; beyond it a load returns 0.
    auto request_peer_values = [&](uint32_t(&key)[kGqaMaxPeers]) __attribute__((always_inline)) {
        if constexpr (MODE == kModeFilter) {
            uint32_t *gb = a.gbound;
            const int hh = 4 * wave + rg;
            const uint64_t peers_at = reinterpret_cast<uint64_t>(gb + gb_first * (kGqaHeads * kGqaSetsPerHead));
            const uint64_t peers_uni = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(peers_at >> 32)) << 32) |
                                       (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)peers_at);
            const __amdgpu_buffer_rsrc_t peers = __builtin_amdgcn_make_buffer_rsrc(
                reinterpret_cast<void *>(peers_uni), 0, __builtin_amdgcn_readfirstlane(n_peers) * (kGqaHeads * kGqaSetsPerHead * 4), kRawBufferFlags);
#pragma unroll
            for (int j = 0; j < kGqaMaxPeers; ++j) {
                // one value of each of up to 32 peers, or four (the waves') of each of up to 8
                const int one = (j * kGqaHeads + hh) * kGqaSetsPerHead + n;
                const int four = ((j / kGqaWaves) * kGqaHeads + hh) * kGqaSetsPerHead + (j % kGqaWaves) * 16 + n;
                key[j] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(peers, (per_wave ? four : one) * 4, 0, kCacheSc1);
            }
        }
    };
    // Second half: the largest 16-bit key that top_k of the row's values reach becomes the head's
    // bound; the other waves pick it up from LDS during the next blocks.
    auto evaluate_peer_values = [&](uint32_t(&key)[kGqaMaxPeers]) __attribute__((always_inline)) {
        if constexpr (MODE == kModeFilter) {
            const int hh = 4 * wave + rg;
#pragma unroll
            for (int j = 0; j < kGqaMaxPeers; ++j) key[j] >>= 16;
            // The published values only rise, so the key sought is at or above the last one found.
            // If fewer than top_k values reach the next binade (the low 7 bits of a 16-bit key are
            // mantissa), it also shares the last key's sign and exponent and only those 7 bits are
            // searched: 8 counting rounds instead of 16, if that holds for all four heads of the wave.
            uint32_t tw = 0u;
            int first_bit = 15;
            {
                const uint32_t next_binade = (tw_last | 0x7fu) + 1u;
                uint32_t reach = 0;
#pragma unroll
                for (int p = 0; p < kGqaMaxPeers; ++p) reach += key[p] >= next_binade ? 1u : 0u;
                reach = row16_sum_u32(reach);
                // (a row without a head never votes for the short search: a wave of such rows alone
                // would always take it and run ahead of the waves whose bounds it has to pick up,
                // which was measured to let 60 % more through)
                const bool same = tw_last != 0u && reach < (uint32_t)a.filter_k;
                if (__builtin_amdgcn_ballot_w64(!same) == 0) {
                    tw = tw_last & ~0x7fu;
                    first_bit = 6;
                }
            }
#pragma unroll 1
            for (int b = first_bit; b >= 0; --b) {
                const uint32_t c = tw | (1u << b);
                uint32_t reach = 0;
#pragma unroll
                for (int p = 0; p < kGqaMaxPeers; ++p) reach += key[p] >= c ? 1u : 0u;
                reach = row16_sum_u32(reach);
                if (reach >= (uint32_t)a.filter_k) tw = c;
            }
            tw_last = tw;
            tw <<= 16;
            if (n == 0 && hh < nh) lds_publish(&wtau[hh], tw > order_key(-INFINITY) ? key_to_float(tw) : -INFINITY);
            // bounds of this lane's own heads: this wave's are current, the others' as of
            // their last refresh
#pragma unroll
            for (int r = 0; r < 4; ++r) tau[r] = fmaxf(tau[r], lds_peek(&wtau[4 * rg + r]));
        }
    };

    // One block.  Software pipeline with a single register buffer: the K rows of the next block
    // are requested as soon as this block's K sits in LDS, its V rows as soon as this block's V
    // has been consumed, so a wave always has 8-16 KiB in flight while it computes.
    auto compute_block = [&](int tb, int tb_next, hg_u32x4(&kreg)[8], hg_u32x4(&vreg)[8]) __attribute__((always_inline)) {
        // K: registers -> LDS (row per token) -> B operands (token per lane)
        if constexpr (!kDirectK) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                *reinterpret_cast<hg_u32x4 *>(kls + (4 * i + rg) * kGqaKRow + n * 16) = kreg[i];
            wave_lds_handover();
        }
        if constexpr (PAGED && MODE == kModeStats) {
            // Pages three blocks ahead, requested before this block's loads: the registers are not
            // touched again until the rotation at the end of the block, a whole block later, so the
            // wave never stands waiting for a table entry (with a shorter look-ahead it did, once
            // per block, for a full memory latency).
            const int tb_3 = tb + 3 * (tb_next - tb);
            if (tb_3 < t1) lookup(tb_3, pg3);
        }
        // K-only modes on a contiguous cache request the rows of the block after next
        // unconditionally (past the end the clamped offsets re-read the segment's last row, at
        // most two blocks' worth per segment): with a conditional request the number of loads in
        // flight is unknown at compile time, the wait for this block's rows becomes a wait for all
        // loads, and the second register buffer buys nothing.
        constexpr bool kAlwaysAhead = !PAGED && (MODE == kModeLogits || MODE == kModeFilter);
        if (!kDirectK && (kAlwaysAhead || tb_next < t1)) {
            load_k(tb_next, kreg, pg1);
            if constexpr (PAGED && (MODE == kModeLogits || MODE == kModeFilter)) {  // blocks are loaded in order: pages of the one after
                if (tb_next + kStride < t1) lookup(tb_next + kStride, pg1);
            }
        }
        hg_f4 s[2];
        if constexpr (MODE == kModeFilter) {
            // all eight LDS reads first, then the products: with every register in use the compiler
            // otherwise sends each read and its product through one register quad, eight LDS round
            // trips in a row
            hg_u32x4 kf[2][4];
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    kf[hf][kk] = *reinterpret_cast<const hg_u32x4 *>(kls + (16 * hf + n) * kGqaKRow + (4 * kk + rg) * 16);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                s[hf] = hg_f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) s[hf] = mfma_16x16x32<BF16>(qa[kk], kf[hf][kk], s[hf]);
            }
        } else {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                s[hf] = hg_f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    hg_u32x4 raw;
                    if constexpr (kDirectK)
                        raw = kreg[4 * hf + kk];
                    else
                        raw = *reinterpret_cast<const hg_u32x4 *>(kls + (16 * hf + n) * kGqaKRow + (4 * kk + rg) * 16);
                    s[hf] = mfma_16x16x32<BF16>(qa[kk], raw, s[hf]);
                }
            }
            if constexpr (kDirectK) {
                if (kAlwaysAhead || tb_next < t1) load_k(tb_next, kreg, pg1);  // the operands are consumed: request the next rows
            }
        }

        if constexpr (MODE == kModeLogits) {
            // export: lane (n, rg) holds heads 4rg..4rg+3 of tokens tb + n and tb + 16 + n; they go
            // to the window at the tokens' places.  (A block past the segment's end, which the paired
            // loop may run, takes no part; every wave makes the same decision for the same
            // workgroup iteration.)
            if (tb < t1) {
                if (win_fill + kGqaIterTokens > win_tokens) flush_window();
                float *buf = lring + win_fill + wave * kGqaBlockTokens + n;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (4 * rg + r < nh) {
                        buf[(4 * rg + r) * win_stride] = s[0][r] * a.qscale;
                        buf[(4 * rg + r) * win_stride + 16] = s[1][r] * a.qscale;
                    }
                }
                win_fill += kGqaIterTokens;
            }
            wave_lds_handover();  // the next block overwrites the K staging area
            return;
        }
        if constexpr (MODE == kModeFilter) {
            // lane (n, rg): logits of heads 4rg..4rg+3 for tokens tb + n and tb + 16 + n, the same
            // values the logits mode exports
            // Common case first, on the vector ALU alone: a full block in which no logit reaches its
            // head's bound (heads beyond the group carry a bound of +inf).  Only then are the exact
            // per-token conditions formed.
            const bool ok0 = tb + n < t1, ok1 = tb + 16 + n < t1;
            float v0[4], v1[4], excess = -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                v0[r] = s[0][r] * a.qscale;
                v1[r] = s[1][r] * a.qscale;
            }
            if (tb + kGqaBlockTokens > t1) {  // last block of the sub-span: tokens past its end count for nothing
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    v0[r] = ok0 ? v0[r] : -INFINITY;
                    v1[r] = ok1 ? v1[r] : -INFINITY;
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) excess = fmaxf(excess, fmaxf(v0[r] - tau[r], v1[r] - tau[r]));  // (fmaxf drops a NaN from -inf - -inf)
            const bool any = excess >= 0.f;
            bool c0[4], c1[4];
            // Survivors go to LDS first, in column order (tokens tb + 0..15, then tb + 16..31; the 16
            // lanes of row group rg are the tokens of heads 4rg..4rg+3), and reach global memory in
            // runs.  A conditional global store in every block would leave the number of memory
            // operations in flight unknown at compile time, and the wait for the next block's K rows
            // would then also wait for the rows requested for the block after it.
            if (__builtin_amdgcn_ballot_w64(any) && !seed) {
                const uint32_t below = (1u << n) - 1u;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const bool head_ok = 4 * rg + r < nh;
                    c0[r] = ok0 && head_ok && v0[r] >= tau[r];
                    c1[r] = ok1 && head_ok && v1[r] >= tau[r];
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint64_t b0 = __builtin_amdgcn_ballot_w64(c0[r]), b1 = __builtin_amdgcn_ballot_w64(c1[r]);
                    if ((b0 | b1) == 0) continue;  // uniform: usually only a few of the 16 heads have a survivor
                    const uint32_t m0 = (uint32_t)(b0 >> (16 * rg)) & 0xffffu;
                    const uint32_t m1 = (uint32_t)(b1 >> (16 * rg)) & 0xffffu;
                    const uint32_t n0 = (uint32_t)__builtin_popcount(m0);
                    const int base = (wave * kGqaHeads + 4 * rg + r) * kGqaStage;
                    if (c0[r]) {
                        const int at = base + (int)(staged[r] + (uint32_t)__builtin_popcount(m0 & below));
                        stage_val[at] = v0[r];
                        stage_col[at] = col0 + (tb - t0) + n;
                    }
                    if (c1[r]) {
                        const int at = base + (int)(staged[r] + n0 + (uint32_t)__builtin_popcount(m1 & below));
                        stage_val[at] = v1[r];
                        stage_col[at] = col0 + (tb - t0) + 16 + n;
                    }
                    staged[r] += n0 + (uint32_t)__builtin_popcount(m1);
                }
                // a block adds at most 32 per head: write out once a head could overflow next time
                bool full = false;
#pragma unroll
                for (int r = 0; r < 4; ++r) full = full || staged[r] > (uint32_t)(kGqaStage - kGqaBlockTokens);
                if (__builtin_amdgcn_ballot_w64(full)) flush_staged();
            }
            const int rank = a.filter_rank;  // uniform, < FJ
            if (n_peers > 0) {  // the shared bound needs every lane's largest logit only
#pragma unroll
                for (int r = 0; r < 4; ++r) tj0[r] = fmaxf(tj0[r], fmaxf(v0[r], v1[r]));
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    track_largest<FJ>(tj0[r], tj1[r], tj2[r], tj3[r], v0[r]);
                    track_largest<FJ>(tj0[r], tj1[r], tj2[r], tj3[r], v1[r]);
                }
            }
            // The bound is refreshed after blocks 2, 4, 9, 22, 54, ... (own bound) or, behind a seed
            // pass, 4, 11, 32, 95, ... (shared bound): it settles like the logarithm of the tokens
            // seen, and a refresh of the shared bound costs a round trip to memory plus the search --
            // about as much as four blocks.
            // Shared bound: a workgroup publishes kGqaPublishLead blocks before it evaluates, so
            // that what it reads from peers that run a little behind it is of this round too.
            if (n_peers > 0 && blk + (seed ? 1 : kGqaPublishLead) >= next_refresh && !published) {
                published = true;
                uint32_t *gb = a.gbound;
                // this lane's largest logits -> LDS; then this row's head: lane n, all waves
#pragma unroll
                for (int r = 0; r < 4; ++r) lds_publish(&wpub[(wave * kGqaHeads + 4 * rg + r) * 16 + n], tj0[r]);
                const int hh = 4 * wave + rg;  // the head this 16-lane row evaluates
                // (a wave's own LDS operations complete in order; what the other waves have
                // written may be older, i.e. lower)
                float mine = lds_peek(&wpub[hh * 16 + n]);
#pragma unroll
                for (int w = 1; w < kGqaWaves; ++w) mine = fmaxf(mine, lds_peek(&wpub[(w * kGqaHeads + hh) * 16 + n]));
                // published as order-preserving keys: 0, the cleared state, is below every logit
                if (takes_part && !per_wave && hh < nh && mine > -INFINITY) {
                    __hip_atomic_store(gb + (slot * kGqaHeads + hh) * kGqaSetsPerHead + n, order_key(mine), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
                if (takes_part && per_wave) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (4 * rg + r < nh && tj0[r] > -INFINITY)
                            __hip_atomic_store(gb + (slot * kGqaHeads + 4 * rg + r) * kGqaSetsPerHead + wave * 16 + n, order_key(tj0[r]),
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
            // (the waves evaluate at about the same time: what the others have found for their
            // heads is picked up during the blocks that follow)
            if (pickup > 0) {
                --pickup;
#pragma unroll
                for (int r = 0; r < 4; ++r) tau[r] = fmaxf(tau[r], lds_peek(&wtau[4 * rg + r]));
            }
            if (blk == next_refresh) {
                next_refresh = seeded ? next_refresh * 3 + 1 : next_refresh * 5 / 2 + 1;
                published = false;
                if (n_peers > 0) {
                    pickup = kGqaPickupBlocks;
                    uint32_t key[kGqaMaxPeers];
                    request_peer_values(key);
                    evaluate_peer_values(key);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float mine = rank == 0 ? tj0[r] : tj1[r];
                        if constexpr (FJ > 2) mine = rank == 2 ? tj2[r] : rank == 3 ? tj3[r] : mine;
                        const float low = row16_min(mine);
                        if (n == 0) lds_publish(&wmin[wave * kGqaHeads + 4 * rg + r], low);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float t = lds_peek(&wmin[4 * rg + r]);
#pragma unroll
                        for (int w = 1; w < kGqaWaves; ++w) t = fminf(t, lds_peek(&wmin[w * kGqaHeads + 4 * rg + r]));
                        tau[r] = fmaxf(tau[r], t);
                    }
                }
            }
            ++blk;
            wave_lds_handover();  // the next block overwrites the K staging area
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
        uint32_t ph[4], pl[4];  // packed (half 0, half 1) weights: fp16 head and fp16 remainder
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p0 = fast_exp2(e0[r]), p1 = fast_exp2(e1[r]);
            lsum[r] += p0 + p1;
            split_weights<BF16>(p0, p1, ph[r], pl[r]);
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
        const hg_u32x4 pa_hi = *reinterpret_cast<const hg_u32x4 *>(pls + n * 64 + rg * 16);
        const hg_u32x4 pa_lo = *reinterpret_cast<const hg_u32x4 *>(pls + kGqaPBytes + n * 64 + rg * 16);

        // V: in-lane transpose of halves, then O[nb] = alpha * O[nb] + P . V[:, channel 8n + nb]
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
            const uint32_t sel = (nb & 1) ? 0x07060302u : 0x05040100u;
            hg_u32x4 braw;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                braw[jj] = __builtin_amdgcn_perm(vreg[2 * jj + 1][nb >> 1], vreg[2 * jj][nb >> 1], sel);
            const hg_u32x4 b = braw;
            o[nb] = mfma_16x16x32<BF16>(pa_hi, b, o[nb]);
            o[nb] = mfma_16x16x32<BF16>(pa_lo, b, o[nb]);
        }
        if (tb_next < t1) {
            load_v(tb_next, vreg, pg1);
            if constexpr (PAGED) {
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    pg1[x] = pg2[x];
                    pg2[x] = pg3[x];
                }
            }
        }
        wave_lds_handover();  // the next block overwrites the K and P staging areas
    };

    // Concat mode block: the given logits come straight from memory in A-operand order (lane: head
    // n, tokens tb + 8rg .. + 7) and take the place of q.k in an online softmax; the weights lie in
    // (0, 1], so the fp16 head + remainder keeps them to ~22 bits.  The records of all segments of a
    // group are merged exactly by the reduce kernel: the one softmax over the concatenated logits.
    // The 8 logits a lane needs for block tb are requested with the V rows of that block: two
    // 16-byte loads when the block is full (they need 4-byte alignment only), clamped single loads
    // in the last block of a segment.  The branch is wave-uniform, so neither side has to wait for
    // its loads before the join.
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
    auto concat_block = [&](int tb, int tb_next, hg_u32x4(&vreg)[8], float(&sv)[8]) __attribute__((always_inline)) {
        // online softmax over the given logits, as in the statistics mode over q.k: a new maximum of
        // some head (rare after the first blocks; a wave-uniform branch) rescales that head's sum and,
        // through 64 bytes of LDS, its accumulators, which live in the lanes of the result tile
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
            const uint32_t sel = (nb & 1) ? 0x07060302u : 0x05040100u;
            hg_u32x4 braw;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                braw[jj] = __builtin_amdgcn_perm(vreg[2 * jj + 1][nb >> 1], vreg[2 * jj][nb >> 1], sel);
            const hg_u32x4 b = braw;
            o[nb] = mfma_16x16x32<BF16>(pa_hi, b, o[nb]);
            o[nb] = mfma_16x16x32<BF16>(pa_lo, b, o[nb]);
        }
        if (tb_next < t1) {
            load_v(tb_next, vreg, pg1);
            load_logits(tb_next, sv);
            if constexpr (PAGED) {
                if (tb_next + kStride < t1) lookup(tb_next + kStride, pg1);
            }
        }
    };

    {
        int tb = MODE == kModeFilter ? t0 : t0 + wave * kGqaBlockTokens;
        if constexpr (MODE == kModeStats) {
            hg_u32x4 kreg[8], vreg[8];
            if (tb < t1) {
                if constexpr (PAGED) {
                    lookup(tb, pg3);
                    if (tb + kStride < t1) lookup(tb + kStride, pg1);
                    if (tb + 2 * kStride < t1) lookup(tb + 2 * kStride, pg2);
                }
                load_k(tb, kreg, pg3);
                load_v(tb, vreg, pg3);
            }
            while (tb < t1) {
                compute_block(tb, tb + kStride, kreg, vreg);
                tb += kStride;
            }
        } else {
            // Only K (logits) or only V (concat) is read: two register buffers, so that two
            // blocks (16 KiB per wave) are in flight as in the statistics mode.
            // Paged: pg1 always holds the pages of the next block to be loaded; the look-up for the
            // block after it goes out right behind the loads and has one block of compute to land.
            hg_u32x4 ra[8], rb[8];
            float sa[8], sb[8];  // concat mode: the logits that go with ra, rb
            auto load_one = [&](int t, hg_u32x4(&reg)[8], float(&sv)[8]) __attribute__((always_inline)) {
                if constexpr (MODE != kModeConcat) {
                    load_k(t, reg, pg1);
                } else {
                    load_v(t, reg, pg1);
                    load_logits(t, sv);
                }
                if constexpr (PAGED) {
                    if (t + kStride < t1) lookup(t + kStride, pg1);
                }
            };
            int seed_tok = 0;  // filter mode, seed pass on a contiguous cache: the tokens it walks over
            auto compute_one = [&](int t, hg_u32x4(&reg)[8], float(&sv)[8]) __attribute__((always_inline)) {
                if constexpr (MODE != kModeConcat) {
                    // (the seed pass ends by requesting its first two blocks again, for the scan proper)
                    int ahead = t + 2 * kStride;
                    if (MODE == kModeFilter && !PAGED && ahead >= t0 + seed_tok) ahead -= seed_tok;
                    compute_block(t, ahead, reg, reg);
                } else {
                    concat_block(t, t + 2 * kStride, reg, sv);
                }
            };
            constexpr bool kAlwaysAhead = !PAGED && (MODE == kModeLogits || MODE == kModeFilter);
            // Filter mode with a shared bound: the first blocks are scanned twice.  Until a bound
            // exists everything would pass, and two blocks of every wave are already one percent
            // of a long sequence -- several times what passes afterwards.  So the seed pass only
            // looks (largest logits, published and evaluated as usual) and the scan proper then
            // starts again at the first block with the bound that the workgroups have found by then.
            if constexpr (MODE == kModeFilter) {
                seed = n_peers > 0 && kGqaSeedBlocks > 0;
                if (seed) next_refresh = kGqaSeedBlocks - 1;
            }
            bool primed = false;
            for (;;) {
                const int t_end = seed ? min(t1, t0 + kGqaSeedBlocks * kStride) : t1;
                // (the loop runs whole pairs of blocks)
                seed_tok = seed && t_end > t0 ? (t_end - t0 + 2 * kStride - 1) / (2 * kStride) * (2 * kStride) : 0;
                if (!primed) {
                    if constexpr (PAGED) {
                        if (tb < t1) lookup(tb, pg1);
                    }
                    if (tb < t1) {
                        load_one(tb, ra, sa);
                        if (kAlwaysAhead || tb + kStride < t1) load_one(tb + kStride, rb, sb);
                    }
                }
                while (tb < t_end) {
                    compute_one(tb, ra, sa);
                    tb += kStride;
                    // (the K-only modes on a contiguous cache run the second block of the pair even past
                    // the end -- all its tokens are then masked -- so that the loop body is one straight line: with the
                    // exit in the middle the compiler no longer knew how many loads are in flight at
                    // the top of the loop and waited there for all of them)
                    if (!kAlwaysAhead && tb >= t_end) break;
                    compute_one(tb, rb, sb);
                    tb += kStride;
                }
                if (!seed) break;
                seed = false;
                primed = !PAGED;
                tb = t0;
                blk = 0;
                next_refresh = kGqaAfterSeed;
                seeded = true;
                published = false;
            }
        }
    }
    if constexpr (MODE == kModeLogits) {
        // A wave without tokens in the segment's last workgroup iteration still takes that
        // iteration's step, so that all waves agree on the window; then the part of the last
        // iteration beyond the segment's end is given back.
        const int n_tok = seg_t1 - seg_t0;
        const int n_iters = (n_tok + kGqaIterTokens - 1) / kGqaIterTokens;
        const int mine = n_tok > wave * kGqaBlockTokens ? (n_tok - wave * kGqaBlockTokens + kGqaIterTokens - 1) / kGqaIterTokens : 0;
        if (mine < n_iters) {
            if (win_fill + kGqaIterTokens > win_tokens) flush_window();
            win_fill += kGqaIterTokens;
        }
        win_fill -= n_iters * kGqaIterTokens - n_tok;
        return;  // nothing to merge or record
    }
    if constexpr (MODE == kModeFilter) {
        flush_staged();
        if (n == 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) a.surv_cnt[(slot * kGqaWaves + wave) * kGqaHeads + 4 * rg + r] = (int32_t)cnt[r];
        }
        __syncthreads();  // the next segment resets the published bounds
        return;
    }

    // per-wave state -> LDS (staging areas are dead now), then merge the four waves
    __syncthreads();
    float(*sm)[kGqaHeads][D + 2] = reinterpret_cast<float(*)[kGqaHeads][D + 2]>(smem);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) sm[wave][4 * rg + r][8 * n + nb] = o[nb][r];
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
    if constexpr (MODE == kModeLogits) {
        if (win_fill > 0) flush_window();
    }
}

}  // namespace hg
