// Host side of the C ABI declared in include/hg_attn.h: validation, work-split planning, launches.
// Nothing here allocates device memory or synchronises with the device; host tables reach the
// GPU inside kernel arguments (small tables) or through chunked upload kernels (large tables),
// so no memcpy semantics are relied upon and every call is safe to record into a HIP graph.

#include "hg_combine.hip.h"
#include "hg_common.hip.h"
#include "hg_gather.hip.h"
#include "hg_select.hip.h"
#include "hg_stream_gqa.hip.h"
#include "hg_stream_gqa64.hip.h"
#include "hg_stream_valu.hip.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <tuple>
#include <type_traits>
#include <utility>
#include <vector>

#include "../../include/hg_attn.h"
#include "../../include/hg_attn_debug.h"

// Scratch of hg_attn_partial_static: part of the device image, so every GPU the library runs on
// holds its own copy at its own address.  Host code never uses this name as an address: it looks
// the address up once per device (static_scratch below) and passes that pointer on.
static __device__ __align__(256) unsigned char scratch[HG_ATTN_STATIC_SCRATCH_BYTES];

namespace {

using namespace hg;

int g_forced_span_tokens = 0;
int g_topk_mode = 0;  // hg_attn_set_topk_mode: 0 = choose, 1 = filter scan wherever it exists, 2 = never, 3 = as 1 with the staged selection behind it

// Optional timing of the streaming kernel alone: event pairs recorded on the caller's stream
// right around its launch (hg_attn_profile_start / hg_attn_profile_stop).
std::vector<hipEvent_t> g_prof_events;  // 2 per slot
int g_prof_used = 0;
int g_prof_repeat = 1;  // launches of the streaming kernel between the two events of a slot

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Launches go through hipLaunchKernel, whose return value is this launch's own status.  The first
// failure of a call is kept per thread and reported by launch_status(); the runtime's "last
// error" is never consulted, so an error that the caller's earlier HIP calls left behind is not
// taken for one of this library's launches (and is not cleared either).
thread_local hipError_t t_launch_error = hipSuccess;

template <typename... KArgs, typename... Args>
void launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream, Args &&...args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<std::remove_cv_t<KArgs>...> vals(std::forward<Args>(args)...);
    void *argv[sizeof...(KArgs)];
    std::apply([&](auto &...v) { int i = 0; ((argv[i++] = static_cast<void *>(&v)), ...); }, vals);
    const hipError_t err = hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, argv, 0, stream);
    if (err != hipSuccess && t_launch_error == hipSuccess) t_launch_error = err;
}
#define HG_LAUNCH(kernel, grid, block, stream, ...) launch_kernel(kernel, grid, block, stream, __VA_ARGS__)

struct Plan {
    WorkSplit ws{};
    int64_t n_workgroups = 0;
    int64_t n_slots = 0;              // segment records: n_workgroups + n_streams * n_ranges
    std::vector<RangeEntry> entries;  // n_ranges + 1 (sentinel)
    // workspace sections (byte offsets)
    size_t off_m = 0, off_l = 0, off_o = 0, off_tab = 0, total = 0;
    size_t off_groups = 0;  // concat path only
};

constexpr int kMaxDevices = 64;

// The current HIP device, or -1 when none can be queried (a host without a GPU).  Queries that
// fail here are this library's own and leave nothing behind.
int current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return -1;
    }
    return dev;
}

// Compute units of the current device (256 on MI355X), looked up once per device; 256 when no
// device can be queried, so that planning also works on a host without a GPU.
int compute_units()
{
    static std::mutex mu;
    static int cached[kMaxDevices] = {};
    const int dev = current_device();
    if (dev < 0) return 256;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev]) return cached[dev];
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
        (void)hipGetLastError();
        return 256;
    }
    cached[dev] = cus;
    return cus;
}

// Device address of `scratch` on the current device, looked up on the first call per device.
hg_status static_scratch(void **ptr)
{
    static std::mutex mu;
    static void *per_device[kMaxDevices] = {};
    const int dev = current_device();
    if (dev < 0) {
        std::fprintf(stderr, "hg_attn: no current HIP device\n");
        return HG_ERR_LAUNCH;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void *p = nullptr;
        const hipError_t err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !p) {
            std::fprintf(stderr, "hg_attn: address of the static scratch buffer on device %d: %s\n", dev, hipGetErrorString(err));
            return HG_ERR_LAUNCH;
        }
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    return HG_OK;
}

hg_status check_desc(const hg_attn_desc *d)
{
    if (!d) return HG_ERR_NULL;
    if (d->dtype != HG_F16 && d->dtype != HG_F32 && d->dtype != HG_BF16) return HG_ERR_DTYPE;
    if (d->batch < 0 || d->n_q_heads <= 0 || d->n_q_heads > 65535 || d->n_kv_heads <= 0) return HG_ERR_SHAPE;
    if (d->n_q_heads % d->n_kv_heads) return HG_ERR_SHAPE;
    if (d->head_dim != 64 && d->head_dim != 128) return HG_ERR_SHAPE;
    if (d->batch == 0) return HG_OK;
    if (!d->q || !d->k || !d->v || !d->seq_lens) return HG_ERR_NULL;
    const int64_t es = d->dtype == HG_F32 ? 4 : 2;
    if (d->stride_t < d->head_dim || d->stride_b < 0 || d->stride_h < 0) return HG_ERR_SHAPE;
    if ((d->stride_t * es) % 16 || (d->stride_b * es) % 16 || (d->stride_h * es) % 16) return HG_ERR_SHAPE;
    if (((uintptr_t)d->q | (uintptr_t)d->k | (uintptr_t)d->v) % 16) return HG_ERR_SHAPE;
    if (!std::isfinite(d->scale)) return HG_ERR_SHAPE;
    for (int32_t b = 0; b < d->batch; ++b)
        if (d->seq_lens[b] < 0) return HG_ERR_RANGE;
    if (d->block_table) {
        const int32_t bt = d->block_tokens;
        if (bt < 16 || bt > 65536 || (bt & (bt - 1))) return HG_ERR_SHAPE;
        if (d->max_blocks < 1) return HG_ERR_SHAPE;
        // the kernels form paged addresses with a 32-bit block stride and a 24-bit row stride
        if (d->stride_b * es >= (int64_t)1 << 32 || d->stride_t * es >= (int64_t)1 << 24) return HG_ERR_SHAPE;
        for (int32_t b = 0; b < d->batch; ++b)
            if (((int64_t)d->seq_lens[b] + bt - 1) / bt > d->max_blocks) return HG_ERR_RANGE;
    }
    return HG_OK;
}

hg_status check_ranges(const hg_attn_desc *d, const hg_range *ranges, int32_t n_ranges)
{
    if (n_ranges < 0) return HG_ERR_SHAPE;
    if (n_ranges && !ranges) return HG_ERR_NULL;
    for (int32_t r = 0; r < n_ranges; ++r) {
        const hg_range &g = ranges[r];
        if (g.seq < 0 || g.seq >= d->batch) return HG_ERR_RANGE;
        if (g.begin < 0 || g.begin > g.end || g.end > d->seq_lens[g.seq]) return HG_ERR_RANGE;
    }
    return HG_OK;
}

// The matrix-core kernels take fp16 or bf16 and at least HG_GQA_MIN_GROUP query heads per KV head.
#ifndef HG_GQA_MIN_GROUP
#define HG_GQA_MIN_GROUP 2
#endif
bool use_gqa_kernel(const hg_attn_desc *d) { return d->dtype != HG_F32 && d->n_q_heads / d->n_kv_heads >= HG_GQA_MIN_GROUP; }

// Workgroups per compute unit of hg_attn_concat.  The matrix-core kernel for 128-byte rows is bound
// by instruction issue in this mode (its waves wait for memory 6 % of the time: per byte it does
// twice the work of the 256-byte-row kernel), and one wave per SIMD has nobody to hand the issue
// slot to; with two workgroups per compute unit it ran in 125 us instead of 143 (8 sequences x
// 64k tokens, 32 query heads on 8 KV heads), with three or four in 146 and 159.  Every other
// kernel was faster or level with one (256-byte rows, 8 query heads per KV head: 350 against 367 us).
int concat_workgroups_per_cu(const hg_attn_desc *d) { return use_gqa_kernel(d) && d->head_dim == 64 ? 2 : 1; }

int32_t pick_group_tile(const hg_attn_desc *d)
{
    const int32_t group = d->n_q_heads / d->n_kv_heads;
    if (use_gqa_kernel(d)) return kGqaHeads;
    if (group >= 8) return 8;
    if (group > 2) return 4;
    return group;  // 1 or 2
}

// Positions per workgroup.  Long inputs get one workgroup (four waves) per compute unit, each
// streaming an equal share: measured on MI355X, about 32 KiB of loads in flight per compute unit
// from as few waves as possible gives the highest HBM read rate (more resident waves lose 4-5 %),
// and the launch ends without a tail.  Short inputs get 64-token spans so that they still spread
// over the chip.
int32_t pick_span(int64_t total, bool gqa, int per_cu_factor)
{
    if (g_forced_span_tokens) return g_forced_span_tokens;
    const int64_t target = (int64_t)(gqa ? kGqaWorkgroupsPerCu : kValuWorkgroupsPerCu) * per_cu_factor * compute_units();
    int64_t t = (total + target - 1) / target;
    t = (t + 63) / 64 * 64;
    if (t < 64) t = 64;
    if (t > 0x40000000) t = 0x40000000;
    return (int32_t)t;
}

hg_status make_plan(const hg_attn_desc *d, const hg_range *ranges, int32_t n_ranges, Plan &p, int workgroups_per_cu = 1)
{
    const int32_t group = d->n_q_heads / d->n_kv_heads;
    p.ws.group = group;
    p.ws.gt = pick_group_tile(d);
    p.ws.n_chunks = (group + p.ws.gt - 1) / p.ws.gt;
    p.ws.n_q_heads = d->n_q_heads;
    const int64_t n_streams = (int64_t)d->n_kv_heads * p.ws.n_chunks;
    p.entries.resize((size_t)n_ranges + 1);
    int64_t ltok = 0;
    for (int32_t r = 0; r < n_ranges; ++r) {
        p.entries[r] = RangeEntry{ranges[r].seq, ranges[r].begin, ranges[r].end, (int32_t)ltok, 0};
        ltok += ranges[r].end - ranges[r].begin;
        if (ltok > 0x7fffffff) return HG_ERR_SHAPE;  // more than 2^31-1 tokens in one call
    }
    p.entries[n_ranges] = RangeEntry{0, 0, 0, (int32_t)ltok, 0};
    p.ws.ltok = (int32_t)ltok;
    p.ws.total = n_streams * ltok;
    // The matrix-core kernel for 128-byte rows is the one kernel close to its instruction-issue
    // limit (one wave per SIMD has to issue a block's instructions in the time its 8 KiB arrive);
    // the table look-ups and 64-bit addresses of a paged cache push it over, and a second
    // workgroup per compute unit fills the gaps: 218 -> 185 us on the d=64 grouped-query shape,
    // where the contiguous cache and the other kernels measured no gain or a small loss.
    const int per_cu_factor = (use_gqa_kernel(d) && d->head_dim == 64 && d->block_table ? 2 : 1) * workgroups_per_cu;
    p.ws.span = pick_span(p.ws.total, use_gqa_kernel(d), per_cu_factor);
    {
        const int64_t row_bytes = d->stride_t * (d->dtype == HG_F32 ? 4 : 2);
        // Long spans whose byte length is a multiple of 1 MiB put every workgroup of the vector
        // kernel at the same phase of the memory interleave, and the workgroups then advance in
        // step.  Measured on three MI355X machines this costs 4-6 % of the bandwidth (84-87 %
        // instead of 90-91 % of the peak) for spans from 8 to 32 MiB, while starts shifted by
        // 32 KiB from one workgroup to the next held 90-91 % on all of them.  Short spans (one
        // workgroup per (sequence, head) slab, a few MiB) and the matrix-core kernels showed no
        // gain or a small loss, so they keep their aligned spans.
        if (!g_forced_span_tokens && !use_gqa_kernel(d) && row_bytes > 0 && p.ws.span >= 32768 &&
            ((int64_t)p.ws.span * row_bytes) % (1 << 20) == 0) {
            const int64_t skew = std::max<int64_t>(64, ((32768 / row_bytes) + 63) / 64 * 64);
            p.ws.span += (int32_t)skew;
        }
        // the streaming kernels address rows inside a workgroup's span with 32-bit byte offsets
        if (row_bytes > 0) {
            const int64_t cap = (0xffffffffll - 65536) / row_bytes / 64 * 64;
            if (cap < 64) return HG_ERR_SHAPE;
            if (p.ws.span > cap) p.ws.span = (int32_t)cap;
        }
    }
    p.n_workgroups = (p.ws.total + p.ws.span - 1) / p.ws.span;
    if (p.n_workgroups > 0x7fffffff) return HG_ERR_SHAPE;
    p.n_slots = p.ws.total ? p.n_workgroups + n_streams * n_ranges : 0;
    const size_t recs = (size_t)p.n_slots * (size_t)p.ws.gt;
    size_t off = 0;
    p.off_m = off;
    off += align_up(recs * sizeof(float));
    p.off_l = off;
    off += align_up(recs * sizeof(float));
    p.off_o = off;
    off += align_up(recs * (size_t)d->head_dim * sizeof(float));
    p.off_tab = off;
    if (n_ranges > kInlineRanges) off += align_up(p.entries.size() * sizeof(RangeEntry));
    p.total = off;
    return HG_OK;
}

hg_status check_workspace(const void *ws, size_t have, size_t need)
{
    if (need == 0) return HG_OK;
    if (!ws || (uintptr_t)ws % kAlign || have < need) return HG_ERR_WORKSPACE;
    return HG_OK;
}

// Status of the launches made since the last call of this function (by this thread).
hg_status launch_status(const char *what)
{
    const hipError_t err = t_launch_error;
    t_launch_error = hipSuccess;
    if (err == hipSuccess) return HG_OK;
    std::fprintf(stderr, "hg_attn: %s failed: %s\n", what, hipGetErrorString(err));
    return HG_ERR_LAUNCH;
}

// Fill the by-value table; large tables go to the workspace through upload kernels.
hg_status stage_table(const Plan &p, int32_t n_ranges, char *ws, hipStream_t stream, RangeTable &tab)
{
    tab.n_ranges = n_ranges;
    tab.pad = 0;
    tab.ext = nullptr;
    if (n_ranges <= kInlineRanges) {
        std::memcpy(tab.inl, p.entries.data(), p.entries.size() * sizeof(RangeEntry));
        return HG_OK;
    }
    RangeEntry *dst = reinterpret_cast<RangeEntry *>(ws + p.off_tab);
    tab.ext = dst;
    const size_t n = p.entries.size();
    for (size_t i = 0; i < n; i += kUploadRanges) {
        RangeChunk chunk;
        const int cnt = (int)std::min<size_t>(kUploadRanges, n - i);
        std::memcpy(chunk.e, p.entries.data() + i, (size_t)cnt * sizeof(RangeEntry));
        HG_LAUNCH(hg_upload_ranges_kernel, dim3(1), dim3(kUploadRanges), stream, dst + i, cnt, chunk);
    }
    return launch_status("range table upload");
}

// Rows in flight per 16-lane group.  The logits and concat modes read only K or only V, so they
// keep twice as many rows in flight to have the same number of bytes outstanding.
template <typename TR, int MODE, bool PAGED>
void launch_valu_gt(const PartialArgs &a, int gt, dim3 grid, hipStream_t stream)
{
    constexpr int F = MODE == kModeStats ? 1 : 2;
    if constexpr (TR::DT != kDtF32) {
        // 16-bit storage with a query group goes to the matrix-core kernels: only one head per lane group here
        HG_LAUNCH((hg_partial_kernel<TR, 1, F * HG_VALU_U, MODE, PAGED>), grid, dim3(kValuBlock), stream, a);
        return;
    }
    switch (gt) {
    case 1: HG_LAUNCH((hg_partial_kernel<TR, 1, F * HG_VALU_U, MODE, PAGED>), grid, dim3(kValuBlock), stream, a); break;
    case 2: HG_LAUNCH((hg_partial_kernel<TR, 2, F * HG_VALU_U, MODE, PAGED>), grid, dim3(kValuBlock), stream, a); break;
    case 4: HG_LAUNCH((hg_partial_kernel<TR, 4, F * 2, MODE, PAGED>), grid, dim3(kValuBlock), stream, a); break;
    default: HG_LAUNCH((hg_partial_kernel<TR, 8, F * 2, MODE, PAGED>), grid, dim3(kValuBlock), stream, a); break;
    }
}

template <int MODE, bool PAGED>
void launch_stream_paged(const hg_attn_desc *d, const PartialArgs &a, int gt, dim3 grid, hipStream_t stream)
{
    const bool bf16 = d->dtype == HG_BF16;
    if (use_gqa_kernel(d)) {
        if (d->head_dim == 128) {
            if (bf16)
                HG_LAUNCH((hg_partial_gqa_kernel<MODE, PAGED, true>), grid, dim3(kGqaBlock), stream, a);
            else
                HG_LAUNCH((hg_partial_gqa_kernel<MODE, PAGED, false>), grid, dim3(kGqaBlock), stream, a);
        } else {
            if (bf16)
                HG_LAUNCH((hg_partial_gqa64_kernel<MODE, PAGED, true>), grid, dim3(kGqaBlock), stream, a);
            else
                HG_LAUNCH((hg_partial_gqa64_kernel<MODE, PAGED, false>), grid, dim3(kGqaBlock), stream, a);
        }
        return;
    }
    if (d->head_dim == 128) {
        if (d->dtype == HG_F16)
            launch_valu_gt<Traits<128, kDtF16>, MODE, PAGED>(a, gt, grid, stream);
        else if (bf16)
            launch_valu_gt<Traits<128, kDtBf16>, MODE, PAGED>(a, gt, grid, stream);
        else
            launch_valu_gt<Traits<128, kDtF32>, MODE, PAGED>(a, gt, grid, stream);
    } else {
        if (d->dtype == HG_F16)
            launch_valu_gt<Traits<64, kDtF16>, MODE, PAGED>(a, gt, grid, stream);
        else if (bf16)
            launch_valu_gt<Traits<64, kDtBf16>, MODE, PAGED>(a, gt, grid, stream);
        else
            launch_valu_gt<Traits<64, kDtF32>, MODE, PAGED>(a, gt, grid, stream);
    }
}

// One launch of the streaming kernel that fits the problem (storage type, head_dim, query group,
// contiguous or paged cache), in the given mode.
template <int MODE>
void launch_stream(const hg_attn_desc *d, const PartialArgs &a, int gt, dim3 grid, hipStream_t stream)
{
    if (d->block_table)
        launch_stream_paged<MODE, true>(d, a, gt, grid, stream);
    else
        launch_stream_paged<MODE, false>(d, a, gt, grid, stream);
}

void fill_pages(const hg_attn_desc *d, PageMap &pages)
{
    if (!d->block_table) return;  // the caller zeroed the structure: table == nullptr means contiguous
    pages.table = d->block_table;
    pages.mask = d->block_tokens - 1;
    pages.shift = 0;
    while ((1 << pages.shift) < d->block_tokens) ++pages.shift;
    pages.max_blocks = d->max_blocks;
}

void fill_stream_args(const hg_attn_desc *d, const Plan &p, char *ws, PartialArgs &pa)
{
    pa.q = d->q;
    pa.k = d->k;
    pa.v = d->v;
    pa.stride_b = d->stride_b;
    pa.stride_h = d->stride_h;
    pa.stride_t = d->stride_t;
    pa.ws = p.ws;
    pa.qscale = d->scale * kLog2e;
    fill_pages(d, pa.pages);
    if (ws) {
        pa.ws_m = reinterpret_cast<float *>(ws + p.off_m);
        pa.ws_l = reinterpret_cast<float *>(ws + p.off_l);
        pa.ws_o = reinterpret_cast<float *>(ws + p.off_o);
    }
}

// Group CSR: by value in the kernel arguments when small, else uploaded to `dst`.
hg_status stage_groups(const int32_t *group_ptr, int32_t n_groups, int32_t *dst, hipStream_t stream, GroupTable &tab)
{
    tab.n_groups = n_groups;
    tab.ext = nullptr;
    if (n_groups <= kInlineGroups) {
        std::memcpy(tab.inl, group_ptr, ((size_t)n_groups + 1) * sizeof(int32_t));
        return HG_OK;
    }
    tab.ext = dst;
    const size_t n = (size_t)n_groups + 1;
    for (size_t i = 0; i < n; i += kUploadInts) {
        IntChunk chunk;
        const int cnt = (int)std::min<size_t>(kUploadInts, n - i);
        std::memcpy(chunk.e, group_ptr + i, (size_t)cnt * sizeof(int32_t));
        HG_LAUNCH(hg_upload_ints_kernel, dim3(1), dim3(kUploadInts), stream, dst + i, cnt, chunk);
    }
    return launch_status("group table upload");
}

// True when no (range, stream) pair is cut by a span boundary and no range is empty: every
// segment is then a whole pair, the streaming kernel writes the results itself and the reduce
// launch is skipped.  (Checked only for tables small enough for the check to be free.)
bool plan_is_direct(const Plan &p, int32_t n_ranges, int64_t n_streams)
{
    if (p.ws.total == 0 || n_streams * n_ranges > 65536) return false;
    for (int64_t s = 0; s < n_streams; ++s)
        for (int32_t r = 0; r < n_ranges; ++r) {
            const int64_t len = p.entries[r + 1].pre - p.entries[r].pre;
            if (len == 0) return false;
            const int64_t p0 = s * p.ws.ltok + p.entries[r].pre;
            if (p0 / p.ws.span != (p0 + len - 1) / p.ws.span) return false;
        }
    return true;
}

// Shared by hg_attn_partial (normalise = 0) and hg_attn_full (normalise = 1).
hg_status run(const hg_attn_desc *d, const hg_range *ranges, int32_t n_ranges, int normalise, float *m, float *l,
              float *o, void *workspace, size_t ws_bytes, void *stream_v)
{
    Plan p;
    hg_status st = make_plan(d, ranges, n_ranges, p);
    if (st != HG_OK) return st;
    st = check_workspace(workspace, ws_bytes, p.total);
    if (st != HG_OK) return st;
    if (n_ranges == 0) return HG_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);

    PartialArgs pa;
    std::memset(&pa, 0, sizeof(pa));
    st = stage_table(p, n_ranges, ws, stream, pa.tab);
    if (st != HG_OK) return st;
    fill_stream_args(d, p, ws, pa);
    pa.direct = plan_is_direct(p, n_ranges, (int64_t)d->n_kv_heads * p.ws.n_chunks) ? 1 : 0;
    pa.normalise = normalise;
    pa.out_m = m;
    pa.out_l = l;
    pa.out_o = o;
    if (p.n_workgroups > 0) {
        dim3 grid((unsigned)p.n_workgroups);
        // In timing mode the kernel is launched g_prof_repeat times back to back between one pair
        // of events (it is idempotent: every launch writes the same segment records), so that the
        // fixed cost of the event records is spread over several launches.
        const bool timed = (size_t)(2 * g_prof_used + 2) <= g_prof_events.size();
        const int reps = timed ? g_prof_repeat : 1;
        if (timed) (void)hipEventRecord(g_prof_events[2 * g_prof_used], stream);
        for (int rep = 0; rep < reps; ++rep) launch_stream<kModeStats>(d, pa, p.ws.gt, grid, stream);
        if (timed) (void)hipEventRecord(g_prof_events[2 * g_prof_used++ + 1], stream);
        st = launch_status("partial kernel");
        if (st != HG_OK) return st;
    }
    if (pa.direct) return HG_OK;

    ReduceArgs ra;
    std::memset(&ra, 0, sizeof(ra));
    ra.tab = pa.tab;
    ra.ws_m = pa.ws_m;
    ra.ws_l = pa.ws_l;
    ra.ws_o = pa.ws_o;
    ra.ws = p.ws;
    ra.normalise = normalise;
    ra.m_out = m;
    ra.l_out = l;
    ra.o_out = o;
    dim3 rgrid((unsigned)n_ranges, (unsigned)d->n_q_heads);
    if (d->head_dim == 128)
        HG_LAUNCH(hg_segment_reduce_kernel<128>, rgrid, dim3(kReduceBlock), stream, ra);
    else
        HG_LAUNCH(hg_segment_reduce_kernel<64>, rgrid, dim3(kReduceBlock), stream, ra);
    return launch_status("segment reduce kernel");
}

// Workspace of hg_attn_concat: the streaming sections, then the group table.
void add_concat_sections(Plan &p, int32_t n_groups, int32_t n_q_heads)
{
    (void)n_q_heads;
    size_t off = p.total;
    p.off_groups = off;
    if (n_groups > kInlineGroups) off += align_up(((size_t)n_groups + 1) * sizeof(int32_t));
    p.total = off;
}

hg_status check_concat_groups(const hg_range *ranges, int32_t n_ranges, const int32_t *group_ptr, int32_t n_groups)
{
    if (n_groups < 0 || n_groups > 65535) return HG_ERR_SHAPE;
    if (!group_ptr) return HG_ERR_NULL;
    if (group_ptr[0] != 0 || group_ptr[n_groups] != n_ranges) return HG_ERR_RANGE;
    for (int32_t i = 0; i < n_groups; ++i) {
        if (group_ptr[i] > group_ptr[i + 1]) return HG_ERR_RANGE;
        for (int32_t r = group_ptr[i] + 1; r < group_ptr[i + 1]; ++r)
            if (ranges[r].seq != ranges[group_ptr[i]].seq) return HG_ERR_RANGE;  // one group, one sequence
    }
    return HG_OK;
}

hg_status full_ranges(const hg_attn_desc *d, std::vector<hg_range> &ranges)
{
    hg_status st = check_desc(d);
    if (st != HG_OK) return st;
    ranges.resize((size_t)d->batch);
    for (int32_t b = 0; b < d->batch; ++b) ranges[b] = hg_range{b, 0, d->seq_lens[b]};
    return HG_OK;
}

size_t merge_ws_bytes(int32_t n_groups)
{
    return n_groups > kInlineGroups ? align_up(((size_t)n_groups + 1) * sizeof(int32_t)) : 0;
}

// The logits call records nothing: its workspace only holds the range table when that does
// not fit in the kernel arguments.
size_t logits_ws_bytes(int32_t n_ranges)
{
    return n_ranges > kInlineRanges ? align_up(((size_t)n_ranges + 1) * sizeof(RangeEntry)) : 0;
}

// Long groups are selected in two stages (candidates per part, then among the candidates).
// The fast path of the selection kernel holds kSelectRegTokens elements per workgroup, which is also the part size.
constexpr int kSelectMaxParts = 64;

// Workspace of hg_attn_select: range table, group table (when they do not fit in kernel
// arguments), then the candidate values and columns of the two-stage path.
struct SelectPlan {
    int32_t parts = 1;
    int64_t longest = 0;     // tokens of the longest group
    int32_t parts2 = 0;      // > 0: a middle stage reduces parts * top_k candidates to parts2 * top_k
    bool fast_first = true;  // fast path possible in the direct / candidates launch: top_k and elements per workgroup fit
    bool fast_final = true;  // the same for the launch that selects among the candidates
    size_t off_tab = 0, off_groups = 0, off_cand_val = 0, off_cand_col = 0, off_cand2_val = 0, off_cand2_col = 0, total = 0;
};

void select_parts(const hg_range *ranges, const int32_t *group_ptr, int32_t n_groups, int32_t top_k, SelectPlan &sp)
{
    int64_t longest = 0;
    for (int32_t i = 0; i < n_groups; ++i) {
        int64_t n = 0;
        for (int32_t r = group_ptr[i]; r < group_ptr[i + 1]; ++r) n += ranges[r].end - ranges[r].begin;
        longest = std::max(longest, n);
    }
    sp.longest = longest;
    sp.parts = (int32_t)std::min<int64_t>(kSelectMaxParts, std::max<int64_t>(1, (longest + kSelectRegTokens - 1) / kSelectRegTokens));
    sp.fast_first = top_k <= kSelectFastKeep && (longest + sp.parts - 1) / sp.parts <= kSelectRegTokens;
    // More candidates than one workgroup of the fast path holds: a middle stage brings them down to
    // parts2 * top_k (at most 4 * 1024), so that no stage has to run the slow passes over them.
    const int64_t cands = (int64_t)sp.parts * top_k;
    sp.parts2 = 0;
    if (sp.parts > 1 && top_k <= kSelectFastKeep && cands > kSelectRegTokens)
        sp.parts2 = (int32_t)((cands + kSelectRegTokens - 1) / kSelectRegTokens);
    sp.fast_final = top_k <= kSelectFastKeep && (sp.parts2 ? (int64_t)sp.parts2 * top_k : cands) <= kSelectRegTokens;
}

SelectPlan plan_select(const hg_range *ranges, int32_t n_ranges, const int32_t *group_ptr, int32_t n_groups,
                       int32_t n_q_heads, int32_t top_k)
{
    SelectPlan sp;
    select_parts(ranges, group_ptr, n_groups, top_k, sp);
    size_t off = 0;
    sp.off_tab = off;
    off += logits_ws_bytes(n_ranges);
    sp.off_groups = off;
    off += merge_ws_bytes(n_groups);
    if (sp.parts > 1) {
        const size_t cand = (size_t)n_groups * (size_t)n_q_heads * (size_t)sp.parts * (size_t)top_k * 4;
        sp.off_cand_val = off;
        off += align_up(cand);
        sp.off_cand_col = off;
        off += align_up(cand);
        if (sp.parts2) {
            const size_t cand2 = (size_t)n_groups * (size_t)n_q_heads * (size_t)sp.parts2 * (size_t)top_k * 4;
            sp.off_cand2_val = off;
            off += align_up(cand2);
            sp.off_cand2_col = off;
            off += align_up(cand2);
        }
    }
    sp.total = off;
    return sp;
}

template <int STAGE, bool FAST>
void launch_select_variant(const hg_attn_desc *desc, const SelectArgs &sa, dim3 grid, hipStream_t stream)
{
    const dim3 block(FAST ? kSelectFastBlock : kSelectBlock);
    if (desc->head_dim == 128) {
        if (desc->dtype == HG_F16)
            HG_LAUNCH((hg_select_kernel<Traits<128, kDtF16>, STAGE, FAST>), grid, block, stream, sa);
        else if (desc->dtype == HG_BF16)
            HG_LAUNCH((hg_select_kernel<Traits<128, kDtBf16>, STAGE, FAST>), grid, block, stream, sa);
        else
            HG_LAUNCH((hg_select_kernel<Traits<128, kDtF32>, STAGE, FAST>), grid, block, stream, sa);
    } else {
        if (desc->dtype == HG_F16)
            HG_LAUNCH((hg_select_kernel<Traits<64, kDtF16>, STAGE, FAST>), grid, block, stream, sa);
        else if (desc->dtype == HG_BF16)
            HG_LAUNCH((hg_select_kernel<Traits<64, kDtBf16>, STAGE, FAST>), grid, block, stream, sa);
        else
            HG_LAUNCH((hg_select_kernel<Traits<64, kDtF32>, STAGE, FAST>), grid, block, stream, sa);
    }
}

template <int STAGE>
void launch_select(const hg_attn_desc *desc, const SelectArgs &sa, dim3 grid, bool fast, hipStream_t stream)
{
    if (fast)
        launch_select_variant<STAGE, true>(desc, sa, grid, stream);
    else
        launch_select_variant<STAGE, false>(desc, sa, grid, stream);
}

void fill_select_args(const hg_attn_desc *desc, const Plan &p, const SelectPlan &sp, SelectArgs &sa, int32_t top_k, int32_t *sel,
                      float *m, float *l, float *o)
{
    sa.v = desc->v;
    fill_pages(desc, sa.pages);
    sa.stride_b = desc->stride_b;
    sa.stride_h = desc->stride_h;
    sa.stride_t = desc->stride_t;
    sa.ltok = p.ws.ltok;
    sa.n_q_heads = desc->n_q_heads;
    sa.group = desc->n_q_heads / desc->n_kv_heads;
    sa.top_k = top_k;
    sa.sel = sel;
    sa.m = m;
    sa.l = l;
    sa.o = o;
    sa.parts = sp.parts;
}

// The launches of a selection whose tables (sa.tab, sa.groups) and input (sa.logits, or the dense
// survivor lists sa.dense_*) are in place: one kernel for short groups, else candidates per part,
// an optional middle stage, and the final selection among the candidates.
hg_status select_stages(const hg_attn_desc *desc, const Plan &p, const SelectPlan &sp, SelectArgs &sa, int32_t n_groups,
                        int32_t top_k, int32_t *sel, float *m, float *l, float *o, char *ws, hipStream_t stream)
{
    fill_select_args(desc, p, sp, sa, top_k, sel, m, l, o);
    dim3 grid((unsigned)n_groups, (unsigned)desc->n_q_heads);
    if (sp.parts == 1) {
        launch_select<kSelectDirect>(desc, sa, grid, sp.fast_first, stream);
        return launch_status("selection kernel");
    }
    sa.cand_val = reinterpret_cast<float *>(ws + sp.off_cand_val);
    sa.cand_col = reinterpret_cast<int32_t *>(ws + sp.off_cand_col);
    if (sa.dense_cnt && top_k <= kSelectFastKeep) {
        // Survivor lists are sized for the worst case but are usually a fraction of a per cent of
        // the group: whichever (group, head) has at most one fast-path workgroup's worth is selected
        // by a single workgroup, and the staged kernels below leave it alone (they decide by the
        // same count, on the device: the host never learns the counts).
        sa.direct_limit = kSelectRegTokens;
        launch_select<kSelectDirect>(desc, sa, grid, true, stream);
        const hg_status st0 = launch_status("selection kernel (short lists)");
        if (st0 != HG_OK) return st0;
    }
    launch_select<kSelectCandidates>(desc, sa, dim3((unsigned)(n_groups * sp.parts), (unsigned)desc->n_q_heads), sp.fast_first, stream);
    hg_status st = launch_status("selection kernel (candidates)");
    if (st != HG_OK) return st;
    if (sp.parts2) {
        sa.parts2 = sp.parts2;
        sa.cand2_val = reinterpret_cast<float *>(ws + sp.off_cand2_val);
        sa.cand2_col = reinterpret_cast<int32_t *>(ws + sp.off_cand2_col);
        launch_select<kSelectMidCands>(desc, sa, dim3((unsigned)(n_groups * sp.parts2), (unsigned)desc->n_q_heads), true, stream);
        st = launch_status("selection kernel (middle stage)");
        if (st != HG_OK) return st;
    }
    launch_select<kSelectFromCands>(desc, sa, grid, sp.fast_final, stream);
    return launch_status("selection kernel (final)");
}

// The selection behind a filter pass in one launch (sa.surv_*, sa.tail_*, sa.ws in place).
hg_status select_survivors(const hg_attn_desc *desc, const Plan &p, const SelectPlan &sp, SelectArgs &sa, int32_t n_groups,
                           int32_t top_k, int32_t *sel, float *m, float *l, float *o, char *ws, hipStream_t stream)
{
    fill_select_args(desc, p, sp, sa, top_k, sel, m, l, o);
    if (sp.parts > 1) {
        sa.cand_val = reinterpret_cast<float *>(ws + sp.off_cand_val);
        sa.cand_col = reinterpret_cast<int32_t *>(ws + sp.off_cand_col);
    }
    const dim3 grid((unsigned)((int64_t)n_groups * desc->n_q_heads), (unsigned)sa.tail_parts), block(kSelectFastBlock);
    if (desc->head_dim == 128) {
        if (desc->dtype == HG_F16)
            HG_LAUNCH((hg_select_survivors_kernel<Traits<128, kDtF16>>), grid, block, stream, sa);
        else if (desc->dtype == HG_BF16)
            HG_LAUNCH((hg_select_survivors_kernel<Traits<128, kDtBf16>>), grid, block, stream, sa);
        else
            HG_LAUNCH((hg_select_survivors_kernel<Traits<128, kDtF32>>), grid, block, stream, sa);
    } else {
        if (desc->dtype == HG_F16)
            HG_LAUNCH((hg_select_survivors_kernel<Traits<64, kDtF16>>), grid, block, stream, sa);
        else if (desc->dtype == HG_BF16)
            HG_LAUNCH((hg_select_survivors_kernel<Traits<64, kDtBf16>>), grid, block, stream, sa);
        else
            HG_LAUNCH((hg_select_survivors_kernel<Traits<64, kDtF32>>), grid, block, stream, sa);
    }
    return launch_status("selection kernel (survivor lists)");
}

// hg_attn_topk: the scan that keeps only logits which can still be among a group's top_k (filter
// mode of the streaming kernels) exists for the matrix-core kernel of 256-byte rows and for the
// vector kernel with one query head per KV head (any storage type), contiguous or paged caches,
// top_k <= kFilterMaxTopK; everything else exports all logits to the workspace and selects from them.
constexpr int kFilterMaxTopK = 256;

bool filter_supported(const hg_attn_desc *d, int32_t top_k)
{
    if (g_topk_mode == 2 || top_k > kFilterMaxTopK) return false;
    if (use_gqa_kernel(d)) return d->head_dim == 128;
    return d->n_q_heads == d->n_kv_heads;  // vector kernel: one query head per KV head
}

// Distinct logits per workgroup that the own bound of the matrix-core filter scan rests on when
// every lane keeps one of them: 4 waves x 16 lanes of a head.  (The vector kernel counts among
// the four logits each of its >= 32 row lanes per wave keeps: 128 per wave, of which it needs
// top_k / 4 <= 64.)
int filter_sets(const hg_attn_desc *) { return kGqaWaves * 16; }

// The filter scan pays off when the bounds rise quickly against the length of the scan; otherwise
// a large share of the logits gets through and the two-call sequence is faster.
//
// Vector kernel (own bounds only): the bound rises like the logarithm of the tokens a workgroup has
// seen, so the groups must be long against top_k.  Measured at top_k 128: the scan loses at 6.5k
// tokens per group (a third survives), wins by 6-8 % at 20k-26k and by a fifth at 105k.
//
// Matrix-core kernel: it has less time to spare per block, and its scan wins where the workgroups
// that share a (range, stream) pair can combine what they have seen -- a shared bound with some
// slack exists, by the kernel's own rule: 3 * 64 * min(workgroups per pair, 8) >= 4 * top_k, and
// at least two of them -- and where the logits not written and read back are a sizeable part of
// the traffic (8 bytes per query head and token against 256 per K row: four or more query heads
// per KV head).  Measured over 8 KV heads, 420k tokens in all, top_k 64 / 128 / 256, where the
// rule holds: the scan takes 0.91-0.99 of the two-call time at 4 query heads per KV head,
// 0.83-0.91 at 8 and 0.71-0.80 at 16; where it does not hold, 0.96-1.5 (and 0.99-1.24 at 2 query
// heads per KV head everywhere).
constexpr int64_t kFilterMinTokensPerKeptValu = 128;
constexpr int32_t kFilterMinQueryGroupGqa = 4;

bool filter_chosen(const hg_attn_desc *d, int32_t top_k, const Plan &p, int32_t n_groups)
{
    if (!filter_supported(d, top_k)) return false;
    if (g_topk_mode == 1 || g_topk_mode == 3) return true;
    const int64_t ltok = p.ws.ltok;
    if (!use_gqa_kernel(d)) return ltok >= kFilterMinTokensPerKeptValu * top_k * std::max<int32_t>(n_groups, 1);
    const int64_t n_ranges = std::max<int64_t>((int64_t)p.entries.size() - 1, 1);
    const int64_t per_pair = ltok / std::max<int64_t>((int64_t)p.ws.span * n_ranges, 1);  // workgroups per (range, stream) pair, on average
    return d->n_q_heads >= kFilterMinQueryGroupGqa * d->n_kv_heads && per_pair >= 2 &&
           3 * 64 * std::min<int64_t>(per_pair, 8) >= 4 * (int64_t)top_k;
}

int filter_sub_spans(const hg_attn_desc *d) { return use_gqa_kernel(d) ? kGqaWaves : kValuWaves; }

// Workgroups per compute unit of the filter pass (a tuning constant; every further segment a group
// is cut into lets more logits through before the bounds have risen).
#ifndef HG_FILTER_WG_PER_CU
#define HG_FILTER_WG_PER_CU 1
#endif
int topk_workgroups_per_cu(const hg_attn_desc *d, int32_t top_k) { return filter_supported(d, top_k) ? HG_FILTER_WG_PER_CU : 1; }
static_assert(HG_FILTER_WG_PER_CU == 1, "with another value the plan of the two-call sequence inside hg_attn_topk would differ from hg_attn_logits'");

struct TopkPlan {
    bool fused = false;
    bool tail = false;      // fused: one selection kernel reads the filter pass's lists (else compaction + staged selection)
    int32_t tail_parts = 1; // its workgroups per (group, head)
    size_t off_tail_cnt = 0, n_tail = 0;
    int32_t n_sub = 0, chunks = 1;
    size_t off_logits = 0;  // unfused: all logits [Hq][ltok]
    size_t off_surv_val = 0, off_surv_col = 0, off_surv_cnt = 0, off_dense_val = 0, off_dense_col = 0, off_dense_cnt = 0;
    size_t n_counts = 0;                  // survivor counts: one per (slot, sub-span, head of the stream)
    size_t off_gbound = 0, n_bounds = 0;  // shared bounds: 64 words per (slot, head of the stream)
    size_t total = 0;
};

// Whether hg_select_survivors_kernel can take the selection behind a filter pass: the items of
// every (group, head) -- sub-span lists in column order; a range of n tokens lies in at most
// (n - 1) / span + 2 workgroups' spans -- fit its table, the longest row fits its slices and the
// candidates of all slices fit one fast-path workgroup.
bool survivors_kernel_fits(const hg_range *ranges, const int32_t *group_ptr, int32_t n_groups, const Plan &p, const SelectPlan &sp,
                           int32_t n_sub, int32_t top_k)
{
    if (top_k > kSelectFastKeep || (int64_t)sp.parts * top_k > kSelectRegTokens) return false;
    if (sp.longest > (int64_t)sp.parts * kSelectRegTokens) return false;
    if ((int64_t)n_groups * p.ws.n_q_heads > 0x7fffffff) return false;  // its grid: one column per (group, head)
    for (int32_t i = 0; i < n_groups; ++i) {
        int64_t items = 0;
        for (int32_t r = group_ptr[i]; r < group_ptr[i + 1]; ++r) {
            const int64_t n = ranges[r].end - ranges[r].begin;
            if (n > 0) items += ((n - 1) / std::max<int32_t>(p.ws.span, 1) + 2) * n_sub;
        }
        if (items > kSurvivorItems) return false;
    }
    return true;
}

TopkPlan plan_topk(const hg_attn_desc *d, const hg_range *ranges, const int32_t *group_ptr, const Plan &p, const SelectPlan &sp,
                   int32_t n_groups, int32_t top_k)
{
    TopkPlan tp;
    tp.fused = filter_chosen(d, top_k, p, n_groups);
    size_t off = align_up(sp.total);
    const size_t rows = align_up((size_t)d->n_q_heads * (size_t)p.ws.ltok * 4);
    if (!tp.fused) {
        tp.off_logits = off;
        off += rows;
    } else {
        tp.n_sub = filter_sub_spans(d);
        const int64_t pairs = std::max<int64_t>(1, (int64_t)n_groups * d->n_q_heads);
        tp.tail = g_topk_mode != 3 && survivors_kernel_fits(ranges, group_ptr, n_groups, p, sp, tp.n_sub, top_k);
        // as many workgroups per pair as fill the device about once (two fit a compute unit)
        tp.tail_parts = (int32_t)std::min<int64_t>(sp.parts, std::max<int64_t>(1, 2 * (int64_t)compute_units() / pairs));
        // (every workgroup of a pair repeats the scan of the counts: up to 8 per pair, 512 in all,
        // measured against 1-64 per pair)
        tp.chunks = (int32_t)std::min<int64_t>(8, std::max<int64_t>(1, 512 / pairs));
        tp.off_surv_val = off;
        off += rows;
        tp.off_surv_col = off;
        off += rows;
        if (!tp.tail) {
            tp.off_dense_val = off;
            off += rows;
            tp.off_dense_col = off;
            off += rows;
        }
        tp.n_counts = (size_t)p.n_slots * (size_t)tp.n_sub * (size_t)p.ws.gt;
        tp.n_bounds = (size_t)p.n_slots * (size_t)p.ws.gt * 64;
        tp.off_surv_cnt = off;
        off += align_up(tp.n_counts * 4);
        tp.off_gbound = off;
        off += align_up(tp.n_bounds * 4);
        tp.off_dense_cnt = off;
        off += align_up((size_t)std::max<int32_t>(n_groups, 1) * (size_t)d->n_q_heads * 4);
        tp.n_tail = (size_t)std::max<int32_t>(n_groups, 1) * (size_t)d->n_q_heads;
        tp.off_tail_cnt = off;
        off += align_up(tp.n_tail * 4);
    }
    tp.total = off;
    return tp;
}

template <typename TR>
void launch_valu_filter(const PartialArgs &a, bool paged, dim3 grid, hipStream_t stream)
{
    if (paged)
        HG_LAUNCH((hg_partial_kernel<TR, 1, 2 * HG_VALU_U, kModeFilter, true>), grid, dim3(kValuBlock), stream, a);
    else
        HG_LAUNCH((hg_partial_kernel<TR, 1, 2 * HG_VALU_U, kModeFilter, false>), grid, dim3(kValuBlock), stream, a);
}

template <bool PAGED>
void launch_gqa_filter(const hg_attn_desc *d, const PartialArgs &a, dim3 grid, hipStream_t stream)
{
    const bool wide = a.filter_rank >= 2;  // four kept logits per lane instead of two
    if (d->dtype == HG_BF16) {
        if (wide)
            HG_LAUNCH((hg_partial_gqa_kernel<kModeFilter, PAGED, true, 4>), grid, dim3(kGqaBlock), stream, a);
        else
            HG_LAUNCH((hg_partial_gqa_kernel<kModeFilter, PAGED, true, 2>), grid, dim3(kGqaBlock), stream, a);
    } else {
        if (wide)
            HG_LAUNCH((hg_partial_gqa_kernel<kModeFilter, PAGED, false, 4>), grid, dim3(kGqaBlock), stream, a);
        else
            HG_LAUNCH((hg_partial_gqa_kernel<kModeFilter, PAGED, false, 2>), grid, dim3(kGqaBlock), stream, a);
    }
}

void launch_filter(const hg_attn_desc *d, const PartialArgs &a, dim3 grid, hipStream_t stream)
{
    // (filter_supported() admits exactly the variants instantiated here)
    const bool paged = d->block_table != nullptr;
    if (!use_gqa_kernel(d)) {
        const bool wide = d->head_dim == 128;
        switch (d->dtype) {
        case HG_F16: wide ? launch_valu_filter<Traits<128, kDtF16>>(a, paged, grid, stream) : launch_valu_filter<Traits<64, kDtF16>>(a, paged, grid, stream); break;
        case HG_BF16: wide ? launch_valu_filter<Traits<128, kDtBf16>>(a, paged, grid, stream) : launch_valu_filter<Traits<64, kDtBf16>>(a, paged, grid, stream); break;
        default: wide ? launch_valu_filter<Traits<128, kDtF32>>(a, paged, grid, stream) : launch_valu_filter<Traits<64, kDtF32>>(a, paged, grid, stream); break;
        }
        return;
    }
    if (paged)
        launch_gqa_filter<true>(d, a, grid, stream);
    else
        launch_gqa_filter<false>(d, a, grid, stream);
}

// hg_attn_merge (one producer: csr_b == nullptr) and hg_attn_merge2 (two producers).
hg_status check_csr(const int32_t *csr, int32_t n_groups, const float *m, const float *l, const float *o)
{
    if (!csr) return HG_ERR_NULL;
    if (csr[0] < 0) return HG_ERR_RANGE;
    for (int32_t i = 0; i < n_groups; ++i)
        if (csr[i] > csr[i + 1]) return HG_ERR_RANGE;
    if (csr[n_groups] > csr[0] && (!m || !l || !o)) return HG_ERR_NULL;
    return HG_OK;
}

hg_status merge_sets(const float *m, const float *l, const float *o, const int32_t *csr, const float *m_b, const float *l_b,
                     const float *o_b, const int32_t *csr_b, int32_t n_groups, int32_t n_q_heads, int32_t head_dim, float *out,
                     float *lse_out, void *workspace, size_t ws_bytes, void *stream_v)
{
    if (n_groups < 0 || n_q_heads <= 0 || n_q_heads > 65535) return HG_ERR_SHAPE;
    if (head_dim != 64 && head_dim != 128) return HG_ERR_SHAPE;
    if (n_groups == 0) return HG_OK;
    if (!out) return HG_ERR_NULL;
    hg_status st = check_csr(csr, n_groups, m, l, o);
    if (st != HG_OK) return st;
    // the second set takes part only if it holds a triple at all
    const bool two = csr_b != nullptr;
    if (two) {
        st = check_csr(csr_b, n_groups, m_b, l_b, o_b);
        if (st != HG_OK) return st;
    }
    const bool use_b = two && csr_b[n_groups] > csr_b[0];
    const size_t one = merge_ws_bytes(n_groups);
    st = check_workspace(workspace, ws_bytes, (two ? 2 : 1) * one);
    if (st != HG_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);

    MergeArgs a;
    std::memset(&a, 0, sizeof(a));
    a.m = m;
    a.l = l;
    a.o = o;
    a.out = out;
    a.lse = lse_out;
    a.n_q_heads = n_q_heads;
    st = stage_groups(csr, n_groups, static_cast<int32_t *>(workspace), stream, a.tab);
    if (st != HG_OK) return st;
    if (use_b) {
        a.m_b = m_b;
        a.l_b = l_b;
        a.o_b = o_b;
        st = stage_groups(csr_b, n_groups, reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + one), stream, a.tab_b);
        if (st != HG_OK) return st;
    }
    dim3 grid((unsigned)n_groups, (unsigned)n_q_heads);
    if (head_dim == 128)
        HG_LAUNCH(hg_merge_kernel<128>, grid, dim3(kReduceBlock), stream, a);
    else
        HG_LAUNCH(hg_merge_kernel<64>, grid, dim3(kReduceBlock), stream, a);
    return launch_status("merge kernel");
}

// hg_attn_partial_merge in one launch: the FUSED variant of the vector kernel, one workgroup per
// (group, stream).  A workgroup alone streams about 28 KiB per microsecond, and the launches it
// saves (segment reduce, merge, and the gaps between three kernels) are worth some 12 us: beyond
// kFusedMaxBytes of K and V rows per (group, KV head) the three-kernel path is faster.
constexpr int64_t kFusedMaxBytes = 320 << 10;

bool fused_single_launch(const hg_attn_desc *d, const hg_range *ranges, int32_t n_ranges, const int32_t *group_ptr,
                         int32_t n_groups, const Plan &p)
{
    if (use_gqa_kernel(d) || d->block_table) return false;
    if (n_groups < 1 || n_groups > kFusedGroups || n_ranges > kInlineRanges) return false;
    const int64_t n_streams = (int64_t)d->n_kv_heads * p.ws.n_chunks;
    if (n_streams * n_groups > compute_units()) return false;
    const int64_t row_bytes = 2 * (int64_t)d->head_dim * (d->dtype == HG_F32 ? 4 : 2);  // a K row and a V row
    for (int32_t i = 0; i < n_groups; ++i) {
        int64_t tokens = 0;
        for (int32_t r = group_ptr[i]; r < group_ptr[i + 1]; ++r) tokens += ranges[r].end - ranges[r].begin;
        if (tokens * row_bytes > kFusedMaxBytes) return false;
    }
    return true;
}

template <typename TR>
void launch_valu_fused(const PartialArgs &a, int gt, dim3 grid, hipStream_t stream)
{
    if constexpr (TR::DT != kDtF32) {
        HG_LAUNCH((hg_partial_kernel<TR, 1, HG_VALU_U, kModeStats, false, true>), grid, dim3(kValuBlock), stream, a);
        return;
    }
    switch (gt) {
    case 1: HG_LAUNCH((hg_partial_kernel<TR, 1, HG_VALU_U, kModeStats, false, true>), grid, dim3(kValuBlock), stream, a); break;
    case 2: HG_LAUNCH((hg_partial_kernel<TR, 2, HG_VALU_U, kModeStats, false, true>), grid, dim3(kValuBlock), stream, a); break;
    case 4: HG_LAUNCH((hg_partial_kernel<TR, 4, 2, kModeStats, false, true>), grid, dim3(kValuBlock), stream, a); break;
    default: HG_LAUNCH((hg_partial_kernel<TR, 8, 2, kModeStats, false, true>), grid, dim3(kValuBlock), stream, a); break;
    }
}

hg_status partial_merge_plan(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, const int32_t *group_ptr,
                             int32_t n_groups, Plan &p)
{
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    st = check_concat_groups(ranges, n_ranges, group_ptr, n_groups);
    if (st != HG_OK) return st;
    return make_plan(desc, ranges, n_ranges, p);
}

}  // namespace

extern "C" {

const char *hg_strerror(hg_status status)
{
    switch (status) {
    case HG_OK: return "ok";
    case HG_ERR_NULL: return "a required pointer is NULL";
    case HG_ERR_SHAPE: return "unsupported shape, stride, alignment or count";
    case HG_ERR_DTYPE: return "unsupported dtype";
    case HG_ERR_RANGE: return "malformed range or offset";
    case HG_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case HG_ERR_LAUNCH: return "HIP launch failed";
    }
    return "unknown status";
}

hg_status hg_attn_set_span_tokens(int32_t span_tokens)
{
    if (span_tokens != 0 && (span_tokens < 64 || span_tokens > (1 << 24) || span_tokens % 64)) return HG_ERR_SHAPE;
    g_forced_span_tokens = span_tokens;
    return HG_OK;
}

hg_status hg_attn_set_topk_mode(int32_t mode)
{
    if (mode < 0 || mode > 3) return HG_ERR_SHAPE;
    g_topk_mode = mode;
    return HG_OK;
}

hg_status hg_sched_init(hg_sched_state *state, int32_t k_min)
{
    if (!state) return HG_ERR_NULL;
    if (k_min < 1) return HG_ERR_SHAPE;
    state->k = k_min;
    state->strategy = HG_SELECT_POST_QK;
    return HG_OK;
}

hg_status hg_sched_step(hg_sched_state *state, float t_gpu, float t_cpu, float t_tx, int32_t k_min, int32_t k_max,
                        int32_t k_step)
{
    if (!state) return HG_ERR_NULL;
    if (k_min < 1 || k_max < k_min || k_step < 1) return HG_ERR_SHAPE;
    if (!(t_gpu >= 0.f) || !(t_cpu >= 0.f) || !(t_tx >= 0.f) || !std::isfinite(t_gpu + t_cpu + t_tx)) return HG_ERR_SHAPE;
    // One clamped step: K moves by k_step towards k_max while the offloaded stage (logits +
    // transfer) hides behind the GPU stage, towards k_min while it does not.  A tick that finds
    // the offloaded stage exposed with K already at its floor has nothing left to shed and asks
    // for selection before the logits are computed.
    const auto clamp_k = [&](int64_t k) { return std::min<int64_t>(std::max<int64_t>(k, k_min), k_max); };
    const bool hidden = t_cpu + t_tx <= t_gpu;
    const int64_t k_now = clamp_k(state->k);
    state->strategy = !hidden && k_now == k_min ? HG_SELECT_PRE_QK : HG_SELECT_POST_QK;
    state->k = (int32_t)clamp_k(k_now + (hidden ? (int64_t)k_step : -(int64_t)k_step));
    return HG_OK;
}

hg_status hg_attn_calibration_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src) return HG_ERR_NULL;
    if (bytes % 16 || ((uintptr_t)dst | (uintptr_t)src) % 16) return HG_ERR_SHAPE;
    if (bytes == 0) return HG_OK;
    HG_LAUNCH(hg_calibration_copy_kernel, dim3(4096), dim3(256), static_cast<hipStream_t>(stream),
                       static_cast<hg_u32x4 *>(dst), static_cast<const hg_u32x4 *>(src), bytes / 16);
    return launch_status("calibration copy");
}

hg_status hg_attn_calibration_stream(const void *src, size_t read_bytes, void *dst, int32_t write_vectors_per_iteration,
                                     int32_t burst_iterations, int32_t streaming_stores, void *stream)
{
    if (!src) return HG_ERR_NULL;
    if ((uintptr_t)src % 16 || (uintptr_t)dst % 16) return HG_ERR_SHAPE;
    if (write_vectors_per_iteration < 0 || write_vectors_per_iteration > 2048 || burst_iterations < 1) return HG_ERR_SHAPE;
    if (write_vectors_per_iteration > 0 && !dst) return HG_ERR_NULL;
    const size_t n_wg = (size_t)compute_units();
    const size_t share_vec = read_bytes / 16 / n_wg / 2048 * 2048;  // whole 32 KiB iterations
    if (share_vec == 0 || share_vec / 2048 > 0x7fffffff / 2048) return HG_ERR_SHAPE;
    HG_LAUNCH(hg_calibration_stream_kernel, dim3((unsigned)n_wg), dim3(256), static_cast<hipStream_t>(stream),
              static_cast<const hg_u32x4 *>(src), share_vec, static_cast<hg_u32x4 *>(dst), (int)write_vectors_per_iteration,
              (int)burst_iterations, (int)streaming_stores);
    return launch_status("calibration stream");
}

hg_status hg_attn_profile_start(int32_t max_calls, int32_t repeat)
{
    if (max_calls < 0 || max_calls > 65536 || repeat < 1 || repeat > 1024) return HG_ERR_SHAPE;
    g_prof_repeat = repeat;
    for (hipEvent_t ev : g_prof_events) (void)hipEventDestroy(ev);
    g_prof_events.clear();
    g_prof_used = 0;
    for (int i = 0; i < 2 * max_calls; ++i) {
        hipEvent_t ev;
        const hipError_t err = hipEventCreate(&ev);
        if (err != hipSuccess) {
            std::fprintf(stderr, "hg_attn: event creation failed: %s\n", hipGetErrorString(err));
            return HG_ERR_LAUNCH;
        }
        g_prof_events.push_back(ev);
    }
    return HG_OK;
}

hg_status hg_attn_profile_times(float *ms_each, int32_t capacity, int32_t *calls)
{
    if (capacity < 0 || (capacity > 0 && !ms_each)) return HG_ERR_NULL;
    hg_status st = HG_OK;
    const int n = g_prof_used < capacity ? g_prof_used : capacity;
    for (int i = 0; i < n; ++i) {
        float ms = 0.f;
        hipError_t err = hipEventSynchronize(g_prof_events[2 * i + 1]);
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, g_prof_events[2 * i], g_prof_events[2 * i + 1]);
        if (err != hipSuccess) {
            std::fprintf(stderr, "hg_attn: event read-out failed: %s\n", hipGetErrorString(err));
            st = HG_ERR_LAUNCH;
        }
        ms_each[i] = ms / (float)g_prof_repeat;
    }
    if (calls) *calls = g_prof_used;
    return st;
}

hg_status hg_attn_profile_stop(float *total_ms, int32_t *launches)
{
    float sum = 0.f;
    hg_status st = HG_OK;
    for (int i = 0; i < g_prof_used; ++i) {
        float ms = 0.f;
        hipError_t err = hipEventSynchronize(g_prof_events[2 * i + 1]);
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, g_prof_events[2 * i], g_prof_events[2 * i + 1]);
        if (err != hipSuccess) {
            std::fprintf(stderr, "hg_attn: event read-out failed: %s\n", hipGetErrorString(err));
            st = HG_ERR_LAUNCH;
        }
        sum += ms;
    }
    if (total_ms) *total_ms = sum;
    if (launches) *launches = g_prof_used * g_prof_repeat;
    for (hipEvent_t ev : g_prof_events) (void)hipEventDestroy(ev);
    g_prof_events.clear();
    g_prof_used = 0;
    return st;
}

#ifndef HG_BUILD_ID
#define HG_BUILD_ID "unknown"
#endif
// (the marker lets a loader read the id from the file without mapping the image)
static const char kBuildIdMarker[] = "hg_attn_build_id=" HG_BUILD_ID;
const char *hg_attn_build_id(void) { return kBuildIdMarker + sizeof("hg_attn_build_id=") - 1; }

hg_status hg_attn_plan(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, int32_t *span_tokens,
                       int64_t *n_workgroups)
{
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    Plan p;
    st = make_plan(desc, ranges, n_ranges, p);
    if (st != HG_OK) return st;
    if (span_tokens) *span_tokens = p.ws.span;
    if (n_workgroups) *n_workgroups = p.n_workgroups;
    return HG_OK;
}

hg_status hg_attn_partial_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                         size_t *bytes)
{
    if (!bytes) return HG_ERR_NULL;
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    Plan p;
    st = make_plan(desc, ranges, n_ranges, p);
    if (st != HG_OK) return st;
    *bytes = p.total;
    return HG_OK;
}

hg_status hg_attn_partial(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, float *m, float *l,
                          float *o, void *workspace, size_t ws_bytes, void *stream)
{
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    if (n_ranges && (!m || !l || !o)) return HG_ERR_NULL;
    return run(desc, ranges, n_ranges, 0, m, l, o, workspace, ws_bytes, stream);
}

hg_status hg_attn_partial_static(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, float *m, float *l,
                                 float *o, void *stream)
{
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    if (n_ranges && (!m || !l || !o)) return HG_ERR_NULL;
    Plan p;
    st = make_plan(desc, ranges, n_ranges, p);
    if (st != HG_OK) return st;
    if (p.total > HG_ATTN_STATIC_SCRATCH_BYTES) {
        std::fprintf(stderr, "hg_attn_partial_static: this problem needs %zu bytes of scratch, the static buffer holds %zu; "
                             "use hg_attn_partial with a workspace\n", p.total, (size_t)HG_ATTN_STATIC_SCRATCH_BYTES);
        return HG_ERR_WORKSPACE;
    }
    if (n_ranges == 0 || p.total == 0) return run(desc, ranges, n_ranges, 0, m, l, o, nullptr, 0, stream);
    void *buf = nullptr;
    st = static_scratch(&buf);
    if (st != HG_OK) return st;
    return run(desc, ranges, n_ranges, 0, m, l, o, buf, HG_ATTN_STATIC_SCRATCH_BYTES, stream);
}

hg_status hg_attn_full_workspace_size(const hg_attn_desc *desc, size_t *bytes)
{
    if (!bytes) return HG_ERR_NULL;
    std::vector<hg_range> ranges;
    hg_status st = full_ranges(desc, ranges);
    if (st != HG_OK) return st;
    Plan p;
    st = make_plan(desc, ranges.data(), (int32_t)ranges.size(), p);
    if (st != HG_OK) return st;
    *bytes = p.total;
    return HG_OK;
}

hg_status hg_attn_full(const hg_attn_desc *desc, float *out, float *lse_out, void *workspace, size_t ws_bytes,
                       void *stream)
{
    std::vector<hg_range> ranges;
    hg_status st = full_ranges(desc, ranges);
    if (st != HG_OK) return st;
    if (desc->batch && !out) return HG_ERR_NULL;
    return run(desc, ranges.data(), (int32_t)ranges.size(), 1, lse_out, nullptr, out, workspace, ws_bytes, stream);
}

hg_status hg_attn_logits_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, size_t *bytes)
{
    if (!bytes) return HG_ERR_NULL;
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    *bytes = logits_ws_bytes(n_ranges);
    return HG_OK;
}

hg_status hg_attn_logits(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, float *logits,
                         void *workspace, size_t ws_bytes, void *stream_v)
{
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    Plan p;
    st = make_plan(desc, ranges, n_ranges, p);
    if (st != HG_OK) return st;
    if (p.n_workgroups == 0) return HG_OK;
    if (!logits) return HG_ERR_NULL;
    st = check_workspace(workspace, ws_bytes, logits_ws_bytes(n_ranges));
    if (st != HG_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    PartialArgs pa;
    std::memset(&pa, 0, sizeof(pa));
    p.off_tab = 0;  // the table is the only thing in this workspace
    st = stage_table(p, n_ranges, static_cast<char *>(workspace), stream, pa.tab);
    if (st != HG_OK) return st;
    fill_stream_args(desc, p, nullptr, pa);
    pa.qscale = desc->scale;  // logits leave in natural-log units
    pa.logits = logits;
    launch_stream<kModeLogits>(desc, pa, p.ws.gt, dim3((unsigned)p.n_workgroups), stream);
    return launch_status("logits kernel");
}

hg_status hg_attn_concat_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                        int32_t n_groups, size_t *bytes)
{
    if (!bytes) return HG_ERR_NULL;
    if (n_groups < 0 || n_groups > 65535) return HG_ERR_SHAPE;
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    Plan p;
    st = make_plan(desc, ranges, n_ranges, p, concat_workgroups_per_cu(desc));
    if (st != HG_OK) return st;
    add_concat_sections(p, n_groups, desc->n_q_heads);
    *bytes = p.total;
    return HG_OK;
}

hg_status hg_attn_concat(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, const float *logits,
                         const int32_t *group_ptr, int32_t n_groups, float *out, float *lse_out, void *workspace,
                         size_t ws_bytes, void *stream_v)
{
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    st = check_concat_groups(ranges, n_ranges, group_ptr, n_groups);
    if (st != HG_OK) return st;
    if (n_groups == 0) return HG_OK;
    if (!out) return HG_ERR_NULL;
    Plan p;
    st = make_plan(desc, ranges, n_ranges, p, concat_workgroups_per_cu(desc));
    if (st != HG_OK) return st;
    if (p.ws.total > 0 && !logits) return HG_ERR_NULL;
    add_concat_sections(p, n_groups, desc->n_q_heads);
    st = check_workspace(workspace, ws_bytes, p.total);
    if (st != HG_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);

    PartialArgs pa;
    std::memset(&pa, 0, sizeof(pa));
    st = stage_table(p, n_ranges, ws, stream, pa.tab);
    if (st != HG_OK) return st;
    fill_stream_args(desc, p, ws, pa);
    pa.logits = const_cast<float *>(logits);
    GroupTable groups;
    st = stage_groups(group_ptr, n_groups, reinterpret_cast<int32_t *>(ws + p.off_groups), stream, groups);
    if (st != HG_OK) return st;

    if (p.n_workgroups > 0) {
        launch_stream<kModeConcat>(desc, pa, p.ws.gt, dim3((unsigned)p.n_workgroups), stream);
        st = launch_status("concat streaming kernel");
        if (st != HG_OK) return st;
    }

    ConcatReduceArgs ra;
    std::memset(&ra, 0, sizeof(ra));
    ra.ws_m = pa.ws_m;
    ra.ws_l = pa.ws_l;
    ra.ws_o = pa.ws_o;
    ra.out = out;
    ra.lse = lse_out;
    ra.ws = p.ws;
    ra.groups = groups;
    ra.tab = pa.tab;
    dim3 rgrid((unsigned)n_groups, (unsigned)desc->n_q_heads);
    if (desc->head_dim == 128)
        HG_LAUNCH(hg_concat_reduce_kernel<128>, rgrid, dim3(kReduceBlock), stream, ra);
    else
        HG_LAUNCH(hg_concat_reduce_kernel<64>, rgrid, dim3(kReduceBlock), stream, ra);
    return launch_status("concat reduce kernel");
}

hg_status hg_attn_select_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                        const int32_t *group_ptr, int32_t n_groups, int32_t top_k, size_t *bytes)
{
    if (!bytes) return HG_ERR_NULL;
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    if (top_k < 1 || top_k > kMaxTopK) return HG_ERR_SHAPE;
    st = check_concat_groups(ranges, n_ranges, group_ptr, n_groups);
    if (st != HG_OK) return st;
    *bytes = plan_select(ranges, n_ranges, group_ptr, n_groups, desc->n_q_heads, top_k).total;
    return HG_OK;
}

hg_status hg_attn_select(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, const float *logits,
                         const int32_t *group_ptr, int32_t n_groups, int32_t top_k, int32_t *sel, float *m, float *l,
                         float *o, void *workspace, size_t ws_bytes, void *stream_v)
{
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    if (top_k < 1 || top_k > kMaxTopK) return HG_ERR_SHAPE;
    st = check_concat_groups(ranges, n_ranges, group_ptr, n_groups);
    if (st != HG_OK) return st;
    if (n_groups == 0) return HG_OK;
    if (!m || !l || !o) return HG_ERR_NULL;
    Plan p;
    st = make_plan(desc, ranges, n_ranges, p);
    if (st != HG_OK) return st;
    if (p.ws.ltok > 0 && !logits) return HG_ERR_NULL;
    const SelectPlan sp = plan_select(ranges, n_ranges, group_ptr, n_groups, desc->n_q_heads, top_k);
    if ((int64_t)n_groups * sp.parts > 0x7fffffff) return HG_ERR_SHAPE;
    st = check_workspace(workspace, ws_bytes, sp.total);
    if (st != HG_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);

    SelectArgs sa;
    std::memset(&sa, 0, sizeof(sa));
    p.off_tab = sp.off_tab;
    st = stage_table(p, n_ranges, ws, stream, sa.tab);
    if (st != HG_OK) return st;
    st = stage_groups(group_ptr, n_groups, reinterpret_cast<int32_t *>(ws + sp.off_groups), stream, sa.groups);
    if (st != HG_OK) return st;
    sa.logits = logits;
    return select_stages(desc, p, sp, sa, n_groups, top_k, sel, m, l, o, ws, stream);
}

hg_status hg_attn_topk_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                      const int32_t *group_ptr, int32_t n_groups, int32_t top_k, size_t *bytes)
{
    if (!bytes) return HG_ERR_NULL;
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    if (top_k < 1 || top_k > kMaxTopK) return HG_ERR_SHAPE;
    st = check_concat_groups(ranges, n_ranges, group_ptr, n_groups);
    if (st != HG_OK) return st;
    Plan p;
    st = make_plan(desc, ranges, n_ranges, p, topk_workgroups_per_cu(desc, top_k));
    if (st != HG_OK) return st;
    const SelectPlan sp = plan_select(ranges, n_ranges, group_ptr, n_groups, desc->n_q_heads, top_k);
    *bytes = plan_topk(desc, ranges, group_ptr, p, sp, n_groups, top_k).total;
    return HG_OK;
}

hg_status hg_attn_topk(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, const int32_t *group_ptr,
                       int32_t n_groups, int32_t top_k, int32_t *sel, float *m, float *l, float *o, void *workspace,
                       size_t ws_bytes, void *stream_v)
{
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    st = check_ranges(desc, ranges, n_ranges);
    if (st != HG_OK) return st;
    if (top_k < 1 || top_k > kMaxTopK) return HG_ERR_SHAPE;
    st = check_concat_groups(ranges, n_ranges, group_ptr, n_groups);
    if (st != HG_OK) return st;
    if (n_groups == 0) return HG_OK;
    if (!m || !l || !o) return HG_ERR_NULL;
    Plan p;
    st = make_plan(desc, ranges, n_ranges, p, topk_workgroups_per_cu(desc, top_k));
    if (st != HG_OK) return st;
    const SelectPlan sp = plan_select(ranges, n_ranges, group_ptr, n_groups, desc->n_q_heads, top_k);
    if ((int64_t)n_groups * sp.parts > 0x7fffffff) return HG_ERR_SHAPE;
    const TopkPlan tp = plan_topk(desc, ranges, group_ptr, p, sp, n_groups, top_k);
    st = check_workspace(workspace, ws_bytes, tp.total);
    if (st != HG_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);

    SelectArgs sa;
    std::memset(&sa, 0, sizeof(sa));
    p.off_tab = sp.off_tab;  // one uploaded table serves the scan, the compaction and the selection
    st = stage_table(p, n_ranges, ws, stream, sa.tab);
    if (st != HG_OK) return st;
    st = stage_groups(group_ptr, n_groups, reinterpret_cast<int32_t *>(ws + sp.off_groups), stream, sa.groups);
    if (st != HG_OK) return st;

    PartialArgs pa;
    std::memset(&pa, 0, sizeof(pa));
    pa.tab = sa.tab;
    fill_stream_args(desc, p, nullptr, pa);
    pa.qscale = desc->scale;  // logits in natural-log units, exactly as hg_attn_logits writes them
    const dim3 sgrid((unsigned)p.n_workgroups);
    if (!tp.fused) {
        float *logits = reinterpret_cast<float *>(ws + tp.off_logits);
        if (p.n_workgroups > 0) {
            pa.logits = logits;
            launch_stream<kModeLogits>(desc, pa, p.ws.gt, sgrid, stream);
            st = launch_status("logits kernel");
            if (st != HG_OK) return st;
        }
        sa.logits = logits;
        return select_stages(desc, p, sp, sa, n_groups, top_k, sel, m, l, o, ws, stream);
    }

    float *dense_val = reinterpret_cast<float *>(ws + tp.off_dense_val);
    int32_t *dense_col = reinterpret_cast<int32_t *>(ws + tp.off_dense_col);
    int32_t *dense_cnt = reinterpret_cast<int32_t *>(ws + tp.off_dense_cnt);
    pa.surv_val = reinterpret_cast<float *>(ws + tp.off_surv_val);
    pa.surv_col = reinterpret_cast<int32_t *>(ws + tp.off_surv_col);
    pa.surv_cnt = reinterpret_cast<int32_t *>(ws + tp.off_surv_cnt);
    pa.filter_rank = (top_k + filter_sets(desc) - 1) / filter_sets(desc) - 1;  // every set keeps rank + 1 logits
    pa.filter_k = top_k;
    pa.gbound = reinterpret_cast<uint32_t *>(ws + tp.off_gbound);
    pa.tail_cnt = reinterpret_cast<uint32_t *>(ws + tp.off_tail_cnt);
    pa.n_tail = tp.tail ? (int64_t)tp.n_tail : 0;
    if (p.n_workgroups > 0) {
        if (use_gqa_kernel(desc)) {  // (the vector kernel shares no bounds)
            const unsigned fill_blocks = (unsigned)std::min<size_t>(1024, (tp.n_bounds + 255) / 256);
            HG_LAUNCH(hg_fill_kernel, dim3(fill_blocks), dim3(256), stream, pa.gbound, (int64_t)tp.n_bounds, 0u);
        }
        launch_filter(desc, pa, sgrid, stream);
        st = launch_status("filter kernel");
        if (st != HG_OK) return st;
    }
    if (tp.tail) {
        sa.surv_val = pa.surv_val;
        sa.surv_col = pa.surv_col;
        sa.surv_cnt = pa.surv_cnt;
        sa.tail_cnt = pa.tail_cnt;
        sa.n_sub = tp.n_sub;
        sa.tail_parts = tp.tail_parts;
        sa.ws = p.ws;
        return select_survivors(desc, p, sp, sa, n_groups, top_k, sel, m, l, o, ws, stream);
    }
    CompactArgs ca;
    std::memset(&ca, 0, sizeof(ca));
    ca.surv_val = pa.surv_val;
    ca.surv_col = pa.surv_col;
    ca.surv_cnt = pa.surv_cnt;
    ca.dense_val = dense_val;
    ca.dense_col = dense_col;
    ca.dense_cnt = dense_cnt;
    ca.n_sub = tp.n_sub;
    ca.chunks = tp.chunks;
    ca.ws = p.ws;
    ca.groups = sa.groups;
    ca.tab = sa.tab;
    HG_LAUNCH(hg_survivor_compact_kernel, dim3((unsigned)n_groups, (unsigned)desc->n_q_heads, (unsigned)tp.chunks),
                       dim3(256), stream, ca);
    st = launch_status("survivor compaction kernel");
    if (st != HG_OK) return st;
    sa.dense_val = dense_val;
    sa.dense_col = dense_col;
    sa.dense_cnt = dense_cnt;
    return select_stages(desc, p, sp, sa, n_groups, top_k, sel, m, l, o, ws, stream);
}

hg_status hg_attn_gather_workspace_size(int32_t n_groups, size_t *bytes)
{
    if (!bytes) return HG_ERR_NULL;
    if (n_groups < 0) return HG_ERR_SHAPE;
    *bytes = merge_ws_bytes(n_groups);
    return HG_OK;
}

hg_status hg_attn_gather(const hg_attn_desc *desc, const int32_t *group_seq, int32_t n_groups, const int32_t *index,
                         int32_t max_k, float *m, float *l, float *o, void *workspace, size_t ws_bytes, void *stream_v)
{
    hg_status st = check_desc(desc);
    if (st != HG_OK) return st;
    if (n_groups < 0 || n_groups > 65535 || max_k < 1 || max_k > (1 << 20)) return HG_ERR_SHAPE;
    if (n_groups == 0) return HG_OK;
    if (!group_seq || !index || !m || !l || !o) return HG_ERR_NULL;
    for (int32_t i = 0; i < n_groups; ++i)
        if (group_seq[i] < 0 || group_seq[i] >= desc->batch) return HG_ERR_RANGE;
    st = check_workspace(workspace, ws_bytes, merge_ws_bytes(n_groups));
    if (st != HG_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);

    GatherArgs ga;
    std::memset(&ga, 0, sizeof(ga));
    ga.q = desc->q;
    ga.k = desc->k;
    ga.v = desc->v;
    ga.stride_b = desc->stride_b;
    ga.stride_h = desc->stride_h;
    ga.stride_t = desc->stride_t;
    fill_pages(desc, ga.pages);
    ga.index = index;
    ga.m = m;
    ga.l = l;
    ga.o = o;
    ga.max_k = max_k;
    ga.n_q_heads = desc->n_q_heads;
    ga.group = desc->n_q_heads / desc->n_kv_heads;
    ga.qscale = desc->scale * kLog2e;
    // the sequences travel like a group CSR (n_groups + 1 entries; the last one is unused)
    std::vector<int32_t> seqs(group_seq, group_seq + n_groups);
    seqs.push_back(0);
    st = stage_groups(seqs.data(), n_groups, static_cast<int32_t *>(workspace), stream, ga.seqs);
    if (st != HG_OK) return st;
    dim3 grid((unsigned)n_groups, (unsigned)desc->n_q_heads);
    const dim3 block(256);
    if (desc->head_dim == 128) {
        if (desc->dtype == HG_F16)
            HG_LAUNCH((hg_gather_kernel<Traits<128, kDtF16>>), grid, block, stream, ga);
        else if (desc->dtype == HG_BF16)
            HG_LAUNCH((hg_gather_kernel<Traits<128, kDtBf16>>), grid, block, stream, ga);
        else
            HG_LAUNCH((hg_gather_kernel<Traits<128, kDtF32>>), grid, block, stream, ga);
    } else {
        if (desc->dtype == HG_F16)
            HG_LAUNCH((hg_gather_kernel<Traits<64, kDtF16>>), grid, block, stream, ga);
        else if (desc->dtype == HG_BF16)
            HG_LAUNCH((hg_gather_kernel<Traits<64, kDtBf16>>), grid, block, stream, ga);
        else
            HG_LAUNCH((hg_gather_kernel<Traits<64, kDtF32>>), grid, block, stream, ga);
    }
    return launch_status("gather kernel");
}

hg_status hg_attn_merge_workspace_size(int32_t n_groups, size_t *bytes)
{
    if (!bytes) return HG_ERR_NULL;
    if (n_groups < 0) return HG_ERR_SHAPE;
    *bytes = merge_ws_bytes(n_groups);
    return HG_OK;
}

hg_status hg_attn_merge(const float *m, const float *l, const float *o, const int32_t *group_ptr, int32_t n_groups,
                        int32_t n_q_heads, int32_t head_dim, float *out, float *lse_out, void *workspace,
                        size_t ws_bytes, void *stream_v)
{
    return merge_sets(m, l, o, group_ptr, nullptr, nullptr, nullptr, nullptr, n_groups, n_q_heads, head_dim, out, lse_out,
                      workspace, ws_bytes, stream_v);
}

hg_status hg_attn_partial_merge_workspace_size(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges,
                                               const int32_t *group_ptr, int32_t n_groups, size_t *bytes)
{
    if (!bytes) return HG_ERR_NULL;
    Plan p;
    const hg_status st = partial_merge_plan(desc, ranges, n_ranges, group_ptr, n_groups, p);
    if (st != HG_OK) return st;
    *bytes = align_up(p.total) + merge_ws_bytes(n_groups);  // the two calls' workspaces, one behind the other
    return HG_OK;
}

hg_status hg_attn_partial_merge(const hg_attn_desc *desc, const hg_range *ranges, int32_t n_ranges, const int32_t *group_ptr,
                                int32_t n_groups, float *m, float *l, float *o, float *out, float *lse_out, void *workspace,
                                size_t ws_bytes, void *stream_v)
{
    Plan p;
    hg_status st = partial_merge_plan(desc, ranges, n_ranges, group_ptr, n_groups, p);
    if (st != HG_OK) return st;
    if (n_groups == 0) return HG_OK;
    if (!out || (n_ranges > 0 && (!m || !l || !o))) return HG_ERR_NULL;
    const size_t first = align_up(p.total);
    st = check_workspace(workspace, ws_bytes, first + merge_ws_bytes(n_groups));
    if (st != HG_OK) return st;
    if (fused_single_launch(desc, ranges, n_ranges, group_ptr, n_groups, p)) {
        hipStream_t stream = static_cast<hipStream_t>(stream_v);
        PartialArgs pa;
        std::memset(&pa, 0, sizeof(pa));
        st = stage_table(p, n_ranges, static_cast<char *>(workspace), stream, pa.tab);  // (fits the kernel arguments: nothing is launched)
        if (st != HG_OK) return st;
        fill_stream_args(desc, p, nullptr, pa);
        pa.direct = 1;
        pa.out_m = m;
        pa.out_l = l;
        pa.out_o = o;
        pa.fused_n_groups = n_groups;
        std::memcpy(pa.fused_groups, group_ptr, ((size_t)n_groups + 1) * sizeof(int32_t));
        pa.merged_out = out;
        pa.merged_lse = lse_out;
        const dim3 grid((unsigned)((int64_t)desc->n_kv_heads * p.ws.n_chunks * n_groups));
        if (desc->head_dim == 128) {
            if (desc->dtype == HG_F16)
                launch_valu_fused<Traits<128, kDtF16>>(pa, p.ws.gt, grid, stream);
            else if (desc->dtype == HG_BF16)
                launch_valu_fused<Traits<128, kDtBf16>>(pa, p.ws.gt, grid, stream);
            else
                launch_valu_fused<Traits<128, kDtF32>>(pa, p.ws.gt, grid, stream);
        } else {
            if (desc->dtype == HG_F16)
                launch_valu_fused<Traits<64, kDtF16>>(pa, p.ws.gt, grid, stream);
            else if (desc->dtype == HG_BF16)
                launch_valu_fused<Traits<64, kDtBf16>>(pa, p.ws.gt, grid, stream);
            else
                launch_valu_fused<Traits<64, kDtF32>>(pa, p.ws.gt, grid, stream);
        }
        return launch_status("fused partial and merge kernel");
    }
    st = run(desc, ranges, n_ranges, 0, m, l, o, workspace, first, stream_v);
    if (st != HG_OK) return st;
    return merge_sets(m, l, o, group_ptr, nullptr, nullptr, nullptr, nullptr, n_groups, desc->n_q_heads, desc->head_dim, out,
                      lse_out, static_cast<char *>(workspace) + first, ws_bytes - first, stream_v);
}

hg_status hg_attn_merge2_workspace_size(int32_t n_groups, size_t *bytes)
{
    if (!bytes) return HG_ERR_NULL;
    if (n_groups < 0) return HG_ERR_SHAPE;
    *bytes = 2 * merge_ws_bytes(n_groups);
    return HG_OK;
}

hg_status hg_attn_merge2(const float *m_a, const float *l_a, const float *o_a, const int32_t *group_ptr_a, const float *m_b,
                         const float *l_b, const float *o_b, const int32_t *group_ptr_b, int32_t n_groups, int32_t n_q_heads,
                         int32_t head_dim, float *out, float *lse_out, void *workspace, size_t ws_bytes, void *stream_v)
{
    if (n_groups > 0 && !group_ptr_b) return HG_ERR_NULL;
    return merge_sets(m_a, l_a, o_a, group_ptr_a, m_b, l_b, o_b, group_ptr_b, n_groups, n_q_heads, head_dim, out, lse_out,
                      workspace, ws_bytes, stream_v);
}

}  // extern "C"
