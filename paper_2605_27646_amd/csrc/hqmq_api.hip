// C ABI of the HQMQ library (declared in include/hqmq.h): argument validation, workspace
// carve-up and the stream-ordered kernel sequences.  No allocation, no synchronisation.
#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>

#include "hqmq_device.h"

namespace hqmq {

static thread_local int32_t g_last_hip_error = 0;

}  // namespace hqmq

// Workspace of hqmq_encode_static, for callers that cannot allocate: every GPU the library runs on holds
// its own copy of this array, at its own address, until the process ends.  Host code never uses the
// array's name as an address: the per-device set-up below asks the runtime for it.
static __device__ __align__(256) unsigned char scratch[HQMQ_STATIC_SCRATCH_BYTES];

namespace hqmq {

// Per-device set-up, done once: the search kernels' LDS limit and the device address of `scratch`.  The flag
// of a device is set only after its set-up succeeded, so a failed attempt is retried by the next call;
// devices beyond the table are set up on every call.
constexpr int kMaxDevices = 64;
static std::atomic<bool> g_device_ready[kMaxDevices];
static void *g_scratch_ptr[kMaxDevices];  // written before the device's flag is set, read after it is seen
static std::mutex g_setup_mutex;

// scratch_out: null, or receives the current device's address of the static scratch array.
static hipError_t ensure_device_setup(void **scratch_out = nullptr)
{
    int device = 0;
    hipError_t err = hipGetDevice(&device);
    if (err != hipSuccess)
        return err;
    const bool tracked = device >= 0 && device < kMaxDevices;
    if (!(tracked && g_device_ready[device].load(std::memory_order_acquire))) {
        std::lock_guard<std::mutex> lock(g_setup_mutex);
        if (!(tracked && g_device_ready[device].load(std::memory_order_relaxed))) {
            err = prepare_search_kernels();
            if (err == hipSuccess)
                err = prepare_attend_kernels();
            if (err != hipSuccess)
                return err;
            void *ptr = nullptr;
            err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (err != hipSuccess)
                return err;
            if (!ptr)
                return hipErrorInvalidSymbol;
            if (!tracked) {  // nowhere to keep it: hand it out and set up again next time
                if (scratch_out)
                    *scratch_out = ptr;
                return hipSuccess;
            }
            g_scratch_ptr[device] = ptr;
            g_device_ready[device].store(true, std::memory_order_release);
        }
    }
    if (scratch_out)
        *scratch_out = g_scratch_ptr[device];
    return hipSuccess;
}

static inline uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

static int index_bits(int S)
{
    int j = 0;
    while ((1ll << j) < 24ll * S)
        ++j;
    return j;
}

// Largest S the search kernel's LDS tables are sized for (paper sweeps S up to 192).
constexpr int kMaxS = HQMQ_MAX_S;

static int32_t check_params(const hqmq_params *p)
{
    if (!p)
        return HQMQ_ERR_INVALID_ARG;
    if (p->B <= 0 || p->H <= 0 || p->T <= 0 || p->D <= 0)
        return HQMQ_ERR_INVALID_ARG;
    if (p->D > 4 * kChunksPerRow)
        return HQMQ_ERR_UNSUPPORTED;
    if (p->S < 1 || p->S > kMaxS || p->b_r < 1 || p->b_r > 8)
        return HQMQ_ERR_UNSUPPORTED;
    if (!(p->flags & HQMQ_FLAG_NO_OUTLIERS) && !(std::isfinite(p->C) && p->C > 0.f))
        return HQMQ_ERR_UNSUPPORTED;
    if (p->stride_b < 0 || p->stride_h < 0 || p->stride_t < p->D)
        return HQMQ_ERR_INVALID_ARG;
    // D = 128 runs the kernels written for full rows: 16-byte accesses, every row aligned to them
    if (p->D == 4 * kChunksPerRow && ((p->stride_b % 8) || (p->stride_h % 8) || (p->stride_t % 8)))
        return HQMQ_ERR_INVALID_ARG;
    if ((int64_t)p->B * p->H > 65535)
        return HQMQ_ERR_UNSUPPORTED;  // grid.y
    const uint64_t n_rows = (uint64_t)p->B * p->H * p->T;
    if (n_rows * kChunksPerRow >= (1ull << 32))
        return HQMQ_ERR_UNSUPPORTED;  // 32-bit outlier offsets and ranks
    return HQMQ_OK;
}

static Geometry make_geometry(const hqmq_params *p)
{
    Geometry g;
    g.B = p->B;
    g.H = p->H;
    g.T = p->T;
    g.D = p->D;
    g.n_c = (p->D + 3) / 4;
    g.n_c_magic = g.n_c >= 2 ? (uint32_t)((1ull << 32) / (uint64_t)g.n_c + 1ull) : 0u;
    g.vec_ok = (p->D % 4 == 0 && p->stride_b % 4 == 0 && p->stride_h % 4 == 0 && p->stride_t % 4 == 0) ? 1 : 0;
    g.S = p->S;
    g.S16 = (p->S + 15) / 16;
    g.A16 = p->S <= kScreenMaxS ? g.S16 : 0;
    g.b_r = p->b_r;
    g.w_idx = index_bits(p->S);
    g.w = g.w_idx + p->b_r;
    g.row_words = (g.n_c * g.w + 31) / 32;
    g.sb = p->stride_b;
    g.sh = p->stride_h;
    g.st = p->stride_t;
    g.inv_S = (1.0f / (float)p->S) * (1.0f + 0x1.0p-18f);
    g.inv_L = 1.0f / (float)((1 << p->b_r) - 1);
    g.log2_S = -1;
    for (int j = 0; j < 16; ++j)
        if ((1 << j) == p->S)
            g.log2_S = j;
    g.check_finite = (p->flags & HQMQ_FLAG_CHECK_FINITE) ? 1 : 0;
    g.fused_by_head = 0;
    g.select_sampled = 0;
    {
        // the sampled select keeps the keys of a few bins around the median: about 2 % of a head's chunks
        const uint64_t n_h = (uint64_t)p->B * p->T * g.n_c;
        const uint64_t want = (n_h / 32 + 1023) / 1024 * 1024;
        g.cand_cap = (int32_t)(want > (uint64_t)kCandCap ? want : (uint64_t)kCandCap);
    }
    g.search_rows = search_rows_for(p->T, g.S16, g.A16, g.D, g.row_words);
    g.n_search_blocks_per_seg = (uint32_t)((p->T + g.search_rows - 1) / g.search_rows);
    return g;
}

struct WorkspaceLayout {
    uint64_t state, thr, hist0, hist1, plan, cand_count, cand, block_sum, block_pre, aop, total;
};

static WorkspaceLayout workspace_layout(const Geometry &g)
{
    WorkspaceLayout l;
    uint64_t off = 0;
    const uint64_t n_blocks = (uint64_t)g.B * g.H * g.n_search_blocks_per_seg;
    auto take = [&](uint64_t bytes) {
        const uint64_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    l.state = take((uint64_t)g.H * sizeof(SelectState));
    l.thr = take((uint64_t)g.H * sizeof(double));
    l.hist0 = take((uint64_t)g.H * kBins0 * sizeof(uint32_t));
    l.hist1 = take((uint64_t)g.H * kBins1 * sizeof(uint32_t));
    l.plan = take((uint64_t)g.H * sizeof(SelectPlan));
    l.cand_count = take((uint64_t)g.H * 3 * sizeof(uint32_t));
    l.cand = take((uint64_t)g.H * g.cand_cap * sizeof(unsigned long long));
    l.block_sum = take(n_blocks * sizeof(uint32_t));
    l.block_pre = take(n_blocks * sizeof(uint32_t));
    l.aop = take((uint64_t)g.H * g.A16 * kATiles * 64 * 16);
    l.total = off;
    return l;
}

static bool misaligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }

static int32_t check_encoded(const hqmq_encoded *e, bool need_counts, uint64_t outlier_capacity)
{
    if (!e || !e->codes || !e->sigma || !e->flags || !e->row_off)
        return HQMQ_ERR_INVALID_ARG;
    if (outlier_capacity > 0 && !e->outliers)
        return HQMQ_ERR_INVALID_ARG;  // an empty list needs no storage
    if (need_counts && (!e->n_outliers || !e->status))
        return HQMQ_ERR_INVALID_ARG;
    if (misaligned(e->codes, 4) || misaligned(e->sigma, 2) || misaligned(e->flags, 4) ||
        misaligned(e->row_off, 4) || misaligned(e->outliers, 8))
        return HQMQ_ERR_INVALID_ARG;
    if (need_counts && (misaligned(e->n_outliers, 4) || misaligned(e->status, 4)))
        return HQMQ_ERR_INVALID_ARG;
    return HQMQ_OK;
}

static EncodedPtrs to_ptrs(const hqmq_encoded *e)
{
    EncodedPtrs p;
    p.codes = e->codes;
    p.sigma = e->sigma;
    p.flags = e->flags;
    p.row_off = e->row_off;
    p.outliers = e->outliers;
    p.n_outliers = e->n_outliers;
    p.status = e->status;
    return p;
}

static int32_t hip_failed(hipError_t err)
{
    g_last_hip_error = (int32_t)err;
    return HQMQ_ERR_HIP;
}

}  // namespace hqmq

using namespace hqmq;

extern "C" int32_t hqmq_last_hip_error(void) { return g_last_hip_error; }

extern "C" int32_t hqmq_init(void)
{
    const hipError_t err = ensure_device_setup();
    return err == hipSuccess ? HQMQ_OK : hip_failed(err);
}

extern "C" int32_t hqmq_sizes(const hqmq_params *params, hqmq_size_info *out)
{
    if (!out)
        return HQMQ_ERR_INVALID_ARG;
    int32_t rc = check_params(params);
    if (rc != HQMQ_OK)
        return rc;
    const Geometry g = make_geometry(params);
    std::memset(out, 0, sizeof(*out));
    const uint64_t n_rows = (uint64_t)g.B * g.H * g.T;
    out->n_rows = n_rows;
    out->index_bits = (uint32_t)g.w_idx;
    out->code_bits = (uint32_t)g.w;
    out->code_words_per_row = (uint32_t)g.row_words;
    out->chunks_per_row = (uint32_t)g.n_c;
    out->code_bytes = n_rows * (uint64_t)g.row_words * 4;
    out->sigma_bytes = n_rows * 2;
    out->flag_bytes = n_rows * 4;
    out->row_off_bytes = (n_rows + 1) * 4;
    out->n_outliers_bytes = ((uint64_t)g.H + 1) * 4;
    out->status_bytes = 4;
    // A chunk is flagged when r^2 > C^2 * median.  For C >= 1 that needs r^2 above the lower
    // median of its head, which at most floor(n_h / 2) chunks are; for C < 1 any chunk may be.
    const uint64_t n_h = (uint64_t)g.B * g.T * g.n_c;
    uint64_t cap = (uint64_t)g.H * n_h;
    if (params->flags & HQMQ_FLAG_NO_OUTLIERS)
        cap = 0;
    else if (params->C >= 1.0f)
        cap = (uint64_t)g.H * (n_h / 2);
    out->outlier_capacity_max = cap;
    out->outlier_bytes_max = cap * 8;
    out->workspace_bytes = workspace_layout(g).total;
    return HQMQ_OK;
}

static WorkspaceOffsets workspace_offsets(const WorkspaceLayout &l)
{
    WorkspaceOffsets o;
    o.state = (uint32_t)l.state;
    o.thr = (uint32_t)l.thr;
    o.hist0 = (uint32_t)l.hist0;
    o.hist1 = (uint32_t)l.hist1;
    o.plan = (uint32_t)l.plan;
    o.cand_count = (uint32_t)l.cand_count;
    o.cand = (uint32_t)l.cand;
    o.block_sum = (uint32_t)l.block_sum;
    o.block_pre = (uint32_t)l.block_pre;
    o.aop = (uint32_t)l.aop;
    return o;
}

// Encode n_tensors tensors of one shape: up to kMaxEncodeBatch of them share each kernel launch
// (select -> search -> outlier list per group); a group's tensor i uses slice i of the workspace.
static int32_t encode_impl(const hqmq_params *params, int32_t n_tensors, const void *const *x_dev,
                           const float *const *sec_dev, const hqmq_encoded *enc,
                           const uint64_t *outlier_capacity, void *workspace_dev, uint64_t workspace_bytes,
                           void *stream, void *const *phase_events, const double *const *thr_given = nullptr,
                           bool static_scratch = false)
{
    int32_t rc = check_params(params);
    if (rc != HQMQ_OK)
        return rc;
    if (n_tensors <= 0 || !x_dev || !sec_dev || !enc || !outlier_capacity)
        return HQMQ_ERR_INVALID_ARG;
    if (static_scratch)  // the library's own array stands in for the caller's workspace
        workspace_bytes = HQMQ_STATIC_SCRATCH_BYTES;
    else if (!workspace_dev || misaligned(workspace_dev, 256))
        return HQMQ_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (!x_dev[i] || !sec_dev[i] || misaligned(x_dev[i], 16) || misaligned(sec_dev[i], 16))
            return HQMQ_ERR_INVALID_ARG;
        rc = check_encoded(&enc[i], true, outlier_capacity[i]);
        if (rc != HQMQ_OK)
            return rc;
    }
    const Geometry g = make_geometry(params);
    const WorkspaceLayout l = workspace_layout(g);
    const int group = n_tensors < kMaxEncodeBatch ? n_tensors : kMaxEncodeBatch;
    if (workspace_bytes < l.total * (uint64_t)group)
        return HQMQ_ERR_BUFFER_TOO_SMALL;
    if (l.total >= (1ull << 32))
        return HQMQ_ERR_UNSUPPORTED;  // 32-bit offsets inside a slice
    const WorkspaceOffsets wo = workspace_offsets(l);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool no_outliers = (params->flags & HQMQ_FLAG_NO_OUTLIERS) != 0;
    if (thr_given) {
        if (no_outliers)
            return HQMQ_ERR_INVALID_ARG;
        for (int32_t i = 0; i < n_tensors; ++i)
            if (!thr_given[i] || misaligned(thr_given[i], 8))
                return HQMQ_ERR_INVALID_ARG;
    }
    {
        void *own = nullptr;
        const hipError_t ready = ensure_device_setup(&own);
        if (ready != hipSuccess)
            return hip_failed(ready);
        if (static_scratch)
            workspace_dev = own;
    }
    auto mark = [&](int i) -> hipError_t {
        if (phase_events && phase_events[i])
            return hipEventRecord(static_cast<hipEvent_t>(phase_events[i]), st);
        return hipSuccess;
    };
    for (int32_t first = 0; first < n_tensors; first += kMaxEncodeBatch) {
        const int n = (n_tensors - first < kMaxEncodeBatch) ? n_tensors - first : kMaxEncodeBatch;
        EncodeBatch batch;
        std::memset(&batch, 0, sizeof(batch));
        for (int i = 0; i < n; ++i) {
            EncodeTensor &t = batch.t[i];
            t.x = static_cast<const _Float16 *>(x_dev[first + i]);
            t.sec = sec_dev[first + i];
            t.enc = to_ptrs(&enc[first + i]);
            t.ws = static_cast<char *>(workspace_dev) + l.total * (uint64_t)i;
            t.outlier_capacity = outlier_capacity[first + i];
            t.thr_given = thr_given ? thr_given[first + i] : nullptr;
        }
        hipError_t err = first == 0 ? mark(0) : hipSuccess;
        if (err != hipSuccess)
            return hip_failed(err);
        // A tensor of a few rows whose thresholds are known beforehand (appended tokens, extraction off)
        // takes two launches: the fused search, then one workgroup per tensor for the outlier list.
        const uint64_t n_rows_t = (uint64_t)g.B * g.H * g.T;
        const uint64_t n_blocks_t = (uint64_t)g.B * g.H * g.n_search_blocks_per_seg;
        const bool fused = (no_outliers || thr_given != nullptr) && n_rows_t <= (uint64_t)kSmallListRows &&
                           n_blocks_t <= (uint64_t)kSmallListBlocks && search_fused_available(g);
        if (fused) {
            // several batch entries whose rows together fill no more than one pass of the workgroup's waves (rows
            // of 128 elements): a workgroup per head takes them all, and builds the head's tables once instead
            // of once per batch entry; more rows than that are faster on workgroups of their own
            Geometry gf = g;
            const int waves = search_waves_for(g.S16, g.A16, g.D, g.row_words, g.search_rows);
            gf.fused_by_head = (g.B > 1 && (int64_t)g.B * g.T <= 2 * waves && g.D == 4 * kChunksPerRow) ? 1 : 0;
            err = mark(1);
            if (err == hipSuccess)
                err = launch_search_fused(gf, wo, batch, n, st);
            if (err == hipSuccess)
                err = mark(2);
            if (err == hipSuccess)
                err = launch_outlier_list_small(g, wo, batch, n, st);
            if (err == hipSuccess)
                err = mark(3);
            if (err != hipSuccess)
                return hip_failed(err);
            continue;
        }
        err = launch_select_median(g, wo, batch, n, params->C, no_outliers || thr_given != nullptr, st);
        if (err == hipSuccess)
            err = mark(1);
        if (err != hipSuccess)
            return hip_failed(err);
        err = launch_search(g, wo, batch, n, st);
        if (err == hipSuccess)
            err = mark(2);
        if (err != hipSuccess)
            return hip_failed(err);
        err = launch_outlier_list(g, wo, batch, n, st);
        if (err == hipSuccess)
            err = mark(3);
        if (err != hipSuccess)
            return hip_failed(err);
    }
    return HQMQ_OK;
}

extern "C" int32_t hqmq_encode(const hqmq_params *params, const void *x_dev, const float *sec_dev,
                               const hqmq_encoded *enc, uint64_t outlier_capacity,
                               void *workspace_dev, uint64_t workspace_bytes, void *stream)
{
    return encode_impl(params, 1, &x_dev, &sec_dev, enc, &outlier_capacity, workspace_dev, workspace_bytes,
                       stream, nullptr);
}

extern "C" int32_t hqmq_encode_static(const hqmq_params *params, const void *x_dev, const float *sec_dev,
                                      const hqmq_encoded *enc, uint64_t outlier_capacity, void *stream)
{
    return encode_impl(params, 1, &x_dev, &sec_dev, enc, &outlier_capacity, nullptr, 0, stream, nullptr, nullptr,
                       true);
}

extern "C" int32_t hqmq_encode_timed(const hqmq_params *params, const void *x_dev,
                                     const float *sec_dev, const hqmq_encoded *enc,
                                     uint64_t outlier_capacity, void *workspace_dev,
                                     uint64_t workspace_bytes, void *stream, void *const *phase_events)
{
    return encode_impl(params, 1, &x_dev, &sec_dev, enc, &outlier_capacity, workspace_dev, workspace_bytes,
                       stream, phase_events);
}

// the multiplier is not used when the thresholds are final
static int32_t params_for_given_thresholds(const hqmq_params *params, hqmq_params *out)
{
    if (!params)
        return HQMQ_ERR_INVALID_ARG;
    *out = *params;
    if (!(out->flags & HQMQ_FLAG_NO_OUTLIERS))
        out->C = 1.0f;
    return HQMQ_OK;
}

extern "C" int32_t hqmq_encode_given_thresholds(const hqmq_params *params, const void *x_dev,
                                                const float *sec_dev, const double *thr_dev,
                                                const hqmq_encoded *enc, uint64_t outlier_capacity,
                                                void *workspace_dev, uint64_t workspace_bytes, void *stream)
{
    hqmq_params p;
    int32_t rc = params_for_given_thresholds(params, &p);
    if (rc != HQMQ_OK)
        return rc;
    if (!thr_dev)
        return HQMQ_ERR_INVALID_ARG;
    return encode_impl(&p, 1, &x_dev, &sec_dev, enc, &outlier_capacity, workspace_dev, workspace_bytes, stream,
                       nullptr, &thr_dev);
}

extern "C" int32_t hqmq_encode_batch_given_thresholds(const hqmq_params *params, int32_t n_tensors,
                                                      const void *const *x_dev, const float *const *sec_dev,
                                                      const double *const *thr_dev, const hqmq_encoded *enc,
                                                      const uint64_t *outlier_capacity, void *workspace_dev,
                                                      uint64_t workspace_bytes, void *stream)
{
    hqmq_params p;
    int32_t rc = params_for_given_thresholds(params, &p);
    if (rc != HQMQ_OK)
        return rc;
    if (!thr_dev)
        return HQMQ_ERR_INVALID_ARG;
    return encode_impl(&p, n_tensors, x_dev, sec_dev, enc, outlier_capacity, workspace_dev, workspace_bytes,
                       stream, nullptr, thr_dev);
}

extern "C" int32_t hqmq_thresholds(const hqmq_params *params, const void *workspace_dev, uint64_t workspace_bytes,
                                   int32_t slice, double *thr_out_dev, void *stream)
{
    int32_t rc = check_params(params);
    if (rc != HQMQ_OK)
        return rc;
    if (!workspace_dev || !thr_out_dev || slice < 0 || slice >= kMaxEncodeBatch ||
        misaligned(workspace_dev, 256) || misaligned(thr_out_dev, 8))
        return HQMQ_ERR_INVALID_ARG;
    const WorkspaceLayout l = workspace_layout(make_geometry(params));
    if (workspace_bytes < l.total * ((uint64_t)slice + 1))
        return HQMQ_ERR_BUFFER_TOO_SMALL;  // the slice lies (partly) outside the caller's workspace
    const char *src = static_cast<const char *>(workspace_dev) + l.total * (uint64_t)slice + l.thr;
    hipError_t err = hipMemcpyAsync(thr_out_dev, src, (size_t)params->H * sizeof(double), hipMemcpyDeviceToDevice,
                                    static_cast<hipStream_t>(stream));
    if (err != hipSuccess)
        return hip_failed(err);
    return HQMQ_OK;
}

extern "C" int32_t hqmq_shard_median_region(const hqmq_params *params, int32_t pass, uint64_t *offset_bytes,
                                            uint64_t *n_counters)
{
    int32_t rc = check_params(params);
    if (rc != HQMQ_OK)
        return rc;
    if (pass < 0 || pass > 5 || !offset_bytes || !n_counters)
        return HQMQ_ERR_INVALID_ARG;
    const WorkspaceLayout l = workspace_layout(make_geometry(params));
    *offset_bytes = pass == 0 ? l.hist0 : l.hist1;
    *n_counters = (uint64_t)params->H * (pass == 0 ? kBins0 : kBins1);
    return HQMQ_OK;
}

extern "C" int32_t hqmq_shard_median_pass(const hqmq_params *params, uint64_t total_chunks_per_head, int32_t pass,
                                          const void *x_dev, void *workspace_dev, uint64_t workspace_bytes,
                                          void *stream)
{
    int32_t rc = check_params(params);
    if (rc != HQMQ_OK)
        return rc;
    if (pass < 0 || pass > 6 || !workspace_dev || misaligned(workspace_dev, 256))
        return HQMQ_ERR_INVALID_ARG;
    if (pass < 6 && (!x_dev || misaligned(x_dev, 16)))  // the finish reads no rows
        return HQMQ_ERR_INVALID_ARG;
    if (params->flags & HQMQ_FLAG_NO_OUTLIERS)
        return HQMQ_ERR_INVALID_ARG;
    const Geometry g = make_geometry(params);
    const uint64_t own = (uint64_t)g.B * g.T * g.n_c;
    if (total_chunks_per_head < own)
        return HQMQ_ERR_INVALID_ARG;
    if (total_chunks_per_head >= (1ull << 32))
        return HQMQ_ERR_UNSUPPORTED;  // 32-bit ranks and counters
    const WorkspaceLayout l = workspace_layout(g);
    if (workspace_bytes < l.total)
        return HQMQ_ERR_BUFFER_TOO_SMALL;
    EncodeBatch batch;
    std::memset(&batch, 0, sizeof(batch));
    batch.t[0].x = static_cast<const _Float16 *>(x_dev);
    batch.t[0].ws = static_cast<char *>(workspace_dev);
    hipError_t err = launch_shard_median_pass(g, workspace_offsets(l), batch, pass, total_chunks_per_head, params->C,
                                              static_cast<hipStream_t>(stream));
    if (err != hipSuccess)
        return hip_failed(err);
    return HQMQ_OK;
}

extern "C" int32_t hqmq_encode_batch(const hqmq_params *params, int32_t n_tensors, const void *const *x_dev,
                                     const float *const *sec_dev, const hqmq_encoded *enc,
                                     const uint64_t *outlier_capacity, void *workspace_dev,
                                     uint64_t workspace_bytes, void *stream, void *const *phase_events)
{
    return encode_impl(params, n_tensors, x_dev, sec_dev, enc, outlier_capacity, workspace_dev, workspace_bytes,
                       stream, phase_events);
}

static int32_t decode_impl(const hqmq_params *params, int32_t n_tensors, const hqmq_encoded *enc,
                           const uint64_t *outlier_capacity, const float *const *sec_dev,
                           void *const *out_dev, void *stream)
{
    int32_t rc = check_params(params);
    if (rc != HQMQ_OK)
        return rc;
    if (n_tensors <= 0 || !enc || !outlier_capacity || !sec_dev || !out_dev)
        return HQMQ_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (!sec_dev[i] || !out_dev[i] || misaligned(out_dev[i], 16) || misaligned(sec_dev[i], 16))
            return HQMQ_ERR_INVALID_ARG;
        rc = check_encoded(&enc[i], false, outlier_capacity[i]);
        if (rc != HQMQ_OK)
            return rc;
    }
    const Geometry g = make_geometry(params);
    for (int32_t first = 0; first < n_tensors; first += kMaxDecodeBatch) {
        const int n = (n_tensors - first < kMaxDecodeBatch) ? n_tensors - first : kMaxDecodeBatch;
        DecodeBatch batch;
        std::memset(&batch, 0, sizeof(batch));
        for (int i = 0; i < n; ++i) {
            const hqmq_encoded &e = enc[first + i];
            DecodeTensor &t = batch.t[i];
            t.codes = e.codes;
            t.sigma = e.sigma;
            t.flags = e.flags;
            t.row_off = e.row_off;
            t.outliers = e.outliers;
            t.sec = sec_dev[first + i];
            t.out = static_cast<_Float16 *>(out_dev[first + i]);
            t.outlier_capacity = outlier_capacity[first + i];
        }
        hipError_t err = launch_decode(g, batch, n, static_cast<hipStream_t>(stream));
        if (err != hipSuccess)
            return hip_failed(err);
    }
    return HQMQ_OK;
}

extern "C" int32_t hqmq_decode(const hqmq_params *params, const hqmq_encoded *enc,
                               uint64_t outlier_capacity, const float *sec_dev, void *out_dev,
                               void *stream)
{
    return decode_impl(params, 1, enc, &outlier_capacity, &sec_dev, &out_dev, stream);
}

extern "C" int32_t hqmq_decode_batch(const hqmq_params *params, int32_t n_tensors,
                                     const hqmq_encoded *enc, const uint64_t *outlier_capacity,
                                     const float *const *sec_dev, void *const *out_dev, void *stream)
{
    return decode_impl(params, n_tensors, enc, outlier_capacity, sec_dev, out_dev, stream);
}

static int32_t check_attend(const hqmq_params *params, int32_t n_q_heads)
{
    int32_t rc = check_params(params);
    if (rc != HQMQ_OK)
        return rc;
    if (n_q_heads <= 0 || n_q_heads % params->H)
        return HQMQ_ERR_INVALID_ARG;
    if (params->D != 128 && params->D != 96 && params->D != 64)
        return HQMQ_ERR_UNSUPPORTED;  // the attention kernel takes the head dimensions of the paper's models
    if (n_q_heads / params->H > kMaxGroup)
        return HQMQ_ERR_UNSUPPORTED;
    return HQMQ_OK;
}

extern "C" uint64_t hqmq_attend_workspace_bytes(const hqmq_params *params, int32_t n_q_heads)
{
    if (check_attend(params, n_q_heads) != HQMQ_OK)
        return 0;
    return plan_attend(make_geometry(params), n_q_heads / params->H, (params->flags & HQMQ_FLAG_ATTEND_TABLES) != 0)
        .total_bytes;
}

static int32_t attend_impl(const hqmq_params *params, int32_t n_q_heads, const void *q_dev,
                           float scale, const hqmq_encoded *enc_k, uint64_t cap_k,
                           const float *sec_k_dev, const hqmq_encoded *enc_v, uint64_t cap_v,
                           const float *sec_v_dev, void *out_dev, float *lse_dev, const int32_t *visible_dev,
                           void *workspace_dev, uint64_t workspace_bytes, void *stream)
{
    int32_t rc = check_attend(params, n_q_heads);
    if (rc != HQMQ_OK)
        return rc;
    if (!q_dev || !out_dev || !sec_k_dev || !sec_v_dev || !workspace_dev || !std::isfinite(scale))
        return HQMQ_ERR_INVALID_ARG;
    if (misaligned(q_dev, 16) || misaligned(out_dev, 16) || misaligned(sec_k_dev, 16) ||
        misaligned(sec_v_dev, 16) || misaligned(workspace_dev, 256))
        return HQMQ_ERR_INVALID_ARG;
    rc = check_encoded(enc_k, false, cap_k);
    if (rc == HQMQ_OK)
        rc = check_encoded(enc_v, false, cap_v);
    if (rc != HQMQ_OK)
        return rc;
    const Geometry g = make_geometry(params);
    const int G = n_q_heads / params->H;
    const AttendPlan plan = plan_attend(g, G, (params->flags & HQMQ_FLAG_ATTEND_TABLES) != 0);
    if (workspace_bytes < plan.total_bytes)
        return HQMQ_ERR_BUFFER_TOO_SMALL;
    {  // the kernels may ask for more LDS than a launch gets by default (large S)
        const hipError_t ready = ensure_device_setup();
        if (ready != hipSuccess)
            return hip_failed(ready);
    }

    auto side = [](const hqmq_encoded *e, const float *sec, uint64_t cap) {
        AttendSide s;
        s.codes = e->codes;
        s.sigma = e->sigma;
        s.flags = e->flags;
        s.row_off = e->row_off;
        s.outliers = e->outliers;
        s.sec = sec;
        s.outlier_capacity = cap;
        return s;
    };
    AttendArgs a;
    a.k = side(enc_k, sec_k_dev, cap_k);
    a.v = side(enc_v, sec_v_dev, cap_v);
    a.q = static_cast<const _Float16 *>(q_dev);
    a.out = static_cast<_Float16 *>(out_dev);
    a.lse = lse_dev;
    a.visible = visible_dev;
    a.part_ml = reinterpret_cast<float *>(workspace_dev);
    a.part_acc = reinterpret_cast<float *>(static_cast<char *>(workspace_dev) + plan.ml_bytes);
    a.qscale = scale * 1.44269504088896340736f;
    a.G = G;
    a.D = params->D;
    a.n_splits = plan.n_splits;
    a.rows_per_split = plan.rows_per_split;
    a.joint = plan.joint;
    hipError_t err = launch_attend(g, a, static_cast<hipStream_t>(stream));
    if (err != hipSuccess)
        return hip_failed(err);
    return HQMQ_OK;
}

extern "C" int32_t hqmq_attend(const hqmq_params *params, int32_t n_q_heads, const void *q_dev,
                               float scale, const hqmq_encoded *enc_k, uint64_t cap_k,
                               const float *sec_k_dev, const hqmq_encoded *enc_v, uint64_t cap_v,
                               const float *sec_v_dev, void *out_dev, void *workspace_dev,
                               uint64_t workspace_bytes, void *stream)
{
    return attend_impl(params, n_q_heads, q_dev, scale, enc_k, cap_k, sec_k_dev, enc_v, cap_v, sec_v_dev, out_dev,
                       nullptr, nullptr, workspace_dev, workspace_bytes, stream);
}

extern "C" int32_t hqmq_attend_lse(const hqmq_params *params, int32_t n_q_heads, const void *q_dev,
                                   float scale, const hqmq_encoded *enc_k, uint64_t cap_k,
                                   const float *sec_k_dev, const hqmq_encoded *enc_v, uint64_t cap_v,
                                   const float *sec_v_dev, void *out_dev, float *lse_dev, void *workspace_dev,
                                   uint64_t workspace_bytes, void *stream)
{
    if (!lse_dev || misaligned(lse_dev, 4))
        return HQMQ_ERR_INVALID_ARG;
    return attend_impl(params, n_q_heads, q_dev, scale, enc_k, cap_k, sec_k_dev, enc_v, cap_v, sec_v_dev, out_dev,
                       lse_dev, nullptr, workspace_dev, workspace_bytes, stream);
}

extern "C" int32_t hqmq_attend_masked(const hqmq_params *params, int32_t n_q_heads, const void *q_dev,
                                      float scale, const hqmq_encoded *enc_k, uint64_t cap_k,
                                      const float *sec_k_dev, const hqmq_encoded *enc_v, uint64_t cap_v,
                                      const float *sec_v_dev, const int32_t *visible_dev, void *out_dev,
                                      float *lse_dev, void *workspace_dev, uint64_t workspace_bytes, void *stream)
{
    if (!visible_dev || misaligned(visible_dev, 4) || misaligned(lse_dev, 4))
        return HQMQ_ERR_INVALID_ARG;
    return attend_impl(params, n_q_heads, q_dev, scale, enc_k, cap_k, sec_k_dev, enc_v, cap_v, sec_v_dev, out_dev,
                       lse_dev, visible_dev, workspace_dev, workspace_bytes, stream);
}
