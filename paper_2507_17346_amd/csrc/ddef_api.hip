// C-ABI of the DD-EF-SGD hot path: context, state machine, launch sequences.
// Every step of the path runs in the kernels of ddef_kernels.hip; this file validates
// arguments, owns the device memory and enqueues launches on the context's stream.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "ddef.h"
#include "ddef_kernels.h"

using namespace ddef;

namespace {

enum Phase { PH_IDLE = 0, PH_GRAD = 1, PH_COMPRESSED = 2, PH_AGGREGATED = 3 };

enum Slot {
    SL_GRAD = 0, SL_EF_FILTER, SL_EF_FILTER_FUSED, SL_RANDK_MARK, SL_RANDK_BIN, SL_RANDK_FILL, SL_EF_RANDK, SL_TAB_SUM, SL_TAB_DECIDE, SL_TAB_ORDER, SL_SEL_BEGIN_ROWS,
    SL_DIGIT_HIST, SL_DIGIT_PICK, SL_CHUNK_COUNT, SL_CHUNK_SCAN, SL_CHUNK_EMIT, SL_QUANTIZE4, SL_SAMPLE, SL_FILL,
    SL_MSG_OFFSETS, SL_AGGREGATE_TILES, SL_AGGREGATE_APPLY, SL_ADVANCE, SL_APPLY, SL_COPY_PROBE, SL_OBJECTIVE,
    SL_EF_FILTER_SPLIT, SL_RESTORE_SURE, SL_MESSAGE_MERGE, SL_COMPOSED_REPEAT, SL_COUNT
};
const char* const kSlotNames[SL_COUNT] = {
    "k_grad", "k_ef_filter", "k_ef_filter_fused", "k_randk_mark", "k_randk_bin", "k_randk_fill", "k_ef_randk", "k_tab_sum", "k_tab_decide", "k_tab_order",
    "k_sel_begin_rows", "k_digit_hist", "k_digit_pick", "k_chunk_count", "k_chunk_scan", "k_chunk_emit", "k_quantize4",
    "k_sample", "k_fill_f4", "k_msg_offsets", "k_aggregate_tiles", "k_aggregate_apply_tiles", "k_advance", "k_apply", "k_copy_f4", "k_objective",
    "k_ef_filter_split", "k_restore_sure", "k_message_merge", "composed_repeat_pass"};

struct ProfRecord { int slot; hipEvent_t start, stop; };

}  // namespace

struct ddef_ctx {
    int device = 0;
    int cus = 256;
    hipStream_t own_stream = nullptr, stream = nullptr;
    uint64_t d = 0, ld = 0, t = 0;
    uint32_t n = 0, tau_max = 0, tau = 0, nchunks = 0;
    float *lambda = nullptr, *xstar = nullptr, *ring = nullptr, *e = nullptr, *g = nullptr, *U = nullptr;
    // messages: [q_slots][n][msg_ld].  Ring form keeps one slot (the messages of this iteration);
    // queue form keeps the messages of the last tau_max+1 iterations, slot = iteration % q_slots,
    // q_k[slot] entries per worker
    uint32_t* msg_idx = nullptr;
    float* msg_val = nullptr;
    uint64_t msg_ld = 0;
    bool queue_form = false;
    uint32_t ring_slots = 1, q_slots = 1;
    uint32_t msg_slot = 0;               // slot of the messages ddef_ef_compress wrote last
    std::vector<uint64_t> q_k;
    SelState* sel = nullptr;
    uint32_t *hist = nullptr, *cnt_gt = nullptr, *cnt_eq = nullptr;
    // candidate filter: per-worker words [bound | overflow | stat_full | cand_total | nonfinite | zero_at |
    // sure_at | sure_total | msg_count] (the last three serve the sure / band split of dense messages), slot
    // counters [n][kSubs], the run table per 256-entry group with its prefixes, and the
    // candidate buffers of `cap` entries per worker
    uint32_t* filt = nullptr;
    uint32_t* cand_count = nullptr;
    uint2* tab = nullptr;
    uint32_t* span_sum = nullptr;
    uint32_t nwc = 0, nspans = 0;
    uint2* cand = nullptr;
    uint32_t* sorted_idx = nullptr;
    float* sorted_val = nullptr;
    uint64_t cap = 0;
    // Dense messages whose bound comes from a sample of this very p are split: candidates sure to be
    // sent are recorded as runs in `sure` (run table `stab`, slot counters `sure_count`) and go to
    // the aggregation as they are; only the band around the expected threshold is ordered, searched
    // and compacted into the message row.  msg_split: the last messages have that two-part form;
    // agg_split: so have the ones named by the last ddef_aggregate.  canon_*: one worker's message
    // in its canonical form, put together when ddef_get_message asks for it.
    uint2* sure = nullptr;
    uint2* stab = nullptr;
    uint32_t* sure_count = nullptr;
    uint64_t sure_cap = 0;
    bool msg_split = false, agg_split = false;
    uint32_t* canon_idx = nullptr;
    float* canon_val = nullptr;
    uint64_t canon_ld = 0;
    int64_t opt_split = 1;
    bool have_bound = false;
    uint64_t bound_k = 0;                // the k the bound was placed for
    uint64_t sel_k = 0;                  // k of the last completed Top-k selection and how many in a row
    uint32_t sel_run = 0;                //   had it (the threshold trend needs two)
    float* sample = nullptr;             // [n][sample_ld] strided sample of p (bound_from_sample)
    uint32_t* sample_total = nullptr;
    uint64_t sample_ld = 0;
    int compressor = DDEF_COMPRESSOR_TOPK;
    // gradient prefetch: the gradient of iteration t+1 only needs x_{t+1-tau}, which exists as soon
    // as iteration t starts (tau >= 1), so it is generated on a second stream into a second buffer
    // while the memory-bound rest of iteration t runs
    int64_t opt_prefetch = 0;
    // fused gradient: ddef_grad launches nothing, the accumulate pass generates the gradient in
    // registers; grad_pending is true from ddef_grad until something needs g in memory
    int64_t opt_fuse = 0;
    bool grad_pending = false, grad_live = false, grad_stored = false;
    float* g_next = nullptr;
    hipStream_t side = nullptr;
    hipEvent_t ev_applied = nullptr, ev_prefetched = nullptr;
    bool pf_valid = false;
    uint64_t pf_t = 0;
    uint32_t pf_tau = 0;
    uint32_t* bitmap = nullptr;          // Random-k: one bit per coordinate, [n][ld/32], all-zero between steps
    double* objective_partial = nullptr; // ddef_objective: one partial sum per block
    uint32_t* region_count = nullptr;    // Random-k, binned marking: [n][2048] bucket fill counts, all-zero between steps
    // composed compressor: share of the coordinates its Random-k stage keeps, and the wire form of
    // the last message: codes [n][codes_ld] bytes (two entries each), steps [n][codes_ld/128] floats
    double rand_ratio = 0.2;
    uint8_t* codes = nullptr;
    float* steps = nullptr;
    uint64_t codes_ld = 0;
    bool codes_valid = false;
    // The messages are summed tile by tile in LDS by ddef_apply_delayed, in the pass that updates
    // the model; ddef_aggregate only locates each tile's entries (agg_off: [n][ld/kTile + 1]
    // message offsets at the tile boundaries).  agg_deferred holds from ddef_aggregate to the next
    // ddef_ef_compress (the messages are intact that long); U is computed on its own only when
    // somebody asks for it (agg_in_U).  u_zero: U is known to be all-zero.
    uint32_t* agg_off = nullptr;
    uint32_t ntiles = 0;
    bool agg_deferred = false, agg_in_U = false, u_zero = true;
    uint32_t agg_slot = 0;
    Phase phase = PH_IDLE;
    bool problem_set = false, step_empty = true;
    float lr_step = 0.0f;
    uint64_t k_step = 0;
    uint64_t seed = 0;
    int noise_kind = 0;
    float noise_scale = 0.0f;
    float zeta = 0.0f;
    int sticky = DDEF_OK;
    uint64_t full_selects = 0;
    int64_t opt_force_full = 0, opt_slack_x16 = 40;
    int64_t opt_bucket_percent = 0;      // Random-k buckets: 0 = expected fill plus slack, else that share of it
    int64_t opt_composed_bound = 1;      // composed compressor: 1 record only the kept entries above a sampled bound
    // ddef_step as a captured graph: the launches of one steady iteration, replayed while
    // (k, lr, tau) stay the same.  Inside the graph the iteration number comes from t_dev.
    int64_t opt_graph = 0;
    uint64_t* t_dev = nullptr;
    uint64_t t_dev_value = ~0ull;        // what *t_dev holds (host's record)
    hipGraphExec_t graph_exec = nullptr;
    bool capturing = false;
    uint64_t graph_k = 0;
    uint32_t graph_lr_bits = 0, graph_tau = 0;
    uint64_t graph_full_selects = 0;     // whole-row selections per replayed iteration
    uint64_t graph_replays = 0;
    bool profiling = false;
    std::vector<ProfRecord> pending;
    std::vector<hipEvent_t> free_events;
    uint64_t prof_launches[SL_COUNT] = {};
    double prof_ms[SL_COUNT] = {};

    float* slot(uint64_t step) const { return ring + (step % (uint64_t)ring_slots) * ld; }
    uint32_t* slot_idx(uint32_t s) const { return msg_idx + (uint64_t)s * n * msg_ld; }
    float* slot_val(uint32_t s) const { return msg_val + (uint64_t)s * n * msg_ld; }
    // The gradient of the iteration in progress: ring form takes it at the snapshot x_{t-tau} with
    // the noise of iteration t; queue form at the current x_t with the noise of the iteration
    // t + tau at which its message is due, so that both forms draw the same noise for the same
    // update under a constant tau.  A falling tau would name the same iteration twice, so the queue
    // form's keys are kept strictly increasing: q_key = max(t + tau, last key + 1), fixed by ddef_grad.
    uint64_t q_key = 0, q_key_floor = 0;
    uint64_t grad_key() const { return queue_form ? q_key : t; }
    const float* grad_snapshot() const { return queue_form ? ring : slot(t - tau); }
};

namespace {

int hip_fail(ddef_ctx* c, hipError_t err) {
    if (err == hipSuccess) return DDEF_OK;
    int code = (err == hipErrorOutOfMemory) ? DDEF_ENOMEM : DDEF_EHIP;
    if (c && code == DDEF_EHIP) c->sticky = DDEF_EHIP;
    (void)hipGetLastError();                 // reported here; not left for a later call to find
    return code;
}

#define HIP_TRY(ctx, expr)                         \
    do {                                           \
        hipError_t err__ = (expr);                 \
        if (err__ != hipSuccess) return hip_fail((ctx), err__); \
    } while (0)

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess && (prev == dev || hipSetDevice(dev) == hipSuccess)) ok = true;
        if (prev == dev) prev = -1;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

hipEvent_t take_event(ddef_ctx* c) {
    if (!c->free_events.empty()) { hipEvent_t e = c->free_events.back(); c->free_events.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct LaunchScope {
    ddef_ctx* c;
    hipStream_t stream;
    hipEvent_t stop = nullptr;
    int slot;
    LaunchScope(ddef_ctx* ctx, hipStream_t st, int s) : c(ctx), stream(st), slot(s) {
        if (!c->profiling) return;
        hipEvent_t start = take_event(c);
        stop = take_event(c);
        if (!start || !stop) { stop = nullptr; return; }
        (void)hipEventRecord(start, stream);
        c->pending.push_back(ProfRecord{slot, start, stop});
    }
    ~LaunchScope() { if (stop) (void)hipEventRecord(stop, stream); }
};

#define LAUNCH_ON(ctx, stream_, slot, kernel, grid, block, ...)                  \
    do {                                                                         \
        LaunchScope scope__((ctx), (stream_), (slot));                           \
        hipLaunchKernelGGL(kernel, (grid), (block), 0, (stream_), __VA_ARGS__);  \
    } while (0)
#define LAUNCH(ctx, slot, kernel, grid, block, ...) \
    LAUNCH_ON(ctx, (ctx)->stream, slot, kernel, grid, block, __VA_ARGS__)

int resolve_profile(ddef_ctx* c) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->side) HIP_TRY(c, hipStreamSynchronize(c->side));
    for (const ProfRecord& r : c->pending) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            c->prof_launches[r.slot] += 1;
            c->prof_ms[r.slot] += (double)ms;
        }
        c->free_events.push_back(r.start);
        c->free_events.push_back(r.stop);
    }
    c->pending.clear();
    return DDEF_OK;
}

uint32_t blocks_for(ddef_ctx* c, uint64_t items_per_row_blocks, uint32_t rows, uint32_t per_cu) {
    uint64_t budget = (uint64_t)c->cus * per_cu / (rows ? rows : 1u);
    if (budget < 1) budget = 1;
    uint64_t b = items_per_row_blocks < budget ? items_per_row_blocks : budget;
    return (uint32_t)(b < 1 ? 1 : b);
}

// The captured iteration is no longer valid (a pointer, an option or the problem changed).
void drop_graph(ddef_ctx* c) {
    if (c->graph_exec) { (void)hipGraphExecDestroy(c->graph_exec); c->graph_exec = nullptr; }
}

// Candidate slots per worker that a selection of k with candidate target kb wants:
// three times the target while messages are sparse, twice otherwise,
// at least 32 slots in each of the kSubs parts of the buffer, plus one whole 256-entry group
// per part (a part fills unevenly when d is small or the selection is dense); never more than
// every coordinate can need
uint64_t candidate_capacity(const ddef_ctx* c, uint64_t k, uint64_t kb) {
    const bool sparse = k * 32u <= c->d;
    uint64_t want = (sparse ? 3u : 2u) * kb;
    if (want < 32u * kSubs) want = 32u * kSubs;
    if (want > c->ld) want = c->ld;
    return ((want + 4095u) & ~(uint64_t)4095u) + 256u * kSubs;
}

// Whether the filter bound of a selection of k is placed from a fine sample of this very p in every
// iteration instead of following the trend of the last thresholds.  Sampling costs a fixed tenth
// of a millisecond or so; a tighter bound saves candidate work in proportion to n * k.  It pays for
// dense messages (k/d > 1/32) and wherever the workers' messages together hold 2^23 entries or more.
bool samples_every_iteration(const ddef_ctx* c, uint64_t k) {
    return k * 32u > c->d || k * (uint64_t)c->n >= ((uint64_t)1 << 23);
}

// candidate target: slack/16 times k where the bound follows the trend of the last thresholds;
// where it comes from a fine sample (up to 65 000 sample entries above it, the sample capped at 2^20
// entries per worker), k + k/24 for dense messages (the count caught misses the target by about
// 0.5 %) and k + k/16 for sparse ones (fewer sample entries above the bound: about 1 %)
uint64_t candidate_target(const ddef_ctx* c, uint64_t k) {
    uint64_t kb = k * (uint64_t)c->opt_slack_x16 / 16u;
    if (k * 32u > c->d) kb = k + k / 24u;
    else if (samples_every_iteration(c, k)) kb = k + k / 16u;
    if (kb < k) kb = k;
    if (kb > c->d) kb = c->d;
    return kb;
}

// Message rows for k entries per worker and `want` candidate slots per worker.
int ensure_capacity(ddef_ctx* c, uint64_t k, uint64_t want) {
    if (k > c->msg_ld) {
        drop_graph(c);
        // longer rows; the messages held so far (queued ones in queue form) move over
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        const uint64_t len = (k + 1023u) & ~(uint64_t)1023u;
        const size_t rows = (size_t)c->q_slots * c->n;
        uint32_t* idx = nullptr;
        float* val = nullptr;
        HIP_TRY(c, hipMalloc((void**)&idx, rows * len * 4u));
        hipError_t err = hipMalloc((void**)&val, rows * len * 4u);
        if (err != hipSuccess) {
            (void)hipFree(idx);
            return hip_fail(c, err);
        }
        err = hipMemset(idx, 0, rows * len * 4u);
        if (err == hipSuccess) err = hipMemset(val, 0, rows * len * 4u);
        if (err == hipSuccess && c->msg_ld)
            err = hipMemcpy2D(idx, len * 4u, c->msg_idx, c->msg_ld * 4u, c->msg_ld * 4u, rows, hipMemcpyDeviceToDevice);
        if (err == hipSuccess && c->msg_ld)
            err = hipMemcpy2D(val, len * 4u, c->msg_val, c->msg_ld * 4u, c->msg_ld * 4u, rows, hipMemcpyDeviceToDevice);
        if (err == hipSuccess) err = hipDeviceSynchronize();
        if (err != hipSuccess) { (void)hipFree(idx); (void)hipFree(val); return hip_fail(c, err); }
        if (c->msg_idx) (void)hipFree(c->msg_idx);
        if (c->msg_val) (void)hipFree(c->msg_val);
        c->msg_idx = idx; c->msg_val = val; c->msg_ld = len;
    }
    if (want > c->cap) {
        drop_graph(c);
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        if (c->cand) (void)hipFree(c->cand);
        if (c->sorted_idx) (void)hipFree(c->sorted_idx);
        if (c->sorted_val) (void)hipFree(c->sorted_val);
        c->cand = nullptr; c->sorted_idx = nullptr; c->sorted_val = nullptr; c->cap = 0;
        HIP_TRY(c, hipMalloc((void**)&c->cand, (size_t)c->n * want * 8u));
        HIP_TRY(c, hipMalloc((void**)&c->sorted_idx, (size_t)c->n * want * 4u));
        HIP_TRY(c, hipMalloc((void**)&c->sorted_val, (size_t)c->n * want * 4u));
        HIP_TRY(c, hipMemsetAsync(c->sorted_idx, 0, (size_t)c->n * want * 4u, c->stream));
        HIP_TRY(c, hipMemsetAsync(c->sorted_val, 0, (size_t)c->n * want * 4u, c->stream));
        c->cap = want;
    }
    return DDEF_OK;
}

SureView sure_view(const ddef_ctx* c, bool split) {
    if (!split) return SureView{nullptr, 0u, nullptr, 0u, nullptr};
    return SureView{c->sure, c->sure_cap, c->stab, c->nwc, c->filt + 7 * c->n};
}

// Buffers of the sure / band split for a selection of k: records for k entries per worker plus a
// quarter (the slots are handed out in kSubs parts that fill unevenly), the run table and the slot
// counters.  All of them or none.
int ensure_split_buffers(ddef_ctx* c, uint64_t k) {
    uint64_t want = k + k / 4u + 256u * kSubs;
    if (want > c->ld + 256u * kSubs) want = c->ld + 256u * kSubs;
    want = (want + 4095u) & ~(uint64_t)4095u;
    if (c->stab && want <= c->sure_cap) return DDEF_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    uint2 *sure = nullptr, *stab = c->stab;
    uint32_t* counters = c->sure_count;
    hipError_t err = hipMalloc((void**)&sure, (size_t)c->n * want * 8u);
    if (err == hipSuccess && !stab) err = hipMalloc((void**)&stab, (size_t)c->n * c->nwc * 8u);
    if (err == hipSuccess && !counters) {
        err = hipMalloc((void**)&counters, (size_t)c->n * kSubs * kSubStride * 4u);
        // on the context's stream: a fill on the null stream is not ordered against this stream's kernels
        if (err == hipSuccess) err = hipMemsetAsync(counters, 0, (size_t)c->n * kSubs * kSubStride * 4u, c->stream);
    }
    if (err != hipSuccess) {
        if (sure) (void)hipFree(sure);
        if (stab && stab != c->stab) (void)hipFree(stab);
        if (counters && counters != c->sure_count) (void)hipFree(counters);
        return hip_fail(c, err);
    }
    if (c->sure) (void)hipFree(c->sure);
    c->sure = sure; c->stab = stab; c->sure_count = counters; c->sure_cap = want;
    return DDEF_OK;
}

// Radix select and ordered compaction of every worker through its view (candidates or row).
void enqueue_select(ddef_ctx* c, uint32_t k, uint32_t kb, int fix_e = 1) {
    const uint32_t n = c->n;
    uint32_t *bound = c->filt, *cand_count = c->cand_count, *overflow = c->filt + n, *cand_total = c->filt + 3 * n;
    const SelViews vs{c->e, c->ld, (uint32_t)c->d, c->sorted_val, c->sorted_idx, c->cap, cand_total};
    // grids sized for the longest view that can occur (any worker may have to search its row)
    const uint64_t span = c->ld;
    const uint32_t gx = blocks_for(c, (span + 1023) / 1024, n, 8);
    for (int level = 0; level < 3; ++level) {
        uint32_t* h = c->hist + (uint64_t)level * n * 2 * 2048;
        LAUNCH(c, SL_DIGIT_HIST, k_digit_hist, dim3(gx, n), dim3(256), vs, (const SelState*)c->sel, h, level);
        LAUNCH(c, SL_DIGIT_PICK, k_digit_pick, dim3(n, 2), dim3(256), c->sel, (const uint32_t*)h, level);
    }
    const uint32_t gc = blocks_for(c, (span + 4095) / 4096, n, 8);
    LAUNCH(c, SL_CHUNK_COUNT, k_chunk_count, dim3(gc, n), dim3(256), vs, (const SelState*)c->sel, c->cnt_gt,
           c->cnt_eq, c->nchunks);
    LAUNCH(c, SL_CHUNK_SCAN, k_chunk_scan, dim3(n), dim3(1024), vs, c->sel, c->cnt_gt, c->cnt_eq, c->nchunks,
           k, kb, bound, c->filt + 5 * n, cand_count, overflow);
    LAUNCH(c, SL_CHUNK_EMIT, k_chunk_emit, dim3(gc, n), dim3(256), vs, (const SelState*)c->sel,
           (const uint32_t*)c->cnt_gt, (const uint32_t*)c->cnt_eq, c->nchunks, c->e, c->slot_idx(c->msg_slot),
           c->slot_val(c->msg_slot), c->msg_ld, k, fix_e);
}

// Sets the bits of the k coordinates Random-k keeps for this (iteration, worker) in the bitmap.
// A few coordinates are set one atomic each; many are first sorted into buckets by coordinate
// region (the candidate buffer, idle at this point, holds the buckets) and set region by region.
int enqueue_randk_mark(ddef_ctx* c, uint64_t k, const SelState* gate = nullptr) {
    const uint32_t n = c->n;
    const uint64_t bitmap_ld = c->ld / 32u;
    if (!c->bitmap) {
        uint32_t* bitmap = nullptr;
        hipError_t err = hipMalloc((void**)&bitmap, (size_t)n * bitmap_ld * 4u);
        if (err == hipSuccess) err = hipMemsetAsync(bitmap, 0, (size_t)n * bitmap_ld * 4u, c->stream);
        if (err != hipSuccess) { if (bitmap) (void)hipFree(bitmap); (void)hipGetLastError(); return hip_fail(c, err); }
        c->bitmap = bitmap;
    }
    uint32_t bits_d = 1;
    while (((uint64_t)1 << bits_d) < c->d) ++bits_d;
    const uint32_t region_bits = bits_d > 29u ? bits_d - 11u : 18u;
    const uint64_t regions = (c->d + (((uint64_t)1 << region_bits) - 1u)) >> region_bits;     // <= 2048
    const double expected = (double)k * (double)((uint64_t)1 << region_bits) / (double)c->d;
    uint64_t bucket_cap = (((uint64_t)(expected + 8.0 * std::sqrt(expected)) + 64u) + 63u) & ~(uint64_t)63u;
    if (c->opt_bucket_percent) bucket_cap = (uint64_t)(expected * (double)c->opt_bucket_percent / 100.0) + 1u;
    const bool binned = k >= ((uint64_t)1 << 20) && regions <= 2048u && regions * bucket_cap <= 2u * c->cap &&
                        bucket_cap < 0xffffffffull;
    if (!binned) {
        LAUNCH(c, gate ? SL_COMPOSED_REPEAT : SL_RANDK_MARK, k_randk_mark, dim3(blocks_for(c, (k + 255u) / 256u, n, 8), n), dim3(256),
               c->bitmap, bitmap_ld, (uint32_t)c->d, (uint32_t)k, (uint32_t)c->seed, (uint32_t)(c->seed >> 32),
               (uint32_t)c->t, (uint32_t)(c->t >> 32), gate);
        return DDEF_OK;
    }
    if (!c->region_count) {
        uint32_t* counts = nullptr;
        hipError_t err = hipMalloc((void**)&counts, (size_t)n * 2048u * 4u);
        if (err == hipSuccess) err = hipMemsetAsync(counts, 0, (size_t)n * 2048u * 4u, c->stream);
        if (err != hipSuccess) { if (counts) (void)hipFree(counts); (void)hipGetLastError(); return hip_fail(c, err); }
        c->region_count = counts;
    }
    uint32_t* bucket = reinterpret_cast<uint32_t*>(c->cand);
    LAUNCH(c, gate ? SL_COMPOSED_REPEAT : SL_RANDK_BIN, k_randk_bin, dim3(blocks_for(c, (k + 8191u) / 8192u, n, 2), n), dim3(1024), bucket,
           2u * c->cap, (uint32_t)bucket_cap, c->region_count, region_bits, (uint32_t)regions, c->bitmap, bitmap_ld,
           (uint32_t)c->d, (uint32_t)k, (uint32_t)c->seed, (uint32_t)(c->seed >> 32), (uint32_t)c->t,
           (uint32_t)(c->t >> 32), gate);
    LAUNCH(c, gate ? SL_COMPOSED_REPEAT : SL_RANDK_FILL, k_randk_fill, dim3((uint32_t)regions, n), dim3(1024), (const uint32_t*)bucket,
           2u * c->cap, (uint32_t)bucket_cap, c->region_count, region_bits, (uint32_t)regions, c->bitmap, bitmap_ld,
           (uint32_t)c->d, gate);
    return DDEF_OK;
}

// The sum of the messages named by the last ddef_aggregate, written to U (a getter wants it;
// the iteration itself never needs U in memory).
void materialize_update(ddef_ctx* c) {
    if (!c->agg_deferred || c->agg_in_U) return;
    LAUNCH(c, SL_AGGREGATE_TILES, k_aggregate_tiles<false>, dim3(c->ntiles), dim3(256), c->U,
           (const uint32_t*)c->slot_idx(c->agg_slot), (const float*)c->slot_val(c->agg_slot), c->msg_ld,
           (const uint32_t*)c->agg_off, c->ntiles, c->n, ModelRows{nullptr, nullptr, nullptr, nullptr, 1u, 0u}, 1.0f,
           sure_view(c, c->agg_split));
    c->u_zero = false;
    c->agg_in_U = true;
}

// U = 0, for an aggregation without messages.
void zero_update(ddef_ctx* c) {
    if (c->u_zero) return;
    const uint64_t quads = c->ld / 4u;
    LAUNCH(c, SL_FILL, k_fill_f4, dim3((uint32_t)((quads + 63) / 64)), dim3(64), c->U, quads);
    c->u_zero = true;
}

// Gradient generator inputs: snapshot xs and the iteration number `key` the noise is drawn for.
GradSource grad_source(const ddef_ctx* c, uint64_t key, const float* xs) {
    GradSource s{c->lambda, c->xstar, xs, (uint32_t)c->seed, (uint32_t)(c->seed >> 32),
                 (uint32_t)key, (uint32_t)(key >> 32), c->noise_kind, c->noise_scale, c->zeta,
                 nullptr, c->ring, c->ring_slots, c->tau, c->ld};
    if (c->capturing) s.t_dev = c->t_dev;          // ring form only: key = t, snapshot = slot(t - tau)
    return s;
}

void enqueue_grad(ddef_ctx* c, hipStream_t stream, float* dest, uint64_t key, const float* xs,
                  uint32_t blocks_per_cu) {
    const uint64_t quads = (c->d + 3) / 4;
    const uint32_t gx = blocks_for(c, (quads + 255) / 256, 1, blocks_per_cu);
    LAUNCH_ON(c, stream, SL_GRAD, k_grad, dim3(gx), dim3(256), grad_source(c, key, xs), dest, c->ld,
              (uint32_t)c->d, c->n);
}

// Fused mode: write this iteration's gradient to memory after all (a getter, the test hook or a
// kernel that reads g needs it).  Valid until the iteration is applied.
void materialize_grad(ddef_ctx* c) {
    if (!c->grad_pending) return;
    if (!c->grad_stored) enqueue_grad(c, c->stream, c->g, c->grad_key(), c->grad_snapshot(), 64u);
    c->grad_stored = true;
    c->grad_pending = false;
}

// Forget a prefetched gradient (its inputs are about to change); waits for the second stream so
// that nothing of it is still reading them.
int drop_prefetch(ddef_ctx* c) {
    c->pf_valid = false;
    if (c->side) HIP_TRY(c, hipStreamSynchronize(c->side));
    return DDEF_OK;
}

// After the gradient of iteration t is in place: start the one of iteration t+1 on the second
// stream.  It reads snapshot x_{t+1-tau} (complete once iteration t-1 was applied, and a
// different ring slot from the one iteration t writes, as 1 <= tau <= tau_max) and writes the
// buffer the accumulate pass of iteration t-1 has finished reading.
int start_prefetch(ddef_ctx* c) {
    // (queue form takes the next gradient at x_{t+1}, which does not exist yet)
    if (!c->opt_prefetch || c->opt_fuse || c->queue_form || c->tau == 0 || c->t + 1 < c->tau) return DDEF_OK;
    if (!c->side) {
        // second stream, its two events and the second gradient buffer: all of them or none, so
        // that a failed set-up can simply be tried again
        const size_t bytes = (size_t)c->ld * 4u * c->n;
        hipStream_t side = nullptr;
        hipEvent_t applied = nullptr, prefetched = nullptr;
        float* next = nullptr;
        hipError_t err = hipStreamCreateWithFlags(&side, hipStreamNonBlocking);
        if (err == hipSuccess) err = hipEventCreateWithFlags(&applied, hipEventDisableTiming);
        if (err == hipSuccess) err = hipEventCreateWithFlags(&prefetched, hipEventDisableTiming);
        if (err == hipSuccess) err = hipMalloc((void**)&next, bytes);
        if (err == hipSuccess) err = hipMemsetAsync(next, 0, bytes, side);
        if (err != hipSuccess) {
            if (side) (void)hipStreamSynchronize(side);
            if (next) (void)hipFree(next);
            if (prefetched) (void)hipEventDestroy(prefetched);
            if (applied) (void)hipEventDestroy(applied);
            if (side) (void)hipStreamDestroy(side);
            (void)hipGetLastError();
            return hip_fail(c, err);
        }
        c->side = side; c->ev_applied = applied; c->ev_prefetched = prefetched; c->g_next = next;
    }
    if (!c->g_next || !c->ev_applied || !c->ev_prefetched) return DDEF_EINTERNAL;
    HIP_TRY(c, hipEventRecord(c->ev_applied, c->stream));        // everything up to here on the main stream
    HIP_TRY(c, hipStreamWaitEvent(c->side, c->ev_applied, 0));
    // fewer resident blocks than the stand-alone launch: the two kernels share the CUs' wave slots
    enqueue_grad(c, c->side, c->g_next, c->t + 1, c->slot(c->t + 1 - c->tau), 16u);
    HIP_TRY(c, hipEventRecord(c->ev_prefetched, c->side));
    c->pf_valid = true; c->pf_t = c->t + 1; c->pf_tau = c->tau;
    return DDEF_OK;
}

// Places bound[] and zero_at[] for a selection of k (candidate target kb) from one entry in `stride`
// of p = e + lr*g (taken eight consecutive coordinates at a time): the radix select of the path, run on the sample for the ranks k/stride and
// kb/stride.  The stride keeps about `above` sample entries above the bound (count error about
// 1/sqrt(above)) within a sample of at most kSampleMax entries per worker; with fewer than 8 above
// the bound sampling says too little, and the iteration goes on with what it had (a whole-row
// search when there is no bound at all).
int bound_from_sample(ddef_ctx* c, uint64_t k, uint64_t kb, float lr, uint64_t above, bool* placed = nullptr) {
    constexpr uint64_t kSampleMax = 1u << 20;
    if (placed) *placed = false;
    uint64_t stride = kb / above;
    const uint64_t least = (c->d + kSampleMax - 1u) / kSampleMax;
    if (stride < least) stride = least;
    if (stride < 1u) stride = 1u;
    const uint64_t count = 8u * ((c->d + 8u * stride - 1u) / (8u * stride));   // whole octets
    const uint64_t kb_s = kb / stride, k_s = k / stride > 0u ? k / stride : 1u;
    if (kb_s < 8u || kb_s > count) return DDEF_OK;
    const uint32_t n = c->n;
    if (!c->sample) {
        // the sample rows and their length words: both or neither
        const uint64_t sample_ld = ((c->d < kSampleMax ? c->d : kSampleMax) + 15u) & ~(uint64_t)3u;
        float* sample = nullptr;
        uint32_t* total = nullptr;
        hipError_t err = hipMalloc((void**)&sample, (size_t)n * sample_ld * 4u);
        if (err == hipSuccess) err = hipMalloc((void**)&total, (size_t)n * 4u);
        if (err == hipSuccess) err = hipMemsetAsync(sample, 0, (size_t)n * sample_ld * 4u, c->stream);
        if (err != hipSuccess) {
            if (total) (void)hipFree(total);
            if (sample) (void)hipFree(sample);
            (void)hipGetLastError();
            return hip_fail(c, err);
        }
        c->sample = sample; c->sample_total = total; c->sample_ld = sample_ld;
        drop_graph(c);
    }
    // a gradient that lives only in the fused accumulate pass is generated for the sampled coordinates
    const GradSource src = grad_source(c, c->grad_key(), c->grad_snapshot());
    if (c->grad_pending) {
        LAUNCH(c, SL_SAMPLE, k_sample_p<true>, dim3((uint32_t)((count + 255u) / 256u), n), dim3(256),
               (const float*)c->e, (const float*)c->g, src, c->ld, (uint32_t)c->d, lr, (uint32_t)stride,
               (uint32_t)count, c->sample, c->sample_ld);
    } else {
        LAUNCH(c, SL_SAMPLE, k_sample_p<false>, dim3((uint32_t)((count + 255u) / 256u), n), dim3(256),
               (const float*)c->e, (const float*)c->g, src, c->ld, (uint32_t)c->d, lr, (uint32_t)stride,
               (uint32_t)count, c->sample, c->sample_ld);
    }
    LAUNCH(c, SL_SAMPLE, k_sample_begin, dim3(n), dim3(256), c->sel, n, (uint32_t)k_s, (uint32_t)kb_s,
           (uint32_t)count, c->sample_total, c->hist);
    const SelViews vs{c->e, c->ld, (uint32_t)c->d, c->sample, (const uint32_t*)nullptr, c->sample_ld,
                      (const uint32_t*)c->sample_total};
    const uint32_t gx = blocks_for(c, (count + 1023u) / 1024u, n, 8);
    for (int level = 0; level < 3; ++level) {
        uint32_t* h = c->hist + (uint64_t)level * n * 2 * 2048;
        LAUNCH(c, SL_DIGIT_HIST, k_digit_hist, dim3(gx, n), dim3(256), vs, (const SelState*)c->sel, h, level);
        LAUNCH(c, SL_DIGIT_PICK, k_digit_pick, dim3(n, 2), dim3(256), c->sel, (const uint32_t*)h, level);
    }
    LAUNCH(c, SL_SAMPLE, k_sample_finish, dim3((n + 255u) / 256u), dim3(256), (const SelState*)c->sel, n, c->filt,
           c->filt + 5 * n, c->filt + 6 * n, (int)c->opt_split - 1);
    HIP_TRY(c, hipGetLastError());
    c->have_bound = true;
    c->bound_k = k;
    if (placed) *placed = true;
    return DDEF_OK;
}

int check_ctx(ddef_ctx* c) {
    if (!c) return DDEF_EINVAL;
    if (c->sticky != DDEF_OK) return c->sticky;
    return DDEF_OK;
}

// Flags the kernels raise on the device, read with the stream idle: a non-finite entry of
// e + lr*g (finite input is required; the selection order is undefined for NaN), and, after a
// Random-k selection, a worker whose runs did not hold exactly k entries (slot overflow).
int check_device_flags(ddef_ctx* c) {
    std::vector<uint32_t> bad(c->n, 0u);
    HIP_TRY(c, hipMemcpy(bad.data(), c->filt + 4 * c->n, (size_t)c->n * 4u, hipMemcpyDeviceToHost));
    for (uint32_t v : bad)
        if (v) { c->sticky = DDEF_ENONFINITE; return DDEF_ENONFINITE; }
    if (c->compressor == DDEF_COMPRESSOR_TOPK || c->k_step == 0) return DDEF_OK;
    std::vector<SelState> st(c->n);
    HIP_TRY(c, hipMemcpy(st.data(), c->sel, sizeof(SelState) * c->n, hipMemcpyDeviceToHost));
    for (const SelState& s : st)
        if (s.active == 2u) { c->sticky = DDEF_EINTERNAL; return DDEF_EINTERNAL; }
    return DDEF_OK;
}

int copy_row_out(ddef_ctx* c, const float* dev_row, float* host) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(host, dev_row, (size_t)c->d * 4u, hipMemcpyDeviceToHost));
    return DDEF_OK;
}

int copy_row_in(ddef_ctx* c, float* dev_row, const float* host) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(dev_row, host, (size_t)c->d * 4u, hipMemcpyHostToDevice));
    return DDEF_OK;
}

}  // namespace

extern "C" {

uint64_t ddef_k_from_delta(double delta, uint64_t d) {
    if (!(delta > 0.0) || !(delta <= 1.0) || d == 0) return 0;
    double want = std::ceil(delta * (double)d);
    if (want < 1.0) return 1;
    if (want >= (double)d) return d;
    return (uint64_t)want;
}

const char* ddef_strerror(int code) {
    switch (code) {
        case DDEF_OK: return "ok";
        case DDEF_EINVAL: return "invalid argument";
        case DDEF_ESTATE: return "call order violated";
        case DDEF_ENOMEM: return "out of memory";
        case DDEF_EHIP: return "HIP runtime error";
        case DDEF_ENONFINITE: return "non-finite value";
        case DDEF_EINTERNAL: return "internal invariant violated";
        default: return "unknown error";
    }
}

static int init_ctx(uint64_t d, uint32_t n, uint32_t tau_max, bool queue_form, ddef_ctx** out) {
    if (!out) return DDEF_EINVAL;
    *out = nullptr;
    if (d == 0 || d >= 0xFFFFE000ull || n == 0 || n > 65535u || tau_max > 4096u) return DDEF_EINVAL;
    ddef_ctx* c = new (std::nothrow) ddef_ctx;
    if (!c) return DDEF_ENOMEM;
    auto fail = [&](int code) { ddef_destroy(c); (void)hipGetLastError(); return code; };
    hipError_t err = hipGetDevice(&c->device);
    if (err != hipSuccess) return fail(DDEF_EHIP);
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, c->device) == hipSuccess && prop.multiProcessorCount > 0)
        c->cus = prop.multiProcessorCount;
    c->d = d; c->n = n; c->tau_max = tau_max; c->tau = tau_max;
    c->queue_form = queue_form;
    c->ring_slots = queue_form ? 1u : tau_max + 1u;
    c->q_slots = queue_form ? tau_max + 1u : 1u;
    c->q_k.assign(c->q_slots, 0);
    c->ld = (d + 4095u) & ~(uint64_t)4095u;
    c->nchunks = (uint32_t)(c->ld / 4096u);
    c->nwc = (uint32_t)(c->ld / 256u);          // 256-entry groups of the filter kernel
    c->nspans = (c->nwc + kSpan - 1u) / kSpan;
    c->ntiles = (uint32_t)(c->ld / kTile);
    if (hipStreamCreateWithFlags(&c->own_stream, hipStreamNonBlocking) != hipSuccess) return fail(DDEF_EHIP);
    c->stream = c->own_stream;
    const size_t row = (size_t)c->ld * 4u;
    struct Want { void** p; size_t bytes; };
    Want wants[] = {
        {(void**)&c->lambda, row}, {(void**)&c->xstar, row}, {(void**)&c->U, row},
        {(void**)&c->ring, row * c->ring_slots}, {(void**)&c->e, row * n}, {(void**)&c->g, row * n},
        {(void**)&c->sel, sizeof(SelState) * n}, {(void**)&c->hist, (size_t)3 * n * 2 * 2048 * 4},
        {(void**)&c->cnt_gt, (size_t)n * c->nchunks * 4}, {(void**)&c->cnt_eq, (size_t)n * c->nchunks * 4},
        {(void**)&c->filt, (size_t)9 * n * 4}, {(void**)&c->cand_count, (size_t)n * kSubs * kSubStride * 4}, {(void**)&c->tab, (size_t)n * c->nwc * 8},
        {(void**)&c->span_sum, (size_t)n * c->nspans * 4},
        {(void**)&c->agg_off, (size_t)n * (c->ntiles + 1u) * 4},
        {(void**)&c->t_dev, 8},
    };
    for (const Want& w : wants) {
        err = hipMalloc(w.p, w.bytes);
        if (err != hipSuccess) { (void)hipGetLastError(); return fail(err == hipErrorOutOfMemory ? DDEF_ENOMEM : DDEF_EHIP); }
        err = hipMemsetAsync(*w.p, 0, w.bytes, c->stream);
        if (err != hipSuccess) return fail(DDEF_EHIP);
    }
    if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(DDEF_EHIP);
    *out = c;
    return DDEF_OK;
}

int ddef_init(uint64_t d, uint32_t n, uint32_t tau_max, ddef_ctx** out) {
    return init_ctx(d, n, tau_max, false, out);
}

int ddef_init_queue(uint64_t d, uint32_t n, uint32_t tau_max, ddef_ctx** out) {
    return init_ctx(d, n, tau_max, true, out);
}

int ddef_destroy(ddef_ctx* c) {
    if (!c) return DDEF_EINVAL;
    DeviceGuard guard(c->device);
    if (c->stream) (void)hipStreamSynchronize(c->stream);
    drop_graph(c);
    if (c->side) { (void)hipStreamSynchronize(c->side); (void)hipStreamDestroy(c->side); }
    if (c->ev_applied) (void)hipEventDestroy(c->ev_applied);
    if (c->ev_prefetched) (void)hipEventDestroy(c->ev_prefetched);
    for (const ProfRecord& r : c->pending) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    for (hipEvent_t e : c->free_events) (void)hipEventDestroy(e);
    void* bufs[] = {c->lambda, c->xstar, c->U, c->ring, c->e, c->g, c->sel, c->hist, c->cnt_gt,
                    c->cnt_eq, c->msg_idx, c->msg_val, c->filt, c->cand_count, c->tab, c->span_sum, c->agg_off, c->t_dev, c->sample, c->sample_total, c->bitmap, c->region_count, c->objective_partial, c->g_next, c->cand,
                    c->sorted_idx, c->sorted_val, c->codes, c->steps, c->sure, c->stab, c->sure_count, c->canon_idx,
                    c->canon_val};
    for (void* b : bufs) if (b) (void)hipFree(b);
    if (c->own_stream) (void)hipStreamDestroy(c->own_stream);
    delete c;
    return DDEF_OK;
}

int ddef_set_stream(ddef_ctx* c, void* hip_stream) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (c->phase != PH_IDLE) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    rc = drop_prefetch(c);
    if (rc) return rc;
    drop_graph(c);
    c->stream = hip_stream ? (hipStream_t)hip_stream : c->own_stream;
    return DDEF_OK;
}

int ddef_set_problem(ddef_ctx* c, const float* host_lambda, const float* host_xstar, const float* host_x0,
                     uint64_t seed, int noise_kind, float noise_scale) {
    if (c && c->sticky == DDEF_ENONFINITE) c->sticky = DDEF_OK;      // a fresh problem starts clean
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_lambda || !host_xstar || !host_x0) return DDEF_EINVAL;
    if (noise_kind < DDEF_NOISE_NONE || noise_kind > DDEF_NOISE_STUDENT_T3) return DDEF_EINVAL;
    if (!std::isfinite(noise_scale)) return DDEF_EINVAL;
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    rc = drop_prefetch(c);
    if (rc) return rc;
    const size_t bytes = (size_t)c->d * 4u;
    HIP_TRY(c, hipMemcpy(c->lambda, host_lambda, bytes, hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(c->xstar, host_xstar, bytes, hipMemcpyHostToDevice));
    for (uint32_t s = 0; s < c->ring_slots; ++s)
        HIP_TRY(c, hipMemcpy(c->ring + (uint64_t)s * c->ld, host_x0, bytes, hipMemcpyHostToDevice));
    std::fill(c->q_k.begin(), c->q_k.end(), (uint64_t)0);
    // fills go on the context's stream, where the kernels that read these buffers run (a fill on the
    // null stream is not ordered against a non-blocking stream)
    HIP_TRY(c, hipMemsetAsync(c->e, 0, (size_t)c->ld * 4u * c->n, c->stream));
    HIP_TRY(c, hipMemsetAsync(c->U, 0, (size_t)c->ld * 4u, c->stream));
    HIP_TRY(c, hipMemsetAsync(c->sel, 0, sizeof(SelState) * c->n, c->stream));
    HIP_TRY(c, hipMemsetAsync(c->filt, 0, (size_t)9 * c->n * 4, c->stream));
    c->msg_split = false; c->agg_split = false;
    HIP_TRY(c, hipMemsetAsync(c->cand_count, 0, (size_t)c->n * kSubs * kSubStride * 4, c->stream));
    if (c->sure_count) HIP_TRY(c, hipMemsetAsync(c->sure_count, 0, (size_t)c->n * kSubs * kSubStride * 4, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->have_bound = false;
    c->sel_k = 0; c->sel_run = 0;
    drop_graph(c);
    c->seed = seed; c->noise_kind = noise_kind; c->noise_scale = noise_scale;
    c->t = 0; c->phase = PH_IDLE; c->problem_set = true; c->step_empty = true; c->k_step = 0;
    c->q_key = 0; c->q_key_floor = 0;
    c->full_selects = 0;
    c->u_zero = true;
    c->agg_deferred = false;
    return DDEF_OK;
}

int ddef_set_compressor(ddef_ctx* c, int kind) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (kind != DDEF_COMPRESSOR_TOPK && kind != DDEF_COMPRESSOR_RANDK && kind != DDEF_COMPRESSOR_COMPOSED)
        return DDEF_EINVAL;
    if (c->queue_form && kind != DDEF_COMPRESSOR_TOPK) return DDEF_EINVAL;
    if (c->phase != PH_IDLE) return DDEF_ESTATE;
    drop_graph(c);
    c->compressor = kind;
    c->codes_valid = false;
    return DDEF_OK;
}

int ddef_set_composed(ddef_ctx* c, double rand_ratio) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!(rand_ratio > 0.0) || !(rand_ratio <= 1.0)) return DDEF_EINVAL;
    if (c->phase != PH_IDLE) return DDEF_ESTATE;
    c->rand_ratio = rand_ratio;
    return DDEF_OK;
}

int ddef_set_heterogeneity(ddef_ctx* c, float zeta) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!std::isfinite(zeta)) return DDEF_EINVAL;
    if (c->phase != PH_IDLE) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    rc = drop_prefetch(c);
    if (rc) return rc;
    drop_graph(c);
    c->zeta = zeta;
    return DDEF_OK;
}

int ddef_set_tau(ddef_ctx* c, uint32_t tau) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (tau > c->tau_max) return DDEF_EINVAL;
    if (c->phase != PH_IDLE) return DDEF_ESTATE;
    if (tau != c->tau) c->pf_valid = false;
    c->tau = tau;
    return DDEF_OK;
}

int ddef_grad(ddef_ctx* c) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!c->problem_set || c->phase != PH_IDLE) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    c->step_empty = !c->queue_form && c->t < c->tau;
    if (c->queue_form) {
        c->q_key = std::max(c->t + c->tau, c->q_key_floor);
        c->q_key_floor = c->q_key + 1u;
    }
    c->grad_pending = false;
    c->grad_stored = false;
    c->grad_live = !c->step_empty;
    if (!c->step_empty && c->opt_fuse) {
        c->grad_pending = true;            // generated inside the accumulate pass
    } else if (!c->step_empty) {
        if (c->pf_valid && c->pf_t == c->t && c->pf_tau == c->tau) {
            HIP_TRY(c, hipStreamWaitEvent(c->stream, c->ev_prefetched, 0));
            float* ready = c->g_next;
            c->g_next = c->g;
            c->g = ready;
            c->pf_valid = false;
        } else {
            enqueue_grad(c, c->stream, c->g, c->grad_key(), c->grad_snapshot(), 64u);
        }
        HIP_TRY(c, hipGetLastError());
        rc = start_prefetch(c);
        if (rc) return rc;
    }
    c->phase = PH_GRAD;
    return DDEF_OK;
}

int ddef_load_grad(ddef_ctx* c, uint32_t worker, const float* host_g) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_g || worker >= c->n) return DDEF_EINVAL;
    if (!c->problem_set || (c->phase != PH_IDLE && c->phase != PH_GRAD)) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    materialize_grad(c);
    rc = copy_row_in(c, c->g + (uint64_t)worker * c->ld, host_g);
    if (rc) return rc;
    c->step_empty = false;
    c->grad_live = true;
    c->phase = PH_GRAD;
    return DDEF_OK;
}

int ddef_ef_compress(ddef_ctx* c, double delta, float lr) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!(delta > 0.0) || !(delta <= 1.0) || !std::isfinite(lr)) return DDEF_EINVAL;
    if (c->phase != PH_GRAD) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    c->lr_step = lr;
    if (c->step_empty) {
        c->k_step = 0;
        c->phase = PH_COMPRESSED;
        return DDEF_OK;
    }
    // composed: Random-k keeps k1 coordinates, Top-k the k = ceil(delta * k1) largest of them
    const bool composed = c->compressor == DDEF_COMPRESSOR_COMPOSED;
    const uint64_t k1 = composed ? ddef_k_from_delta(c->rand_ratio, c->d) : 0u;
    const uint64_t k = composed ? ddef_k_from_delta(delta, k1) : ddef_k_from_delta(delta, c->d);
    c->agg_deferred = false;               // the messages it would read are about to be replaced
    c->msg_split = false;
    const uint64_t kb = candidate_target(c, k);
    rc = composed ? ensure_capacity(c, k, candidate_capacity(c, k1, candidate_target(c, k1)))
                  : ensure_capacity(c, k, candidate_capacity(c, k, kb));
    if (rc) return rc;
    c->msg_slot = (uint32_t)(c->t % c->q_slots);
    c->q_k[c->msg_slot] = 0;               // set again once the launches are enqueued
    const uint32_t n = c->n;
    uint32_t *bound = c->filt, *cand_count = c->cand_count, *overflow = c->filt + n, *stat_full = c->filt + 2 * n;
    uint32_t* cand_total = c->filt + 3 * n;
    uint32_t* zero_at = c->filt + 5 * n;
    if (c->compressor != DDEF_COMPRESSOR_TOPK) materialize_grad(c);
    if (composed) {
        if (c->codes_ld != c->msg_ld / 2u) {       // follows the message rows (msg_ld is a multiple of 1024)
            HIP_TRY(c, hipStreamSynchronize(c->stream));
            if (c->codes) (void)hipFree(c->codes);
            if (c->steps) (void)hipFree(c->steps);
            c->codes = nullptr; c->steps = nullptr; c->codes_ld = 0;
            HIP_TRY(c, hipMalloc((void**)&c->codes, (size_t)n * (c->msg_ld / 2u)));
            HIP_TRY(c, hipMalloc((void**)&c->steps, (size_t)n * (c->msg_ld / 256u) * 4u));
            c->codes_ld = c->msg_ld / 2u;
        }
        const uint64_t bitmap_ld = c->ld / 32u;
        // The k largest of the kept entries lie above the magnitude that about k of the kept ones
        // exceed, and a random subset has the quantiles of the whole row: a sample of p places a
        // bound that a few more than k kept entries are expected to pass (margin: a 24th of k, at
        // least six standard deviations of the count), and only those are recorded.  Should fewer
        // than k pass after all, the pass runs again over the stored p without a bound.
        bool bounded = false;
        const uint64_t margin = std::max<uint64_t>(k / 24u, (uint64_t)(6.0 * std::sqrt((double)k)) + 1u) + 16u;
        uint64_t kb2 = k + margin;
        if (c->opt_composed_bound == 2) kb2 = k / 2u;       // test knob: a bound that is too high
        if (c->opt_composed_bound && !c->opt_force_full && kb2 >= 8u && 2u * kb2 <= k1) {
            const double scale = (double)c->d / (double)k1;
            const uint64_t k_row = std::min<uint64_t>(c->d, (uint64_t)std::ceil((double)k * scale));
            const uint64_t kb_row = std::min<uint64_t>(c->d, (uint64_t)std::ceil((double)kb2 * scale));
            c->have_bound = false;
            rc = bound_from_sample(c, k_row, kb_row, lr, 65536u);
            if (rc) return rc;
            bounded = c->have_bound;
        }
        // gate: a repeat pass, whose kernels run only for the workers the first pass flagged (active == 3)
        auto record = [&](bool with_bound, int accumulate, const SelState* gate) -> int {
            int rcm = enqueue_randk_mark(c, k1, gate);
            if (rcm) return rcm;
            const uint32_t gx = gate ? std::min<uint32_t>(c->nwc, (uint32_t)c->cus * 32u) : c->nwc;
            // (the repeat pass's launches are timed under a slot of their own: they return at once as a rule)
            LAUNCH(c, gate ? SL_COMPOSED_REPEAT : SL_EF_RANDK, k_ef_randk, dim3(gx, n), dim3(64), c->e, c->g, c->ld, (uint32_t)c->d, lr, 0,
                   accumulate, with_bound ? (const uint32_t*)bound : (const uint32_t*)nullptr, c->bitmap, bitmap_ld,
                   c->cand, c->cap, cand_count, overflow, c->tab, c->nwc, c->filt + 4 * n, gate);
            LAUNCH(c, gate ? SL_COMPOSED_REPEAT : SL_TAB_SUM, k_tab_sum, dim3(c->nspans, n), dim3(1024), (const uint2*)c->tab, c->nwc,
                   c->span_sum, c->nspans, gate);
            LAUNCH(c, gate ? SL_COMPOSED_REPEAT : SL_TAB_DECIDE, k_tab_decide_composed, dim3(n), dim3(256), c->span_sum, c->nspans, overflow,
                   (uint32_t)k1, (uint32_t)k, n, with_bound ? 0 : 1, c->sel, cand_total, cand_count, c->hist,
                   stat_full, gate ? 1 : 0);
            return DDEF_OK;
        };
        rc = record(bounded, 1, nullptr);
        if (rc) return rc;
        if (bounded) {
            // Whether every worker caught enough is known on the device only.  The repeat of the pass
            // (over the stored p, without the bound) is therefore enqueued every time, and its
            // kernels return at once for the workers that need none: no wait for the stream here.
            rc = record(false, 0, c->sel);
            if (rc) return rc;
        }
        LAUNCH(c, SL_TAB_ORDER, k_tab_order, dim3(c->nspans, n), dim3(1024), (const uint2*)c->tab, c->nwc,
               (const uint32_t*)c->span_sum, c->nspans, (const SelState*)c->sel, (const uint2*)c->cand, c->cap,
               c->sorted_idx, c->sorted_val, c->cap, (float*)nullptr, (uint64_t)0);
        enqueue_select(c, (uint32_t)k, (uint32_t)k, 0);      // e is completed by the 4-bit stage
        LAUNCH(c, SL_QUANTIZE4, k_quantize4, dim3((uint32_t)((k + 255u) / 256u), n), dim3(256),
               (const uint32_t*)c->slot_idx(c->msg_slot), c->slot_val(c->msg_slot), c->msg_ld, (uint32_t)k,
               (const SelState*)c->sel, c->e, c->ld, c->codes, c->codes_ld, c->steps, c->codes_ld / 128u);
        HIP_TRY(c, hipGetLastError());
        c->have_bound = false;          // the filter words now describe this selection, not a Top-k of e
        c->sel_k = 0; c->sel_run = 0;
        c->codes_valid = true;
        c->k_step = k;
        c->q_k[c->msg_slot] = k;
        c->phase = PH_COMPRESSED;
        return DDEF_OK;
    }
    if (c->compressor == DDEF_COMPRESSOR_RANDK) {
        const uint64_t bitmap_ld = c->ld / 32u;
        rc = enqueue_randk_mark(c, k);
        if (rc) return rc;
        LAUNCH(c, SL_EF_RANDK, k_ef_randk, dim3(c->nwc, n), dim3(64), c->e, c->g, c->ld, (uint32_t)c->d, lr, 1,
               1, (const uint32_t*)nullptr, c->bitmap, bitmap_ld, c->cand, c->cap, cand_count, overflow, c->tab, c->nwc, c->filt + 4 * n,
               (const SelState*)nullptr);
        LAUNCH(c, SL_TAB_SUM, k_tab_sum, dim3(c->nspans, n), dim3(1024), (const uint2*)c->tab, c->nwc,
               c->span_sum, c->nspans, (const SelState*)nullptr);
        LAUNCH(c, SL_TAB_DECIDE, k_tab_decide_randk, dim3(n), dim3(256), c->span_sum, c->nspans, overflow,
               (uint32_t)k, c->sel, cand_total, cand_count);
        LAUNCH(c, SL_TAB_ORDER, k_tab_order, dim3(c->nspans, n), dim3(1024), (const uint2*)c->tab, c->nwc,
               (const uint32_t*)c->span_sum, c->nspans, (const SelState*)c->sel, (const uint2*)c->cand, c->cap,
               c->slot_idx(c->msg_slot), c->slot_val(c->msg_slot), c->msg_ld, (float*)nullptr, (uint64_t)0);
        HIP_TRY(c, hipGetLastError());
        c->have_bound = false;          // a Top-k bound from before no longer describes e
        c->sel_k = 0; c->sel_run = 0;
        c->k_step = k;
        c->q_k[c->msg_slot] = k;
        c->phase = PH_COMPRESSED;
        return DDEF_OK;
    }
    // the filter pays off only for sparse messages and needs a bound: the last selection's, or,
    // where that was placed for another k or there was none, one from a sample of this p
    // (or the last selections' bound has no trend behind it yet: the first two iterations with a k).
    // Dense messages (k/d > 1/32) sample every time, and more finely: there the entries between the
    // expected and the true threshold each cost a scattered store in the compaction, many enough
    // to outweigh the sampling by far, and the trend of noisy thresholds misses by more.
    const bool can_filter = !c->opt_force_full && 2 * kb <= c->d;
    const bool dense = samples_every_iteration(c, k);
    bool sampled = false;
    if (can_filter && (dense || !c->have_bound || c->bound_k != k || c->sel_k != k || c->sel_run < 2u)) {
        rc = bound_from_sample(c, k, kb, lr, dense ? 65536u : 256u, &sampled);
        if (rc) return rc;
    }
    const bool use_filter = can_filter && c->have_bound;
    // dense messages (k/d > 1/32) with a bound and an expected threshold fresh from this p: sure / band
    // split.  (Measured on d = 1.3e9, n = 4: 20.6 -> 15.5 ms per iteration at delta = 0.1; at
    // delta = 0.01 the runs are two or three entries long and reading them costs the aggregation more
    // than the selection saves, 12.4 -> 12.9 ms, so sparser messages keep the one-part form.)  The
    // queue form keeps whole messages in its slots and stays with the one-part form, too.
    const bool split = use_filter && sampled && k * 32u > c->d && !c->queue_form && c->opt_split;
    if (split) {
        rc = ensure_split_buffers(c, k);
        if (rc) return rc;
    }
    const SureRuns sp{c->filt + 6 * n, c->sure, c->sure_cap, c->sure_count, c->stab};
    const GradSource src = grad_source(c, c->grad_key(), c->grad_snapshot());
    if (c->grad_pending && split) {
        LAUNCH(c, SL_EF_FILTER_FUSED, (k_ef_filter<true, true>), dim3(c->nwc * n), dim3(64), c->e, (const float*)c->g, src,
               n, c->ld, (uint32_t)c->d, lr, (const uint32_t*)bound, (const uint32_t*)zero_at, 1,
               c->cand, c->cap, cand_count, overflow, c->tab, c->nwc, c->filt + 4 * n, sp);
    } else if (c->grad_pending) {
        LAUNCH(c, SL_EF_FILTER_FUSED, (k_ef_filter<true, false>), dim3(c->nwc * n), dim3(64), c->e, (const float*)c->g, src,
               n, c->ld, (uint32_t)c->d, lr, (const uint32_t*)bound, (const uint32_t*)zero_at, use_filter ? 1 : 0,
               c->cand, c->cap, cand_count, overflow, c->tab, c->nwc, c->filt + 4 * n, sp);
    } else if (split) {
        LAUNCH(c, SL_EF_FILTER_SPLIT, (k_ef_filter<false, true>), dim3(c->nwc, n), dim3(64), c->e, (const float*)c->g, src, n,
               c->ld, (uint32_t)c->d, lr, (const uint32_t*)bound, (const uint32_t*)zero_at, 1,
               c->cand, c->cap, cand_count, overflow, c->tab, c->nwc, c->filt + 4 * n, sp);
    } else {
        LAUNCH(c, SL_EF_FILTER, (k_ef_filter<false, false>), dim3(c->nwc, n), dim3(64), c->e, (const float*)c->g, src, n,
               c->ld, (uint32_t)c->d, lr, (const uint32_t*)bound, (const uint32_t*)zero_at, use_filter ? 1 : 0,
               c->cand, c->cap, cand_count, overflow, c->tab, c->nwc, c->filt + 4 * n, sp);
    }
    c->msg_split = split;
    if (use_filter) {
        LAUNCH(c, SL_TAB_SUM, k_tab_sum, dim3(c->nspans, n), dim3(1024), (const uint2*)c->tab, c->nwc,
               c->span_sum, c->nspans, (const SelState*)nullptr);
        LAUNCH(c, SL_TAB_DECIDE, k_tab_decide, dim3(n), dim3(256), c->span_sum, c->nspans,
               (const uint32_t*)overflow, (uint32_t)k, (uint32_t)kb, (uint32_t)c->d, n, c->sel, cand_total,
               stat_full, (const uint32_t*)zero_at, c->hist, split ? c->sure_count : (uint32_t*)nullptr,
               split ? c->filt + 7 * n : (uint32_t*)nullptr, split ? c->filt + 8 * n : (uint32_t*)nullptr);
        if (split)
            LAUNCH(c, SL_RESTORE_SURE, k_restore_sure, dim3((c->nwc + 255u) / 256u, n), dim3(256),
                   (const SelState*)c->sel, sp, c->nwc, c->e, c->ld);
        LAUNCH(c, SL_TAB_ORDER, k_tab_order, dim3(c->nspans, n), dim3(1024), (const uint2*)c->tab, c->nwc,
               (const uint32_t*)c->span_sum, c->nspans, (const SelState*)c->sel, (const uint2*)c->cand, c->cap,
               c->sorted_idx, c->sorted_val, c->cap, c->e, c->ld);
    } else {
        LAUNCH(c, SL_SEL_BEGIN_ROWS, k_sel_begin_rows, dim3(n), dim3(256), c->sel, n, (uint32_t)k, (uint32_t)kb,
               (uint32_t)c->d, cand_total, c->hist);
        c->full_selects += n;
    }
    enqueue_select(c, (uint32_t)k, (uint32_t)kb);
    c->have_bound = true;
    c->bound_k = k;
    if (c->sel_k == k) { if (c->sel_run < 2u) c->sel_run += 1u; } else { c->sel_k = k; c->sel_run = 1u; }
    HIP_TRY(c, hipGetLastError());
    c->k_step = k;
    c->q_k[c->msg_slot] = k;
    c->phase = PH_COMPRESSED;
    return DDEF_OK;
}

int ddef_aggregate(ddef_ctx* c) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (c->phase != PH_COMPRESSED) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    // ring form: the messages of this iteration; queue form: the ones sent tau iterations ago,
    // nothing while t < tau (Delta_{t-tau} = 0 by convention, Section 3.2)
    uint32_t src = c->msg_slot;
    uint64_t ka = c->k_step;
    if (c->queue_form) {
        src = (uint32_t)((c->t + c->q_slots - c->tau) % c->q_slots);
        ka = c->t >= c->tau ? c->q_k[src] : 0;
    }
    if (ka) {
        c->agg_split = c->msg_split && !c->queue_form;
        LAUNCH(c, SL_MSG_OFFSETS, k_msg_offsets, dim3((c->ntiles + 1u + 255u) / 256u, c->n), dim3(256),
               (const uint32_t*)c->slot_idx(src), c->msg_ld, (uint32_t)ka, c->ntiles, c->agg_off,
               c->agg_split ? (const uint32_t*)(c->filt + 8 * c->n) : (const uint32_t*)nullptr);
        c->agg_deferred = true;
        c->agg_in_U = false;
        c->agg_slot = src;
    } else {
        c->agg_deferred = false;
        zero_update(c);
    }
    HIP_TRY(c, hipGetLastError());
    c->phase = PH_AGGREGATED;
    return DDEF_OK;
}

int ddef_apply_delayed(ddef_ctx* c, float lr) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (c->phase != PH_AGGREGATED) return DDEF_ESTATE;
    if (std::memcmp(&lr, &c->lr_step, sizeof(float)) != 0) return DDEF_EINVAL;
    DeviceGuard guard(c->device);
    const uint64_t quads = (c->d + 3) / 4;
    if (c->agg_deferred && !c->agg_in_U) {
        LAUNCH(c, SL_AGGREGATE_APPLY, k_aggregate_tiles<true>, dim3(c->ntiles), dim3(256), (float*)nullptr,
               (const uint32_t*)c->slot_idx(c->agg_slot), (const float*)c->slot_val(c->agg_slot), c->msg_ld,
               (const uint32_t*)c->agg_off, c->ntiles, c->n,
               ModelRows{c->slot(c->t), c->slot(c->t + 1), c->capturing ? c->t_dev : nullptr, c->ring,
                         c->ring_slots, c->ld},
               (float)c->n, sure_view(c, c->agg_split));
    } else {
        LAUNCH(c, SL_APPLY, k_apply, dim3((uint32_t)((quads + 63) / 64)), dim3(64), c->slot(c->t),
               c->U, c->slot(c->t + 1), (uint32_t)c->d, (float)c->n);
    }
    HIP_TRY(c, hipGetLastError());
    c->t += 1;
    c->phase = PH_IDLE;
    if (c->opt_fuse) c->grad_live = false;
    return DDEF_OK;
}

static int step_eager(ddef_ctx* c, double delta, float lr) {
    int rc = ddef_grad(c);
    if (rc == DDEF_OK) rc = ddef_ef_compress(c, delta, lr);
    if (rc == DDEF_OK) rc = ddef_aggregate(c);
    if (rc == DDEF_OK) rc = ddef_apply_delayed(c, lr);
    return rc;
}

int ddef_step(ddef_ctx* c, double delta, float lr) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!(delta > 0.0) || !(delta <= 1.0) || !std::isfinite(lr)) return DDEF_EINVAL;
    if (!c->problem_set || c->phase != PH_IDLE) return DDEF_ESTATE;
    const uint64_t k = ddef_k_from_delta(delta, c->d);
    const uint64_t kb = candidate_target(c, k);
    uint32_t lr_bits;
    std::memcpy(&lr_bits, &lr, 4);
    // A steady iteration only: ring form, Top-k, not empty, a filter bound placed for this very k
    // (so that neither a whole-row start nor the sampling of a new bound is part of it), nothing to reallocate,
    // no per-launch events, no second stream.
    const bool steady = c->opt_graph && !c->queue_form && c->compressor == DDEF_COMPRESSOR_TOPK &&
                        !c->profiling && !c->opt_prefetch && c->t >= c->tau && c->have_bound && c->bound_k == k &&
                        c->sel_k == k && c->sel_run >= 2u && !samples_every_iteration(c, k) &&
                        k <= c->msg_ld && candidate_capacity(c, k, kb) <= c->cap;
    if (!steady) return step_eager(c, delta, lr);
    DeviceGuard guard(c->device);
    if (c->graph_exec && (c->graph_k != k || c->graph_lr_bits != lr_bits || c->graph_tau != c->tau)) drop_graph(c);
    if (c->t_dev_value != c->t) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        HIP_TRY(c, hipMemcpy(c->t_dev, &c->t, 8, hipMemcpyHostToDevice));
        c->t_dev_value = c->t;
    }
    if (!c->graph_exec) {
        // record this iteration's launches (nothing runs yet), then run the recording once
        const uint64_t fulls_before = c->full_selects;
        hipGraph_t graph = nullptr;
        HIP_TRY(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
        c->capturing = true;
        rc = step_eager(c, delta, lr);
        if (rc == DDEF_OK) LAUNCH(c, SL_ADVANCE, k_advance, dim3(1), dim3(64), c->t_dev);
        c->capturing = false;
        const hipError_t ended = hipStreamEndCapture(c->stream, &graph);
        if (rc != DDEF_OK || ended != hipSuccess || graph == nullptr) {
            if (graph) (void)hipGraphDestroy(graph);
            c->sticky = DDEF_EHIP;           // the host state has moved on without the device
            return rc != DDEF_OK ? rc : DDEF_EHIP;
        }
        const hipError_t made = hipGraphInstantiate(&c->graph_exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (made != hipSuccess) { c->graph_exec = nullptr; c->sticky = DDEF_EHIP; return DDEF_EHIP; }
        c->graph_k = k; c->graph_lr_bits = lr_bits; c->graph_tau = c->tau;
        c->graph_full_selects = c->full_selects - fulls_before;
        HIP_TRY(c, hipGraphLaunch(c->graph_exec, c->stream));
        c->t_dev_value = c->t;               // the host counter moved during the recording
        return DDEF_OK;
    }
    HIP_TRY(c, hipGraphLaunch(c->graph_exec, c->stream));
    // what the four calls would have left on the host
    c->t += 1;
    c->t_dev_value = c->t;
    c->full_selects += c->graph_full_selects;
    c->graph_replays += 1;
    c->lr_step = lr;
    c->k_step = k;
    c->step_empty = false;
    c->grad_stored = false;
    c->grad_pending = c->opt_fuse != 0;
    c->grad_live = c->opt_fuse == 0;
    c->agg_deferred = true;
    c->agg_in_U = false;
    c->agg_slot = c->msg_slot;
    return DDEF_OK;
}

int ddef_graph_replays(ddef_ctx* c, uint64_t* count) {
    if (!c || !count) return DDEF_EINVAL;
    *count = c->graph_replays;
    return DDEF_OK;
}

int ddef_sync(ddef_ctx* c) {
    int rc = check_ctx(c);
    if (rc) return rc;
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->side) HIP_TRY(c, hipStreamSynchronize(c->side));
    return check_device_flags(c);
}

int ddef_step_index(ddef_ctx* c, uint64_t* t) {
    if (!c || !t) return DDEF_EINVAL;
    *t = c->t;
    return DDEF_OK;
}

int ddef_get_model(ddef_ctx* c, float* host_x) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_x) return DDEF_EINVAL;
    DeviceGuard guard(c->device);
    return copy_row_out(c, c->slot(c->t), host_x);
}

int ddef_objective(ddef_ctx* c, double* host_f) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_f) return DDEF_EINVAL;
    if (!c->problem_set) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    const uint32_t blocks = blocks_for(c, ((c->d + 3u) / 4u + 255u) / 256u, 1, 8);
    const uint32_t most = (uint32_t)c->cus * 8u;
    if (!c->objective_partial) HIP_TRY(c, hipMalloc((void**)&c->objective_partial, (size_t)most * 8u));
    GradSource src = grad_source(c, 0, c->slot(c->t));
    src.t_dev = nullptr;                       // the iterate is named by the host's counter
    LAUNCH(c, SL_OBJECTIVE, k_objective, dim3(blocks), dim3(256), src, (uint32_t)c->d, c->n, c->objective_partial);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    std::vector<double> partial(blocks);
    HIP_TRY(c, hipMemcpy(partial.data(), c->objective_partial, (size_t)blocks * 8u, hipMemcpyDeviceToHost));
    double total = 0.0;
    for (double v : partial) total += v;
    *host_f = 0.5 * total;
    return DDEF_OK;
}

int ddef_set_model(ddef_ctx* c, const float* host_x) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_x) return DDEF_EINVAL;
    if (c->phase != PH_IDLE) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    rc = drop_prefetch(c);                 // a prefetched gradient may have been taken at this snapshot
    if (rc) return rc;
    return copy_row_in(c, c->slot(c->t), host_x);
}

int ddef_get_snapshot(ddef_ctx* c, uint32_t age, float* host_x) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_x || age > c->tau_max || (uint64_t)age > c->t) return DDEF_EINVAL;
    if (c->queue_form || c->phase != PH_IDLE) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    return copy_row_out(c, c->slot(c->t - age), host_x);
}

int ddef_set_snapshot(ddef_ctx* c, uint32_t age, const float* host_x) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_x || age > c->tau_max) return DDEF_EINVAL;
    if (c->queue_form || c->phase != PH_IDLE) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    rc = drop_prefetch(c);
    if (rc) return rc;
    // slots are numbered by iteration modulo the ring size, so ages beyond t wrap harmlessly
    return copy_row_in(c, c->slot(c->t + (uint64_t)c->ring_slots - age), host_x);
}

int ddef_set_step_index(ddef_ctx* c, uint64_t t) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!c->problem_set || c->queue_form || c->phase != PH_IDLE) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    rc = drop_prefetch(c);
    if (rc) return rc;
    c->t = t;
    c->have_bound = false;             // the filter bound belonged to another point of the run
    c->sel_k = 0; c->sel_run = 0;
    c->agg_deferred = false;
    c->k_step = 0;
    return DDEF_OK;
}

int ddef_get_error(ddef_ctx* c, uint32_t worker, float* host_e) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_e || worker >= c->n) return DDEF_EINVAL;
    DeviceGuard guard(c->device);
    return copy_row_out(c, c->e + (uint64_t)worker * c->ld, host_e);
}

int ddef_set_error(ddef_ctx* c, uint32_t worker, const float* host_e) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_e || worker >= c->n) return DDEF_EINVAL;
    if (c->phase != PH_IDLE && c->phase != PH_GRAD) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    return copy_row_in(c, c->e + (uint64_t)worker * c->ld, host_e);
}

int ddef_get_grad(ddef_ctx* c, uint32_t worker, float* host_g) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_g || worker >= c->n) return DDEF_EINVAL;
    if (c->opt_fuse && !c->grad_live) return DDEF_ESTATE;   // fused: the gradient was never stored
    DeviceGuard guard(c->device);
    if (c->opt_fuse && !c->grad_stored && c->phase != PH_IDLE) {
        // generate it from the same inputs (the snapshot is intact until the iteration is applied)
        enqueue_grad(c, c->stream, c->g, c->grad_key(), c->grad_snapshot(), 64u);
        c->grad_stored = true;
    }
    return copy_row_out(c, c->g + (uint64_t)worker * c->ld, host_g);
}

int ddef_get_update(ddef_ctx* c, float* host_U) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!host_U) return DDEF_EINVAL;
    DeviceGuard guard(c->device);
    materialize_update(c);
    return copy_row_out(c, c->U, host_U);
}

// A worker's split message (sure runs + band part of its row) as one list in ascending coordinate
// order, written to the canon buffers.  *merged stays false where the row already holds the whole
// message (no split, a worker that fell back to its row, or no sure entries).
static int canonical_message(ddef_ctx* c, uint32_t worker, bool* merged) {
    *merged = false;
    if (!c->msg_split) return DDEF_OK;
    const uint32_t n = c->n;
    uint32_t sure_total = 0;
    HIP_TRY(c, hipMemcpy(&sure_total, c->filt + 7 * n + worker, 4u, hipMemcpyDeviceToHost));
    if (sure_total == 0u) return DDEF_OK;
    if (c->canon_ld < c->k_step) {
        const uint64_t len = (c->k_step + 1023u) & ~(uint64_t)1023u;
        uint32_t* idx = nullptr;
        float* val = nullptr;
        hipError_t err = hipMalloc((void**)&idx, (size_t)len * 4u);
        if (err == hipSuccess) err = hipMalloc((void**)&val, (size_t)len * 4u);
        if (err != hipSuccess) { if (idx) (void)hipFree(idx); return hip_fail(c, err); }
        if (c->canon_idx) (void)hipFree(c->canon_idx);
        if (c->canon_val) (void)hipFree(c->canon_val);
        c->canon_idx = idx; c->canon_val = val; c->canon_ld = len;
    }
    const SureView sv = sure_view(c, true);
    // where each tile's band entries start in the rows (what ddef_aggregate computes, too), how many
    // sure entries precede each tile (the compaction's chunk counters are idle between selections and
    // have one word per tile), then the merge
    LAUNCH(c, SL_MSG_OFFSETS, k_msg_offsets, dim3((c->ntiles + 1u + 255u) / 256u, n), dim3(256),
           (const uint32_t*)c->slot_idx(c->msg_slot), c->msg_ld, (uint32_t)c->k_step, c->ntiles, c->agg_off,
           (const uint32_t*)(c->filt + 8 * n));
    LAUNCH(c, SL_MESSAGE_MERGE, k_tile_sure_count, dim3((c->ntiles + 255u) / 256u), dim3(256), sv, worker, c->ntiles,
           c->cnt_gt);
    LAUNCH(c, SL_MESSAGE_MERGE, k_tile_scan, dim3(1), dim3(1024), c->cnt_gt, c->ntiles);
    LAUNCH(c, SL_MESSAGE_MERGE, k_message_merge, dim3(c->ntiles), dim3(256), sv, worker,
           (const uint32_t*)c->slot_idx(c->msg_slot), (const float*)c->slot_val(c->msg_slot), c->msg_ld,
           (const uint32_t*)c->agg_off, c->ntiles, (const uint32_t*)c->cnt_gt, c->canon_idx, c->canon_val,
           (uint32_t)c->k_step);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    *merged = true;
    return DDEF_OK;
}

int ddef_get_message(ddef_ctx* c, uint32_t worker, uint32_t* host_idx, float* host_val, uint64_t* k) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!k || worker >= c->n) return DDEF_EINVAL;
    if (c->phase != PH_COMPRESSED && c->phase != PH_AGGREGATED && c->phase != PH_IDLE) return DDEF_ESTATE;
    *k = c->k_step;
    if (!host_idx || !host_val || c->k_step == 0) return DDEF_OK;
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    rc = check_device_flags(c);
    if (rc) return rc;
    bool merged = false;
    rc = canonical_message(c, worker, &merged);
    if (rc) return rc;
    const uint32_t* src_idx = merged ? c->canon_idx : c->slot_idx(c->msg_slot) + (uint64_t)worker * c->msg_ld;
    const float* src_val = merged ? c->canon_val : c->slot_val(c->msg_slot) + (uint64_t)worker * c->msg_ld;
    HIP_TRY(c, hipMemcpy(host_idx, src_idx, (size_t)c->k_step * 4u, hipMemcpyDeviceToHost));
    HIP_TRY(c, hipMemcpy(host_val, src_val, (size_t)c->k_step * 4u, hipMemcpyDeviceToHost));
    return DDEF_OK;
}

int ddef_get_message_codes(ddef_ctx* c, uint32_t worker, uint8_t* host_codes, float* host_steps, uint64_t* k) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!k || worker >= c->n) return DDEF_EINVAL;
    if (c->compressor != DDEF_COMPRESSOR_COMPOSED) return DDEF_ESTATE;
    if (c->phase != PH_COMPRESSED && c->phase != PH_AGGREGATED && c->phase != PH_IDLE) return DDEF_ESTATE;
    *k = c->k_step;
    if (!host_codes || !host_steps || c->k_step == 0) return DDEF_OK;
    if (!c->codes_valid) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    rc = check_device_flags(c);
    if (rc) return rc;
    HIP_TRY(c, hipMemcpy(host_codes, c->codes + (uint64_t)worker * c->codes_ld, (size_t)((c->k_step + 1u) / 2u),
                         hipMemcpyDeviceToHost));
    HIP_TRY(c, hipMemcpy(host_steps, c->steps + (uint64_t)worker * (c->codes_ld / 128u),
                         (size_t)((c->k_step + 255u) / 256u) * 4u, hipMemcpyDeviceToHost));
    return DDEF_OK;
}

int ddef_get_threshold(ddef_ctx* c, uint32_t worker, uint32_t* T, uint64_t* r) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!T || !r || worker >= c->n) return DDEF_EINVAL;
    if (c->k_step == 0) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    SelState s;
    HIP_TRY(c, hipMemcpy(&s, c->sel + worker, sizeof(SelState), hipMemcpyDeviceToHost));
    *T = s.T;
    *r = s.r;
    return DDEF_OK;
}

int ddef_get_filter_state(ddef_ctx* c, uint32_t worker, uint32_t* next_bound, uint32_t* candidates,
                          uint32_t* searched_row) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!next_bound || !candidates || !searched_row || worker >= c->n) return DDEF_EINVAL;
    if (c->k_step == 0) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    SelState s;
    HIP_TRY(c, hipMemcpy(&s, c->sel + worker, sizeof(SelState), hipMemcpyDeviceToHost));
    HIP_TRY(c, hipMemcpy(next_bound, c->filt + worker, 4u, hipMemcpyDeviceToHost));
    *candidates = s.seen;
    *searched_row = s.active;
    return DDEF_OK;
}

int ddef_device_info(ddef_ctx* c, uint32_t* compute_units, uint32_t* wave_size, uint64_t* lds_bytes_per_cu,
                     uint64_t* memory_bytes, uint32_t* clock_khz, uint32_t* memory_clock_khz,
                     uint32_t* memory_bus_bits, char* arch_name, uint32_t name_len) {
    if (!c) return DDEF_EINVAL;
    hipDeviceProp_t prop;
    HIP_TRY(c, hipGetDeviceProperties(&prop, c->device));
    if (compute_units) *compute_units = (uint32_t)prop.multiProcessorCount;
    if (wave_size) *wave_size = (uint32_t)prop.warpSize;
    if (lds_bytes_per_cu) *lds_bytes_per_cu = (uint64_t)prop.maxSharedMemoryPerMultiProcessor;
    if (memory_bytes) *memory_bytes = (uint64_t)prop.totalGlobalMem;
    if (clock_khz) *clock_khz = (uint32_t)prop.clockRate;
    if (memory_clock_khz) *memory_clock_khz = (uint32_t)prop.memoryClockRate;
    if (memory_bus_bits) *memory_bus_bits = (uint32_t)prop.memoryBusWidth;
    if (arch_name && name_len) {
        std::strncpy(arch_name, prop.gcnArchName, name_len - 1u);
        arch_name[name_len - 1u] = '\0';
    }
    return DDEF_OK;
}

int ddef_copy_probe(ddef_ctx* c, uint64_t* bytes_each_way) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (c->phase != PH_IDLE) return DDEF_ESTATE;
    DeviceGuard guard(c->device);
    const uint64_t quads = c->ld / 4u;
    LAUNCH(c, SL_COPY_PROBE, k_copy_f4, dim3((uint32_t)((quads + 63) / 64)), dim3(64), (const float*)c->g, c->g, quads);
    HIP_TRY(c, hipGetLastError());
    if (bytes_each_way) *bytes_each_way = c->ld * 4u;
    return DDEF_OK;
}

int ddef_profile_enable(ddef_ctx* c, int on) {
    int rc = check_ctx(c);
    if (rc) return rc;
    DeviceGuard guard(c->device);
    rc = resolve_profile(c);
    if (rc) return rc;
    if (on) {
        for (int s = 0; s < SL_COUNT; ++s) { c->prof_launches[s] = 0; c->prof_ms[s] = 0.0; }
    }
    c->profiling = on != 0;
    return DDEF_OK;
}

int ddef_profile_slots(void) { return SL_COUNT; }

int ddef_profile_read(ddef_ctx* c, int slot, const char** name, uint64_t* launches, double* total_ms) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (slot < 0 || slot >= SL_COUNT) return DDEF_EINVAL;
    DeviceGuard guard(c->device);
    rc = resolve_profile(c);
    if (rc) return rc;
    if (name) *name = kSlotNames[slot];
    if (launches) *launches = c->prof_launches[slot];
    if (total_ms) *total_ms = c->prof_ms[slot];
    return DDEF_OK;
}

int ddef_full_select_count(ddef_ctx* c, uint64_t* count) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!count) return DDEF_EINVAL;
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    std::vector<uint32_t> fell_back(c->n, 0u);
    HIP_TRY(c, hipMemcpy(fell_back.data(), c->filt + 2 * c->n, (size_t)c->n * 4u, hipMemcpyDeviceToHost));
    uint64_t total = c->full_selects;
    for (uint32_t v : fell_back) total += v;
    *count = total;
    return DDEF_OK;
}

int ddef_set_option(ddef_ctx* c, int option, int64_t value) {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (c->phase != PH_IDLE) return DDEF_ESTATE;
    drop_graph(c);
    switch (option) {
        case DDEF_OPT_FORCE_FULL_SELECT: c->opt_force_full = value != 0; return DDEF_OK;
        case DDEF_OPT_PREFETCH_GRAD:
            c->opt_prefetch = value != 0;
            if (!c->opt_prefetch) return drop_prefetch(c);
            return DDEF_OK;
        case DDEF_OPT_FUSE_GRAD:
            c->opt_fuse = value != 0;
            if (c->opt_fuse) return drop_prefetch(c);
            return DDEF_OK;
        case DDEF_OPT_GRAPH: c->opt_graph = value != 0; return DDEF_OK;
        case DDEF_OPT_DENSE_SPLIT:
            if (value < 0 || value > 4) return DDEF_EINVAL;
            c->opt_split = value;
            return DDEF_OK;
        case DDEF_OPT_COMPOSED_BOUND:
            if (value < 0 || value > 2) return DDEF_EINVAL;
            c->opt_composed_bound = value;
            return DDEF_OK;
        case DDEF_OPT_RANDK_BUCKET_PERCENT:
            if (value < 0 || value > 400) return DDEF_EINVAL;
            c->opt_bucket_percent = value;
            return DDEF_OK;
        case DDEF_OPT_CANDIDATE_SLACK_X16:
            if (value < 16 || value > 1024) return DDEF_EINVAL;
            c->opt_slack_x16 = value;
            return DDEF_OK;
        default: return DDEF_EINVAL;
    }
}

}  // extern "C"

// ---- error feedback + Top-k on the caller's buffers, without any allocation -----------------
// Work memory of ddef_ef_compress_static: selection state, digit histograms, flag words, slot
// counters and the per-chunk counts of the compaction, for at most kStaticWorkers workers and
// kStaticChunks 4096-coordinate chunks over all workers together.  One copy per GPU, for the life
// of the process.
namespace {

constexpr uint32_t kStaticWorkers = 64;
constexpr uint64_t kStaticChunks = (uint64_t)1 << 21;
constexpr size_t kStaticSelOff = 0;
constexpr size_t kStaticSelBytes = (sizeof(SelState) * kStaticWorkers + 255u) & ~(size_t)255u;
constexpr size_t kStaticFiltOff = kStaticSelOff + kStaticSelBytes;
constexpr size_t kStaticFiltBytes = ((size_t)6 * kStaticWorkers * 4u + 255u) & ~(size_t)255u;
constexpr size_t kStaticHistOff = kStaticFiltOff + kStaticFiltBytes;
constexpr size_t kStaticHistBytes = (size_t)3 * kStaticWorkers * 2u * 2048u * 4u;
constexpr size_t kStaticCountersOff = kStaticHistOff + kStaticHistBytes;
constexpr size_t kStaticCountersBytes = (size_t)kStaticWorkers * kSubs * kSubStride * 4u;
constexpr size_t kStaticGtOff = kStaticCountersOff + kStaticCountersBytes;
constexpr size_t kStaticEqOff = kStaticGtOff + kStaticChunks * 4u;
constexpr size_t kStaticBytes = kStaticEqOff + kStaticChunks * 4u;

constexpr int kStaticDevices = 64;
std::mutex g_static_mutex;
unsigned char* g_static_ptr[kStaticDevices] = {};     // device address of `scratch` on each GPU
int g_static_cus[kStaticDevices] = {};

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

// Device address of this GPU's copy of `scratch` (looked up once per device, with that device
// current) and its compute-unit count.
int static_scratch(int device, unsigned char** ptr, int* cus) {
    if (device < 0 || device >= kStaticDevices) return DDEF_EINVAL;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[device]) {
        void* at = nullptr;
        hipError_t err = hipGetSymbolAddress(&at, HIP_SYMBOL(scratch));
        if (err != hipSuccess || at == nullptr) { (void)hipGetLastError(); return DDEF_EHIP; }
        int count = 0;
        err = hipDeviceGetAttribute(&count, hipDeviceAttributeMultiprocessorCount, device);
        if (err != hipSuccess || count <= 0) { (void)hipGetLastError(); count = 256; }
        g_static_cus[device] = count;
        g_static_ptr[device] = static_cast<unsigned char*>(at);
    }
    *ptr = g_static_ptr[device];
    *cus = g_static_cus[device];
    return DDEF_OK;
}

}  // namespace

extern "C" int ddef_ef_compress_static(float* dev_e, const float* dev_g, uint64_t ld, uint64_t d, uint32_t n,
                                       double delta, float lr, uint32_t* dev_msg_idx, float* dev_msg_val,
                                       uint64_t msg_ld, void* hip_stream) {
    if (!dev_e || !dev_g || !dev_msg_idx || !dev_msg_val) return DDEF_EINVAL;
    if (d == 0 || d >= 0xFFFFE000ull || n == 0 || n > kStaticWorkers) return DDEF_EINVAL;
    if (!(delta > 0.0) || !(delta <= 1.0) || !std::isfinite(lr)) return DDEF_EINVAL;
    if (ld < d || (ld & 3u) != 0u) return DDEF_EINVAL;
    if ((reinterpret_cast<uintptr_t>(dev_e) & 15u) != 0u || (reinterpret_cast<uintptr_t>(dev_g) & 15u) != 0u)
        return DDEF_EINVAL;
    const uint64_t nchunks = (d + 4095u) / 4096u;
    if (nchunks * n > kStaticChunks) return DDEF_EINVAL;          // beyond what the work memory holds
    const uint64_t k = ddef_k_from_delta(delta, d);
    if (msg_ld < k) return DDEF_EINVAL;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) { (void)hipGetLastError(); return DDEF_EHIP; }
    unsigned char* base = nullptr;
    int cus = 256;
    int rc = static_scratch(device, &base, &cus);
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    SelState* sel = reinterpret_cast<SelState*>(base + kStaticSelOff);
    uint32_t* filt = reinterpret_cast<uint32_t*>(base + kStaticFiltOff);
    uint32_t* hist = reinterpret_cast<uint32_t*>(base + kStaticHistOff);
    uint32_t* counters = reinterpret_cast<uint32_t*>(base + kStaticCountersOff);
    uint32_t* cnt_gt = reinterpret_cast<uint32_t*>(base + kStaticGtOff);
    uint32_t* cnt_eq = reinterpret_cast<uint32_t*>(base + kStaticEqOff);
    uint32_t *bound = filt, *overflow = filt + n, *cand_total = filt + 3 * n, *nonfinite = filt + 4 * n,
             *zero_at = filt + 5 * n;
    auto blocks = [&](uint64_t row_blocks, uint32_t per_cu) {
        uint64_t budget = (uint64_t)cus * per_cu / n;
        if (budget < 1) budget = 1;
        const uint64_t b = row_blocks < budget ? row_blocks : budget;
        return (uint32_t)(b < 1 ? 1 : b);
    };
    // p = e + lr*g over e; every state word the later kernels read is written by a kernel of this
    // call first (k_sel_begin_rows: selection state and histograms; k_chunk_count: the counts), so
    // what an earlier call left in the work memory does not matter
    const uint32_t groups = (uint32_t)((d + 255u) / 256u);
    const GradSource none{};
    hipLaunchKernelGGL((k_ef_filter<false, false>), dim3(groups, n), dim3(64), 0, stream, dev_e, dev_g, none, n, ld,
                       (uint32_t)d, lr, (const uint32_t*)nullptr, (const uint32_t*)nullptr, 0, (uint2*)nullptr,
                       (uint64_t)0, (uint32_t*)nullptr, (uint32_t*)nullptr, (uint2*)nullptr, groups, nonfinite,
                       SureRuns{});
    hipLaunchKernelGGL(k_sel_begin_rows, dim3(n), dim3(256), 0, stream, sel, n, (uint32_t)k, (uint32_t)k,
                       (uint32_t)d, cand_total, hist);
    const SelViews vs{dev_e, ld, (uint32_t)d, (const float*)nullptr, (const uint32_t*)nullptr, (uint64_t)0,
                      (const uint32_t*)cand_total};
    const uint32_t gx = blocks((d + 1023u) / 1024u, 8);
    for (int level = 0; level < 3; ++level) {
        uint32_t* h = hist + (uint64_t)level * n * 2 * 2048;
        hipLaunchKernelGGL(k_digit_hist, dim3(gx, n), dim3(256), 0, stream, vs, (const SelState*)sel, h, level);
        hipLaunchKernelGGL(k_digit_pick, dim3(n, 2), dim3(256), 0, stream, sel, (const uint32_t*)h, level);
    }
    const uint32_t gc = blocks(nchunks, 8);
    hipLaunchKernelGGL(k_chunk_count, dim3(gc, n), dim3(256), 0, stream, vs, (const SelState*)sel, cnt_gt, cnt_eq,
                       (uint32_t)nchunks);
    hipLaunchKernelGGL(k_chunk_scan, dim3(n), dim3(1024), 0, stream, vs, sel, cnt_gt, cnt_eq, (uint32_t)nchunks,
                       (uint32_t)k, (uint32_t)k, bound, zero_at, counters, overflow);
    hipLaunchKernelGGL(k_chunk_emit, dim3(gc, n), dim3(256), 0, stream, vs, (const SelState*)sel,
                       (const uint32_t*)cnt_gt, (const uint32_t*)cnt_eq, (uint32_t)nchunks, dev_e, dev_msg_idx,
                       dev_msg_val, msg_ld, (uint32_t)k, 1);
    if (hipGetLastError() != hipSuccess) return DDEF_EHIP;
    return DDEF_OK;
}
