// Internal: kernel declarations shared by the kernel file and the C-ABI file.
#ifndef DDEF_KERNELS_H
#define DDEF_KERNELS_H
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ddef {

// A worker's candidate buffer is split into this many parts, each with its own slot counter.
constexpr uint32_t kSubs = 256;
// Each slot counter sits in a cache line of its own (stride in 32-bit words), so that atomics
// on different counters do not queue up behind one line.
constexpr uint32_t kSubStride = 32;
// The run table is scanned in spans of this many 256-entry groups (one block each).
constexpr uint32_t kSpan = 1024;
constexpr uint32_t kTile = 4096;      // coordinates per block of the tile sum

// Per-worker selection state in device memory.
struct SelState {
    uint32_t active;      // 1: search the whole row; 0: search the filtered candidates; 2: invariant broken;
                          // 3: composed compressor, too few kept entries passed the bound: repeat the pass without it
    uint32_t prefix[2];   // magnitude pattern built so far for rank 0 (k) and rank 1 (filter)
    uint32_t krem[2];     // rank still to find inside the current prefix group (1-based)
    uint32_t T, r;        // threshold pattern and how many entries equal to T are sent
    uint32_t next_bound;  // magnitude pattern of the rank-1 entry
    uint32_t seen;        // candidates the filter caught in the last selection
    uint32_t T_prev;      // threshold pattern of the selection before the last one
    uint32_t k_prev;      // its k (0: none)
    uint32_t zero_used;   // candidates at or above this pattern were written to e as +0 ahead of time
};

// Where the selection kernels find a worker's entries: its whole row of e (d entries, the
// position is the coordinate) or its ordered candidates (cand_total[w] entries of
// cand_val / cand_idx rows of `cap` entries), chosen per worker by SelState::active.
struct SelViews {
    const float* e;
    uint64_t ld;
    uint32_t d;
    const float* cand_val;
    const uint32_t* cand_idx;
    uint64_t cap;
    const uint32_t* cand_total;
};

// Everything the synthetic gradient of one iteration is made from.
struct GradSource {
    const float* lambda;
    const float* xstar;
    const float* xs;             // snapshot x_{t-tau}
    uint32_t seed_lo, seed_hi, t_lo, t_hi;
    int kind;
    float scale;
    float zeta;                  // 0: all workers share the optimum xstar
    // Inside a captured graph nothing may change from launch to launch, so the iteration number
    // comes from device memory (t_dev non-null) and with it the noise key (t_lo, t_hi) and the
    // snapshot xs = ring + ((t - tau) mod ring_slots) * ring_ld, both overriding the fields above.
    const uint64_t* t_dev;
    const float* ring;
    uint32_t ring_slots, tau;
    uint64_t ring_ld;
};

// Dense messages, sure / band split: where the accumulate pass records the candidates that are sure
// to be sent (runs of (index, value) per 256-coordinate group, like the candidate buffer), and the
// same buffers as the aggregation reads them.
struct SureRuns {
    const uint32_t* sure_at;     // per worker: magnitude pattern from which a candidate counts as sure
    uint2* sure;                 // [n][cap] records
    uint64_t cap;
    uint32_t* count;             // [n][kSubs * kSubStride] slot counters
    uint2* stab;                 // [n][ngroups] run table (first slot, count)
};
struct SureView {
    const uint2* sure;           // null: messages are not split
    uint64_t cap;
    const uint2* stab;
    uint32_t ngroups;
    const uint32_t* total;       // per worker: sure entries that belong to its message (0: none)
};

__global__ void k_grad(GradSource s, float* g, uint64_t ld, uint32_t d, uint32_t n);
__global__ void k_objective(GradSource s, uint32_t d, uint32_t n, double* partial);
template <bool kFusedGrad, bool kSplit>
__global__ void k_ef_filter(float* e, const float* g, GradSource src, uint32_t n, uint64_t ld, uint32_t d,
                            float lr, const uint32_t* bound, const uint32_t* zero_at, int use_filter, uint2* cand, uint64_t cap,
                            uint32_t* cand_count, uint32_t* overflow, uint2* tab, uint32_t ngroups,
                            uint32_t* nonfinite, SureRuns sp);
__global__ void k_tab_sum(const uint2* tab, uint32_t nwc, uint32_t* span_sum, uint32_t nspans, const SelState* gate);
__global__ void k_tab_decide(uint32_t* span_sum, uint32_t nspans, const uint32_t* overflow, uint32_t k,
                             uint32_t kb, uint32_t d, uint32_t n, SelState* sel, uint32_t* cand_total,
                             uint32_t* stat_full, const uint32_t* zero_at, uint32_t* hist, uint32_t* sure_count,
                             uint32_t* sure_total, uint32_t* msg_count);
__global__ void k_restore_sure(const SelState* sel, SureRuns sp, uint32_t ngroups, float* e, uint64_t ld);
__global__ void k_sel_begin_rows(SelState* sel, uint32_t n, uint32_t k, uint32_t kb, uint32_t d,
                                 uint32_t* cand_total, uint32_t* hist);
__global__ void k_tab_order(const uint2* tab, uint32_t ngroups, const uint32_t* span_off, uint32_t nspans,
                            const SelState* sel, const uint2* cand, uint64_t cap, uint32_t* sorted_idx,
                            float* sorted_val, uint64_t out_ld, float* e_row, uint64_t e_ld);
__global__ void k_randk_mark(uint32_t* bitmap, uint64_t bitmap_ld, uint32_t d, uint32_t k, uint32_t seed_lo,
                             uint32_t seed_hi, uint32_t t_lo, uint32_t t_hi, const SelState* gate);
__global__ void k_randk_bin(uint32_t* bucket, uint64_t bucket_ld, uint32_t bucket_cap, uint32_t* gcount,
                            uint32_t region_bits, uint32_t regions, uint32_t* bitmap, uint64_t bitmap_ld, uint32_t d,
                            uint32_t k, uint32_t seed_lo, uint32_t seed_hi, uint32_t t_lo, uint32_t t_hi,
                            const SelState* gate);
__global__ void k_randk_fill(const uint32_t* bucket, uint64_t bucket_ld, uint32_t bucket_cap, uint32_t* gcount,
                             uint32_t region_bits, uint32_t regions, uint32_t* bitmap, uint64_t bitmap_ld, uint32_t d,
                             const SelState* gate);
__global__ void k_ef_randk(float* e, const float* g, uint64_t ld, uint32_t d, float lr, int zero_marked, int accumulate,
                           const uint32_t* bound, uint32_t* bitmap,
                           uint64_t bitmap_ld, uint2* cand, uint64_t cap, uint32_t* cand_count,
                           uint32_t* overflow, uint2* tab, uint32_t ngroups, uint32_t* nonfinite,
                           const SelState* gate);
__global__ void k_tab_decide_randk(uint32_t* span_sum, uint32_t nspans, uint32_t* overflow, uint32_t k,
                                   SelState* sel, uint32_t* cand_total, uint32_t* cand_count);
__global__ void k_tab_decide_composed(uint32_t* span_sum, uint32_t nspans, uint32_t* overflow, uint32_t k1, uint32_t k,
                                      uint32_t n, int exact, SelState* sel, uint32_t* cand_total, uint32_t* cand_count,
                                      uint32_t* hist, uint32_t* stat_repeat, int gated);
__global__ void k_quantize4(const uint32_t* msg_idx, float* msg_val, uint64_t msg_ld, uint32_t k, const SelState* sel,
                            float* e, uint64_t ld, uint8_t* codes, uint64_t codes_ld, float* steps, uint64_t steps_ld);
__global__ void k_digit_hist(SelViews vs, const SelState* sel, uint32_t* hist, int level);
__global__ void k_digit_pick(SelState* sel, const uint32_t* hist, int level);
__global__ void k_chunk_count(SelViews vs, const SelState* sel, uint32_t* cnt_gt, uint32_t* cnt_eq,
                              uint32_t stride);
__global__ void k_chunk_scan(SelViews vs, SelState* sel, uint32_t* cnt_gt, uint32_t* cnt_eq,
                             uint32_t stride, uint32_t k, uint32_t kb, uint32_t* bound, uint32_t* zero_at,
                             uint32_t* cand_count, uint32_t* overflow);
template <bool kFusedGrad>
__global__ void k_sample_p(const float* e, const float* g, GradSource src, uint64_t ld, uint32_t d, float lr, uint32_t stride,
                           uint32_t count,
                           float* sample, uint64_t sample_ld);
__global__ void k_sample_begin(SelState* sel, uint32_t n, uint32_t k_s, uint32_t kb_s, uint32_t count,
                               uint32_t* sample_total, uint32_t* hist);
__global__ void k_sample_finish(const SelState* sel, uint32_t n, uint32_t* bound, uint32_t* zero_at,
                                uint32_t* sure_at, int sure_mode);
__global__ void k_chunk_emit(SelViews vs, const SelState* sel, const uint32_t* out_base,
                             const uint32_t* eq_before, uint32_t stride, float* e, uint32_t* msg_idx,
                             float* msg_val, uint64_t msg_ld, uint32_t k, int fix_e);
__global__ void k_apply(const float* x, const float* U, float* xn, uint32_t d, float nf);
__global__ void k_msg_offsets(const uint32_t* idx, uint64_t msg_ld, uint32_t k, uint32_t ntiles, uint32_t* off,
                              const uint32_t* count);
// Where the model update reads x_t and writes x_{t+1}: given rows, or (inside a captured graph)
// slots t and t+1 of the ring with t read from device memory.
struct ModelRows {
    const float* x;
    float* xn;
    const uint64_t* t_dev;
    float* ring;
    uint32_t ring_slots;
    uint64_t ring_ld;
};
template <bool kApply>
__global__ void k_aggregate_tiles(float* U, const uint32_t* idx, const float* val, uint64_t msg_ld,
                                  const uint32_t* off, uint32_t ntiles, uint32_t n, ModelRows rows, float nf,
                                  SureView sv);
__global__ void k_tile_sure_count(SureView sv, uint32_t w, uint32_t ntiles, uint32_t* tile_count);
__global__ void k_tile_scan(uint32_t* tile_count, uint32_t ntiles);
__global__ void k_message_merge(SureView sv, uint32_t w, const uint32_t* idx, const float* val, uint64_t msg_ld,
                                const uint32_t* off, uint32_t ntiles, const uint32_t* sure_before, uint32_t* out_idx,
                                float* out_val, uint32_t k);
__global__ void k_advance(uint64_t* t_dev);
__global__ void k_fill_f4(float* p, uint64_t quads);
__global__ void k_copy_f4(const float* src, float* dst, uint64_t quads);

}  // namespace ddef
#endif
