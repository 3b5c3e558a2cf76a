// Internal: kernel declarations shared by the kernel file and the C-ABI file.
#ifndef DDEF_KERNELS_H
#define DDEF_KERNELS_H
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ddef {

// Per-worker selection state in device memory.
struct SelState {
    uint32_t active;      // 1: this worker's selection runs over the whole row
    uint32_t prefix[2];   // magnitude pattern built so far for rank 0 (k) and rank 1 (filter)
    uint32_t krem[2];     // rank still to find inside the current prefix group (1-based)
    uint32_t T, r;        // threshold pattern and how many entries equal to T are sent
    uint32_t next_bound;  // magnitude pattern of the rank-1 entry
};

__global__ void k_grad(const float* lambda, const float* xstar, const float* xs, float* g,
                       uint64_t ld, uint32_t d, uint32_t n, uint32_t seed_lo, uint32_t seed_hi,
                       uint32_t t_lo, uint32_t t_hi, int kind, float scale);
__global__ void k_ef_accumulate(float* e, const float* g, uint64_t ld, uint32_t d, float lr);
__global__ void k_digit_hist(const float* src, uint64_t ld, uint32_t cnt_fixed,
                             const uint32_t* cnt_dev, const SelState* sel, uint32_t* hist, int level);
__global__ void k_digit_pick(SelState* sel, uint32_t* hist, int level);
__global__ void k_chunk_count(const float* e, uint64_t ld, uint32_t d, const SelState* sel,
                              uint32_t* cnt_gt, uint32_t* cnt_eq, uint32_t nchunks);
__global__ void k_chunk_scan(const SelState* sel, uint32_t* cnt_gt, uint32_t* cnt_eq, uint32_t nchunks);
__global__ void k_chunk_emit(float* e, uint64_t ld, uint32_t d, const SelState* sel,
                             const uint32_t* out_base, const uint32_t* eq_before, uint32_t nchunks,
                             uint32_t* msg_idx, float* msg_val, uint64_t msg_ld, uint32_t k);
__global__ void k_scatter_add(float* U, const uint32_t* idx, const float* val, uint32_t k, uint32_t d);
__global__ void k_apply(const float* x, const float* U, float* xn, uint32_t d, float nf);
__global__ void k_fill_u32(uint32_t* p, uint64_t count, uint32_t value);
__global__ void k_copy_f4(const float* src, float* dst, uint64_t quads);
__global__ void k_sel_begin(SelState* sel, uint32_t n, uint32_t k, uint32_t kb, uint32_t all_active);

}  // namespace ddef
#endif
