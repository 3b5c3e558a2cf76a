// Device kernels of the DD-EF-SGD hot path for gfx950 (wave64).
//
// Layout in HBM: every length-d vector lives in a row of `ld` floats (d rounded up to the
// 4096-element chunk), so rows of e[n][ld], g[n][ld] and the snapshot ring start 16 KiB
// aligned and every 16-byte access of a row stays inside the row's allocation.  Entries
// past d are never counted, selected or compared.
//
// Everything here is HBM-bound streaming, histogramming in LDS, wave ballots and prefix
// scans; there is no dense contraction, hence no MFMA.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ddef_kernels.h"

namespace ddef {

// ------------------------------------------------------------------------------------
// small device helpers
// ------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

// number of set bits of `mask` strictly below this lane
__device__ __forceinline__ uint32_t mask_rank(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t up = __shfl_up(v, off, 64);
        if (lane_id() >= (uint32_t)off) v += up;
    }
    return v;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Exclusive prefix of `v` over the block in thread order; *total receives the block sum.
// `lds` holds at least blockDim.x/64 + 1 words.  Contains two barriers; every thread of the
// block must call it.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* lds, uint32_t* total) {
    const uint32_t wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    uint32_t incl = wave_incl_scan(v);
    if (lane_id() == 63u) lds[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
    for (uint32_t w = 0; w < nw; ++w) {
        uint32_t s = lds[w];
        if (w < wave) before += s;
        all += s;
    }
    __syncthreads();
    *total = all;
    return before + incl - v;
}

typedef float vec4f __attribute__((ext_vector_type(4)));

// 16-byte load that does not displace reusable lines from the caches (streamed-once data)
__device__ __forceinline__ float4 load_stream4(const float* p) {
    const vec4f v = __builtin_nontemporal_load(reinterpret_cast<const vec4f*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void store_stream4(float* p, const float (&v)[4]) {
    const vec4f x = {v[0], v[1], v[2], v[3]};
    __builtin_nontemporal_store(x, reinterpret_cast<vec4f*>(p));
}

__device__ __forceinline__ uint32_t mag_key(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// True for the whole wave when any lane holds an Inf or NaN among its four values (entries of
// the row padding are zero and never trigger).
__device__ __forceinline__ bool note_nonfinite(const float (&v)[4]) {
    bool bad = false;
#pragma unroll
    for (int c = 0; c < 4; ++c) bad |= mag_key(v[c]) >= 0x7f800000u;
    return __ballot(bad) != 0ull;
}

// ------------------------------------------------------------------------------------
// gradient noise: Philox4x32-10 (Salmon et al., SC'11) + Box-Muller out of +,-,*,/,sqrt and
// explicit fused multiply-adds.  Every fp32 operation is written out (the file is compiled
// with contraction off, so the compiler fuses nothing on its own) so that the CPU can
// reproduce each draw bit for bit.
// ------------------------------------------------------------------------------------
struct U4 { uint32_t a, b, c, d; };

__device__ __forceinline__ U4 philox_block(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                           uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // one 32x32->64 multiply per product (both halves are needed)
        const uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t y0 = (uint32_t)(prod1 >> 32) ^ c1 ^ k0, y2 = (uint32_t)(prod0 >> 32) ^ c3 ^ k1;
        c0 = y0; c1 = (uint32_t)prod1; c2 = y2; c3 = (uint32_t)prod0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return U4{c0, c1, c2, c3};
}

// -2 ln u, u = ((w >> 8) + 1) 2^-24: split off the exponent, fold the mantissa into
// (sqrt 1/2, sqrt 2], ln(1 + f) = f + f^2 g(f) for f = m - 1 with a degree-7 polynomial g (the
// Chebyshev interpolant of (ln(1+f) - f) / f^2 on that interval) in Horner form with explicit
// fused multiply-adds (single rounding, reproducible on the CPU); no division.
__device__ __forceinline__ float radius_sq(uint32_t w) {
    const uint32_t fb = __float_as_uint((float)((w >> 8) + 1u));
    int ex = (int)(fb >> 23) - 127;
    const uint32_t mant = fb & 0x7fffffu;
    float m = __uint_as_float(mant | 0x3f800000u);
    if (mant > 0x3504f3u) { m = m * 0.5f; ex += 1; }
    const float f = m - 1.0f;
    float h = 0x1.67ed28p-4f;
    h = __builtin_fmaf(h, f, -0x1.21fd54p-3f);
    h = __builtin_fmaf(h, f, 0x1.2fd102p-3f);
    h = __builtin_fmaf(h, f, -0x1.53bb74p-3f);
    h = __builtin_fmaf(h, f, 0x1.99071p-3f);
    h = __builtin_fmaf(h, f, -0x1.000302p-2f);
    h = __builtin_fmaf(h, f, 0x1.555638p-2f);
    h = __builtin_fmaf(h, f, -0x1.fffffep-2f);
    const float lnm = __builtin_fmaf(f * f, h, f);
    float v = __builtin_fmaf((float)(24 - ex), 0x1.62e43p-1f, -lnm);
    v = v < 0.0f ? 0.0f : v;
    return 2.0f * v;
}

// (cos, sin) of 2 pi ((w >> 8) + 1/2) 2^-24: quadrant after an eighth-turn shift, Taylor
// series on (-pi/4, pi/4).
__device__ __forceinline__ void circle_point(uint32_t w, float& co, float& si) {
    const uint32_t b = ((w >> 8) + 0x200000u) & 0xffffffu;
    const uint32_t quad = b >> 22;
    const int rem = (int)(b & 0x3fffffu) - 0x200000;
    const float phi = (float)(2 * rem + 1) * 0x1.921fb6p-23f;
    const float p2 = phi * phi;
    float a = 1.0f / 362880.0f;
    a = __builtin_fmaf(a, p2, -1.0f / 5040.0f);
    a = __builtin_fmaf(a, p2, 1.0f / 120.0f);
    a = __builtin_fmaf(a, p2, -1.0f / 6.0f);
    a = __builtin_fmaf(a, p2, 1.0f);
    const float s = phi * a;
    float c = -1.0f / 3628800.0f;
    c = __builtin_fmaf(c, p2, 1.0f / 40320.0f);
    c = __builtin_fmaf(c, p2, -1.0f / 720.0f);
    c = __builtin_fmaf(c, p2, 1.0f / 24.0f);
    c = __builtin_fmaf(c, p2, -0.5f);
    c = __builtin_fmaf(c, p2, 1.0f);
    co = (quad == 0u) ? c : (quad == 1u) ? -s : (quad == 2u) ? -c : s;
    si = (quad == 0u) ? s : (quad == 1u) ? c : (quad == 2u) ? -s : -c;
}

// Normal draws for the four coordinates 4q .. 4q+3 from the one block of counter (q, worker, t):
// two Box-Muller pairs, (R cos, R sin) from words (0, 1) and from words (2, 3).
__device__ __forceinline__ void draw_normal4(uint32_t q, uint32_t worker, uint32_t t_lo, uint32_t t_hi,
                                             uint32_t seed_lo, uint32_t seed_hi, float (&z)[4]) {
    const U4 w = philox_block(q, worker, t_lo, t_hi, seed_lo, seed_hi);
    float co, si;
    float radius = __builtin_sqrtf(radius_sq(w.a));
    circle_point(w.b, co, si);
    z[0] = radius * co;
    z[1] = radius * si;
    radius = __builtin_sqrtf(radius_sq(w.c));
    circle_point(w.d, co, si);
    z[2] = radius * co;
    z[3] = radius * si;
}

// Student-t(3) from three words (radius, angle, chi-square):
// z0 / sqrt((z1^2 + chi2_2) / 3) with (z0, z1) = (R cos, R sin) the Box-Muller pair of the first
// two words and chi2_2 = -2 ln u of the third, computed as
// cos * sqrt(3 R^2 / (R^2 sin^2 + chi2_2)): one division and one square root.
__device__ __forceinline__ float t3_of(uint32_t w_radius, uint32_t w_angle, uint32_t w_chi) {
    float c01, s01;
    const float r2 = radius_sq(w_radius);
    circle_point(w_angle, c01, s01);
    const float chi2_3 = __builtin_fmaf(r2, s01 * s01, radius_sq(w_chi));
    if (chi2_3 == 0.0f) return 0.0f;
    const float ratio = (3.0f * r2) / chi2_3;
    return c01 * __builtin_sqrtf(ratio);
}

// Student-t(3) draws for the four coordinates 4q .. 4q+3: the twelve words of the blocks with
// counters (3q, worker, t), (3q+1, ..), (3q+2, ..), three to a coordinate in order.
__device__ __forceinline__ void draw_t3x4(uint32_t q, uint32_t worker, uint32_t t_lo, uint32_t t_hi,
                                          uint32_t seed_lo, uint32_t seed_hi, float (&z)[4]) {
    const U4 a = philox_block(3u * q, worker, t_lo, t_hi, seed_lo, seed_hi);
    const U4 b = philox_block(3u * q + 1u, worker, t_lo, t_hi, seed_lo, seed_hi);
    const U4 c = philox_block(3u * q + 2u, worker, t_lo, t_hi, seed_lo, seed_hi);
    z[0] = t3_of(a.a, a.b, a.c);
    z[1] = t3_of(a.d, b.a, b.b);
    z[2] = t3_of(b.c, b.d, c.a);
    z[3] = t3_of(c.b, c.c, c.d);
}

// ------------------------------------------------------------------------------------
// S0  g_i = lambda * (x_{t-tau} - x*) + scale * z      (Assumption 2; stale iterate)
// ------------------------------------------------------------------------------------
// The iteration number from device memory, where the launch is part of a captured graph.
__device__ __forceinline__ void resolve_iteration(GradSource& s) {
    if (s.t_dev == nullptr) return;
    const uint64_t t = *s.t_dev;
    s.t_lo = (uint32_t)t;
    s.t_hi = (uint32_t)(t >> 32);
    s.xs = s.ring + ((t - s.tau) % s.ring_slots) * s.ring_ld;
}

// what all workers share at four consecutive coordinates
struct Shared4 { float lam[4], opt[4], x[4]; };

__device__ __forceinline__ Shared4 grad_shared4(const GradSource& s, uint32_t j) {
    const float4 lam = *reinterpret_cast<const float4*>(s.lambda + j);
    const float4 xo = *reinterpret_cast<const float4*>(s.xstar + j);
    const float4 xv = *reinterpret_cast<const float4*>(s.xs + j);
    return Shared4{{lam.x, lam.y, lam.z, lam.w}, {xo.x, xo.y, xo.z, xo.w}, {xv.x, xv.y, xv.z, xv.w}};
}

// worker's gradient at coordinates j..j+3 (zero past d, which keeps the row padding at zero).
// With zeta != 0 the worker's objective has its own optimum x* + zeta * u_i (heterogeneous
// local objectives, Assumption 3), u_i a fixed standard normal vector drawn under the step
// key 2^64 - 2, which no iteration uses.
__device__ __forceinline__ void grad_quad(const GradSource& s, const Shared4& sh, uint32_t worker,
                                          uint32_t j, uint32_t d, float (&out)[4]) {
    float shift[4] = {0.f, 0.f, 0.f, 0.f}, z[4] = {0.f, 0.f, 0.f, 0.f};
    if (s.zeta != 0.0f) draw_normal4(j >> 2, worker, 0xfffffffeu, 0xffffffffu, s.seed_lo, s.seed_hi, shift);
    if (s.kind == 1) {
        draw_normal4(j >> 2, worker, s.t_lo, s.t_hi, s.seed_lo, s.seed_hi, z);
    } else if (s.kind == 2) {
        draw_t3x4(j >> 2, worker, s.t_lo, s.t_hi, s.seed_lo, s.seed_hi, z);
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        float optimum = sh.opt[c];
        if (s.zeta != 0.0f) optimum = sh.opt[c] + s.zeta * shift[c];
        const float mean = sh.lam[c] * (sh.x[c] - optimum);
        float xi = 0.0f;
        if (s.kind != 0) xi = s.scale * z[c];
        out[c] = (j + c < d) ? mean + xi : 0.0f;
    }
}

// One thread owns four consecutive coordinates and loops over the workers, so lambda, x* and
// the snapshot are read once for all n workers.
__global__ __launch_bounds__(256) void k_grad(GradSource s, float* __restrict__ g, uint64_t ld, uint32_t d,
                                              uint32_t n) {
    resolve_iteration(s);
    const uint32_t quads = (d + 3u) >> 2;
    for (uint32_t q = blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += gridDim.x * blockDim.x) {
        const uint32_t j = q << 2;
        const Shared4 sh = grad_shared4(s, j);
        for (uint32_t i = 0; i < n; ++i) {
            float out[4];
            grad_quad(s, sh, i, j, d, out);
            *reinterpret_cast<float4*>(g + (uint64_t)i * ld + j) = make_float4(out[0], out[1], out[2], out[3]);
        }
    }
}

// The objective at the iterate x (Section 2.1, problem (1)): f(x) = (1/n) sum_i f_i(x) with
// f_i(x) = 1/2 sum_j lambda_j (x_j - x*_ij)^2 and x*_i = x* + zeta u_i as in the gradient,
// accumulated in double.  Each block writes the sum of its coordinates' terms (without the
// factor 1/2) to partial[blockIdx.x]; the host adds the partials in block order.
__global__ __launch_bounds__(256) void k_objective(GradSource s, uint32_t d, uint32_t n,
                                                   double* __restrict__ partial) {
    __shared__ double red[4];
    const uint32_t quads = (d + 3u) >> 2;
    double acc = 0.0;
    for (uint32_t q = blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += gridDim.x * blockDim.x) {
        const uint32_t j = q << 2;
        const Shared4 sh = grad_shared4(s, j);
        double squares[4] = {0.0, 0.0, 0.0, 0.0};
        const uint32_t workers = s.zeta != 0.0f ? n : 1u;      // identical optima: one term stands for all
        for (uint32_t i = 0; i < workers; ++i) {
            float shift[4] = {0.f, 0.f, 0.f, 0.f};
            if (s.zeta != 0.0f) draw_normal4(j >> 2, i, 0xfffffffeu, 0xffffffffu, s.seed_lo, s.seed_hi, shift);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float optimum = sh.opt[c];
                if (s.zeta != 0.0f) optimum = sh.opt[c] + s.zeta * shift[c];
                const double diff = (double)sh.x[c] - (double)optimum;
                squares[c] += diff * diff;
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (j + c < d) acc += (double)sh.lam[c] * (squares[c] / (double)workers);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane_id() == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// ------------------------------------------------------------------------------------
// S1 (+ candidate filter of S2/S3)   p = e + lr * g, written over e   (Algorithm 1, worker side)
//
// grid (ld/256, n), one wave per block: the wave owns 256 consecutive coordinates of worker
// blockIdx.y, one 16-byte access per lane and array.  (Single-wave blocks over a grid in
// address order stream markedly faster on this chip than persistent blocks striding over
// the row.)  While p is in registers, every entry whose magnitude pattern is >= bound[w] is
// a *candidate* for the top-k.  The wave counts its candidates with ballots, reserves that
// many slots with one atomic add and writes (index, value) pairs there in index order;
// tab[w][group] records (first slot, count), so that the runs can be read back in coordinate
// order although slots are handed out in arbitrary order.  To keep the atomics from
// serialising on one address, a worker's candidate buffer is split into kSubs equal parts
// with a counter each, and group number mod kSubs picks the part.
// With use_filter == 0 this is the plain accumulate pass.  With kFusedGrad the gradient is not
// read from g but generated in place (same arithmetic as k_grad), so it never touches HBM.
//
// Residual ahead of time: candidates whose magnitude pattern is >= zero_at[w] (the threshold
// this selection is expected to end at) are written to e as +0 right here, in the dense store
// that happens anyway, on the guess that they will be sent.  Their values live on in the
// candidate buffer; once the exact threshold is known, only the entries between the guess and
// the truth need a scattered store (k_chunk_emit), instead of all k sent ones.  A group that
// gets no slots keeps all its entries in e and records an empty run.
// ------------------------------------------------------------------------------------
//
// kSplit (dense messages, bound placed from a sample of this very p): the candidates fall into two
// classes.  Those at or above sure_at[w] -- a pattern as far above the expected threshold as the
// bound lies below it -- are *sure* to be sent: they are recorded as runs in a buffer of their own
// (sp.sure, run table sp.stab, slot counters sp.count) and never looked at again by the selection;
// the aggregation reads them straight from their runs.  Only the narrow *band* between bound[w] and
// sure_at[w] goes through the candidate buffer, the ordering, the radix select and the compaction,
// for the rank k minus the number of sure entries.  Should the guess be wrong (more sure entries
// than k, or fewer than k candidates in all), the worker falls back to its whole row as always.
template <bool kFusedGrad, bool kSplit>
__global__ __launch_bounds__(64) void k_ef_filter(float* __restrict__ e, const float* __restrict__ g,
                                                  GradSource src, uint32_t n,
                                                  uint64_t ld, uint32_t d, float lr,
                                                  const uint32_t* __restrict__ bound,
                                                  const uint32_t* __restrict__ zero_at, int use_filter,
                                                  uint2* __restrict__ cand, uint64_t cap,
                                                  uint32_t* __restrict__ cand_count,
                                                  uint32_t* __restrict__ overflow,
                                                  uint2* __restrict__ tab, uint32_t ngroups,
                                                  uint32_t* __restrict__ nonfinite, SureRuns sp) {
    // plain: grid (groups, n).  fused: 1-D grid with the worker index fastest, so that the blocks
    // that need the same lambda / x* / snapshot lines run at about the same time
    if (kFusedGrad) resolve_iteration(src);
    // fused: consecutive block numbers go to different XCDs (round robin over the 8 of them), and the
    // n blocks of one group read the same lambda / x* / snapshot lines: hand each XCD a contiguous
    // eighth of the logical blocks, so that those n blocks share one L2
    uint32_t bid = blockIdx.x;
    if (kFusedGrad) {
        const uint32_t per_xcd = gridDim.x >> 3;
        if (bid < (per_xcd << 3)) bid = (bid & 7u) * per_xcd + (bid >> 3);
    }
    const uint32_t w = kFusedGrad ? bid % n : blockIdx.y;
    const uint32_t grp = kFusedGrad ? bid / n : blockIdx.x;
    const uint32_t lane = threadIdx.x;
    const uint32_t j = grp * 256u + lane * 4u;
    float pv[4] = {0.f, 0.f, 0.f, 0.f};
    float* ep = e + (uint64_t)w * ld + j;
    if (j < d) {
        const float4 ev = load_stream4(ep);
        float gq[4];
        if (kFusedGrad) {
            grad_quad(src, grad_shared4(src, j), w, j, d, gq);
        } else {
            const float4 gv = load_stream4(g + (uint64_t)w * ld + j);
            gq[0] = gv.x; gq[1] = gv.y; gq[2] = gv.z; gq[3] = gv.w;
        }
        pv[0] = ev.x + lr * gq[0];
        pv[1] = ev.y + lr * gq[1];
        pv[2] = ev.z + lr * gq[2];
        pv[3] = ev.w + lr * gq[3];
    }
    if (note_nonfinite(pv) && lane == 0) nonfinite[w] = 1u;
    if (!use_filter) {
        if (j < d) store_stream4(ep, pv);
        return;
    }
    const uint32_t L = bound[w], H = zero_at[w];
    const uint32_t S = kSplit ? sp.sure_at[w] : 0xffffffffu;       // split: [L, S) is the band, [S, ..) is sure
    bool f[4], sure[4];
    bool any = false, any_sure = false;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint32_t key = mag_key(pv[c]);
        const bool in = j + c < d;
        f[c] = in && key >= L && key < S;
        sure[c] = kSplit && in && key >= S;
        any |= f[c];
        any_sure |= sure[c];
    }
    // the dense store goes out first, already with +0 at the candidates expected to be sent
    // (a group that then gets no slots stores its values once more, below)
    if (j < d) {
        float ov[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) ov[c] = ((f[c] || sure[c]) && mag_key(pv[c]) >= H) ? 0.0f : pv[c];
        store_stream4(ep, ov);
    }
    const uint32_t sub = grp & (kSubs - 1u);
    bool keep_all = false;                     // a class got no slots: the group's entries stay in e
    uint32_t first = 0, total = 0, sfirst = 0, stotal = 0;
    if (__ballot(any || any_sure)) {           // most groups of a sparse selection hold no candidate at all
        uint32_t below = 0, sbelow = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint64_t m = __ballot(f[c]);
            below += mask_rank(m);
            total += (uint32_t)__popcll(m);
            if (kSplit) {
                const uint64_t ms = __ballot(sure[c]);
                sbelow += mask_rank(ms);
                stotal += (uint32_t)__popcll(ms);
            }
        }
        // slots for both classes in one go: lane 0 reserves the band's, lane 1 the sure entries', so
        // that the two reservations are in flight together
        uint32_t got = 0;
        if (lane == 0 && total != 0u) got = atomicAdd(&cand_count[(w * kSubs + sub) * kSubStride], total);
        if (kSplit && lane == 1 && stotal != 0u) got = atomicAdd(&sp.count[(w * kSubs + sub) * kSubStride], stotal);
        const uint32_t got_band = __shfl(got, 0, 64);
        if (total != 0u) {
            const uint32_t sub_cap = (uint32_t)(cap / kSubs);
            if (got_band + total > sub_cap) {
                if (lane == 0) overflow[w] = 1u;
                total = 0;                     // nothing recorded for this group
                keep_all = true;
            } else {
                first = sub * sub_cap + got_band;
                uint2* cw = cand + (uint64_t)w * cap;
                uint32_t pos = first + below;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (f[c]) { cw[pos] = make_uint2(j + c, __float_as_uint(pv[c])); ++pos; }
            }
        }
        if (kSplit && stotal != 0u) {
            const uint32_t got_sure = __shfl(got, 1, 64);
            const uint32_t sub_cap = (uint32_t)(sp.cap / kSubs);
            if (got_sure + stotal > sub_cap) {
                if (lane == 0) overflow[w] = 1u;
                stotal = 0;
                keep_all = true;
            } else {
                sfirst = sub * sub_cap + got_sure;
                uint2* sw = sp.sure + (uint64_t)w * sp.cap;
                uint32_t pos = sfirst + sbelow;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (sure[c]) { sw[pos] = make_uint2(j + c, __float_as_uint(pv[c])); ++pos; }
            }
        }
    }
    if (lane == 0) {
        tab[(uint64_t)w * ngroups + grp] = make_uint2(first, total);
        if (kSplit) sp.stab[(uint64_t)w * ngroups + grp] = make_uint2(sfirst, stotal);
    }
    // (same lane, same address as the store above: the two stay in order.  The worker falls back to
    // its row, and the entries that were recorded are written back there with the same values.)
    if (keep_all && j < d) store_stream4(ep, pv);
}

#define DDEF_EF_FILTER_INSTANCE(fused, split)                                                                  \
    template __global__ void k_ef_filter<fused, split>(float*, const float*, GradSource, uint32_t, uint64_t, uint32_t, \
                                                       float, const uint32_t*, const uint32_t*, int, uint2*, uint64_t,  \
                                                       uint32_t*, uint32_t*, uint2*, uint32_t, uint32_t*, SureRuns);
DDEF_EF_FILTER_INSTANCE(false, false)
DDEF_EF_FILTER_INSTANCE(false, true)
DDEF_EF_FILTER_INSTANCE(true, false)
DDEF_EF_FILTER_INSTANCE(true, true)
#undef DDEF_EF_FILTER_INSTANCE

// ------------------------------------------------------------------------------------
// Random-k sparsifier (the paper's appendix on other sparsifiers): worker w keeps the k
// coordinates pi(0..k-1) of a keyed permutation pi of [0, d), drawn afresh for every
// (worker, iteration).  pi: 4-round Feistel network on 2w bits, round function = MurmurHash3's
// 32-bit finaliser of (half ^ round key) cut to w bits, cycle-walked into [0, d); round keys =
// the Philox block of counter (0xFFFFFFFF, worker, t), which no noise draw uses.
// k_randk_mark sets the chosen coordinates' bits in a bitmap; k_ef_randk is the accumulate
// pass that reads its 256 bits per group, sends the marked entries (same run mechanism as the
// Top-k candidates, but here the runs *are* the message) and writes the residual in one go.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t fmix32(uint32_t h) {
    h ^= h >> 16; h *= 0x85ebca6bu; h ^= h >> 13; h *= 0xc2b2ae35u; h ^= h >> 16;
    return h;
}

struct RandkPerm { uint32_t key[4]; uint32_t half, mask, d; };

__device__ __forceinline__ RandkPerm randk_perm(uint32_t w, uint32_t d, uint32_t seed_lo, uint32_t seed_hi,
                                                uint32_t t_lo, uint32_t t_hi) {
    RandkPerm p;
    const U4 rk = philox_block(0xffffffffu, w, t_lo, t_hi, seed_lo, seed_hi);
    p.key[0] = rk.a; p.key[1] = rk.b; p.key[2] = rk.c; p.key[3] = rk.d;
    p.half = 1;
    while (((uint64_t)1 << (2u * p.half)) < (uint64_t)d) ++p.half;
    p.mask = (uint32_t)(((uint64_t)1 << p.half) - 1u);
    p.d = d;
    return p;
}

// one pass through the four Feistel rounds (a bijection of [0, 4^half))
__device__ __forceinline__ uint64_t randk_rounds(const RandkPerm& p, uint64_t y) {
    uint32_t left = (uint32_t)(y >> p.half), right = (uint32_t)y & p.mask;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint32_t nr = left ^ (fmix32(right ^ p.key[r]) & p.mask);
        left = right;
        right = nr;
    }
    return ((uint64_t)left << p.half) | right;
}

__device__ __forceinline__ uint32_t randk_image(const RandkPerm& p, uint64_t m) {
    uint64_t y = m;
    do y = randk_rounds(p, y); while (y >= (uint64_t)p.d);   // walk until the image falls inside [0, d)
    return (uint32_t)y;
}

__global__ __launch_bounds__(256) void k_randk_mark(uint32_t* __restrict__ bitmap, uint64_t bitmap_ld,
                                                    uint32_t d, uint32_t k, uint32_t seed_lo,
                                                    uint32_t seed_hi, uint32_t t_lo, uint32_t t_hi,
                                                    const SelState* __restrict__ gate) {
    const uint32_t w = blockIdx.y;
    if (gate != nullptr && gate[w].active != 3u) return;       // a repeat pass: only the workers that ask for it
    const RandkPerm perm = randk_perm(w, d, seed_lo, seed_hi, t_lo, t_hi);
    uint32_t* row = bitmap + (uint64_t)w * bitmap_ld;
    for (uint32_t m = blockIdx.x * blockDim.x + threadIdx.x; m < k; m += gridDim.x * blockDim.x) {
        const uint32_t y = randk_image(perm, m);
        atomicOr(&row[y >> 5], 1u << (y & 31u));
    }
}

// Marking many coordinates (k a sizeable share of d) bit by bit costs one memory-side atomic on
// a random line per coordinate.  Instead the images are first sorted coarsely: the coordinate
// range is cut into `regions` regions of 2^region_bits coordinates, and each image is appended to
// its region's bucket (bucket_cap entries; gcount[w][region] counts them).  A block takes 8192
// values of m, counts its images per region in LDS, reserves a run in every bucket it needs
// with one atomic per region, and writes the images there.  An image that finds its bucket full
// is set in the bitmap directly.  k_randk_fill then sets a region's bits in LDS and writes the
// words out.  grid (blocks, n), 1024 threads; regions <= 2048.
__global__ __launch_bounds__(1024) void k_randk_bin(uint32_t* __restrict__ bucket, uint64_t bucket_ld,
                                                    uint32_t bucket_cap, uint32_t* __restrict__ gcount,
                                                    uint32_t region_bits, uint32_t regions,
                                                    uint32_t* __restrict__ bitmap, uint64_t bitmap_ld,
                                                    uint32_t d, uint32_t k, uint32_t seed_lo,
                                                    uint32_t seed_hi, uint32_t t_lo, uint32_t t_hi,
                                                    const SelState* __restrict__ gate) {
    __shared__ uint32_t cnt[2048];
    __shared__ uint32_t base[2048];
    __shared__ uint32_t images[8192];         // images[i * 1024 + thread]: the thread's i-th image
    const uint32_t w = blockIdx.y;
    if (gate != nullptr && gate[w].active != 3u) return;
    const RandkPerm perm = randk_perm(w, d, seed_lo, seed_hi, t_lo, t_hi);
    uint32_t* mine = bucket + (uint64_t)w * bucket_ld;
    const uint32_t chunks = (uint32_t)(((uint64_t)k + 8191u) >> 13);
    for (uint32_t chunk = blockIdx.x; chunk < chunks; chunk += gridDim.x) {
        for (uint32_t r = threadIdx.x; r < regions; r += blockDim.x) cnt[r] = 0u;
        __syncthreads();
        // The walk into [0, d) takes a different number of passes for every m (about 4^half / d
        // on average).  Walking one m after the other, a wave would wait for its slowest lane
        // eight times over; instead every lane walks through its eight values back to back and
        // the wave ends when the lane with the most passes in total is done.
        const uint64_t m0 = ((uint64_t)chunk << 13) + threadIdx.x;
        uint32_t items = 0;
        if (m0 < (uint64_t)k) {
            const uint64_t room = ((uint64_t)k - m0 + 1023u) >> 10;
            items = room < 8u ? (uint32_t)room : 8u;
        }
        uint32_t cur = 0;
        uint64_t val = m0;
        while (__any(cur < items)) {
            if (cur < items) {
                val = randk_rounds(perm, val);
                if (val < (uint64_t)d) {
                    images[cur * 1024u + threadIdx.x] = (uint32_t)val;
                    ++cur;
                    val = m0 + (uint64_t)cur * 1024u;
                }
            }
        }
        uint32_t y[8], rank[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            y[i] = 0u; rank[i] = 0u;
            if ((uint32_t)i < items) {
                y[i] = images[(uint32_t)i * 1024u + threadIdx.x];
                rank[i] = atomicAdd(&cnt[y[i] >> region_bits], 1u);
            }
        }
        __syncthreads();
        for (uint32_t r = threadIdx.x; r < regions; r += blockDim.x) {
            const uint32_t c = cnt[r];
            base[r] = c ? atomicAdd(&gcount[(uint64_t)w * regions + r], c) : 0u;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if ((uint32_t)i < items) {
                const uint32_t r = y[i] >> region_bits;
                const uint64_t pos = (uint64_t)base[r] + rank[i];
                if (pos < (uint64_t)bucket_cap) mine[(uint64_t)r * bucket_cap + pos] = y[i];
                else atomicOr(&bitmap[(uint64_t)w * bitmap_ld + (y[i] >> 5)], 1u << (y[i] & 31u));
            }
        }
        __syncthreads();
    }
}

// grid (regions, n), 1024 threads: sets the region's bits tile by tile (2^18 coordinates, 32 KB of
// LDS) from its bucket and ORs the words into the bitmap (no other block touches these words);
// leaves gcount at zero for the next iteration.
__global__ __launch_bounds__(1024) void k_randk_fill(const uint32_t* __restrict__ bucket, uint64_t bucket_ld,
                                                     uint32_t bucket_cap, uint32_t* __restrict__ gcount,
                                                     uint32_t region_bits, uint32_t regions,
                                                     uint32_t* __restrict__ bitmap, uint64_t bitmap_ld,
                                                     uint32_t d, const SelState* __restrict__ gate) {
    __shared__ uint32_t bits[8192];
    const uint32_t w = blockIdx.y, r = blockIdx.x;
    if (gate != nullptr && gate[w].active != 3u) return;
    uint32_t count = gcount[(uint64_t)w * regions + r];
    if (count > bucket_cap) count = bucket_cap;
    __syncthreads();
    if (threadIdx.x == 0) gcount[(uint64_t)w * regions + r] = 0u;
    if (count == 0u) return;
    const uint32_t* mine = bucket + (uint64_t)w * bucket_ld + (uint64_t)r * bucket_cap;
    uint32_t* row = bitmap + (uint64_t)w * bitmap_ld;
    const uint32_t tiles = 1u << (region_bits - 18u);
    for (uint32_t s = 0; s < tiles; ++s) {
        const uint64_t tile_first = ((uint64_t)r << region_bits) + ((uint64_t)s << 18);
        if (tile_first >= (uint64_t)d) break;
        const uint32_t tile_id = (uint32_t)(tile_first >> 18);
        for (uint32_t q = threadIdx.x; q < 8192u; q += blockDim.x) bits[q] = 0u;
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < count; i += blockDim.x) {
            const uint32_t y = mine[i];
            if ((y >> 18) == tile_id) atomicOr(&bits[(y & 0x3ffffu) >> 5], 1u << (y & 31u));
        }
        __syncthreads();
        const uint64_t word0 = tile_first >> 5;
        for (uint32_t q = threadIdx.x; q < 8192u; q += blockDim.x) {
            const uint32_t v = bits[q];
            if (v != 0u && word0 + q < bitmap_ld) row[word0 + q] |= v;
        }
        __syncthreads();
    }
}

// grid (ld/256, n), one wave per block, as k_ef_filter.  Eight lanes share one bitmap word;
// the first of them clears it after the group has read it, so the bitmap is all-zero again
// when the pass is over.  zero_marked = 0 leaves the marked entries' values in e (the composed
// compressor decides later which of them are sent).  With `bound` non-null only the marked entries
// whose magnitude pattern is >= bound[w] are recorded (the composed compressor needs the largest of
// the marked entries, not all of them).  accumulate = 0 takes p = e as it stands (a second pass
// over a row that already holds e + lr*g) and stores nothing.
__global__ __launch_bounds__(64) void k_ef_randk(float* __restrict__ e, const float* __restrict__ g,
                                                 uint64_t ld, uint32_t d, float lr, int zero_marked,
                                                 int accumulate, const uint32_t* __restrict__ bound,
                                                 uint32_t* __restrict__ bitmap, uint64_t bitmap_ld,
                                                 uint2* __restrict__ cand, uint64_t cap,
                                                 uint32_t* __restrict__ cand_count,
                                                 uint32_t* __restrict__ overflow,
                                                 uint2* __restrict__ tab, uint32_t ngroups,
                                                 uint32_t* __restrict__ nonfinite,
                                                 const SelState* __restrict__ gate) {
    const uint32_t w = blockIdx.y, lane = threadIdx.x;
    if (gate != nullptr && gate[w].active != 3u) return;     // a repeat pass: only the workers that ask for it
    // (one group per block in the main pass; a repeat pass is launched with fewer blocks, which stride)
    for (uint32_t grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
    const uint32_t j = grp * 256u + lane * 4u;
    uint32_t* word = bitmap + (uint64_t)w * bitmap_ld + (j >> 5);
    const uint32_t bitsel = (*word >> (j & 31u)) & 0xfu;     // this lane's four coordinates
    float pv[4] = {0.f, 0.f, 0.f, 0.f};
    if (j < d) {
        float* ep = e + (uint64_t)w * ld + j;
        const float4 ev = load_stream4(ep);
        if (accumulate) {
            const float4 gv = load_stream4(g + (uint64_t)w * ld + j);
            pv[0] = ev.x + lr * gv.x;
            pv[1] = ev.y + lr * gv.y;
            pv[2] = ev.z + lr * gv.z;
            pv[3] = ev.w + lr * gv.w;
            float res[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) res[c] = (zero_marked && ((bitsel >> c) & 1u)) ? 0.0f : pv[c];
            store_stream4(ep, res);
        } else {
            pv[0] = ev.x; pv[1] = ev.y; pv[2] = ev.z; pv[3] = ev.w;
        }
    }
    if (note_nonfinite(pv) && lane == 0) nonfinite[w] = 1u;
    const uint32_t L = bound ? bound[w] : 0u;
    if (__ballot(bitsel != 0u) && (lane & 7u) == 0u) *word = 0u;   // every lane of the group has read it
    bool f[4];
    uint32_t first = 0, total = 0, below = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        f[c] = ((bitsel >> c) & 1u) && mag_key(pv[c]) >= L;
        const uint64_t m = __ballot(f[c]);
        below += mask_rank(m);
        total += (uint32_t)__popcll(m);
    }
    if (total != 0u) {                                       // wave-uniform
        const uint32_t sub = grp & (kSubs - 1u);
        const uint32_t sub_cap = (uint32_t)(cap / kSubs);
        uint32_t got = 0;
        if (lane == 0) got = atomicAdd(&cand_count[(w * kSubs + sub) * kSubStride], total);
        got = __shfl(got, 0, 64);
        if (got + total > sub_cap) {
            if (lane == 0) overflow[w] = 1u;
            total = 0;
        } else {
            first = sub * sub_cap + got;
            uint2* cw = cand + (uint64_t)w * cap;
            uint32_t pos = first + below;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (f[c]) { cw[pos] = make_uint2(j + c, __float_as_uint(pv[c])); ++pos; }
        }
    }
    if (lane == 0) tab[(uint64_t)w * ngroups + grp] = make_uint2(first, total);
    }
}

// One block per worker: span sums -> span offsets; the runs must hold exactly k entries.
// sel[w].active = 0 lets k_tab_order copy the runs; 2 flags a broken invariant (slot overflow).
__global__ __launch_bounds__(256) void k_tab_decide_randk(uint32_t* __restrict__ span_sum, uint32_t nspans,
                                                          uint32_t* __restrict__ overflow, uint32_t k,
                                                          SelState* __restrict__ sel,
                                                          uint32_t* __restrict__ cand_total,
                                                          uint32_t* __restrict__ cand_count) {
    __shared__ uint32_t lds[5];
    const uint32_t w = blockIdx.x;
    uint32_t* sw = span_sum + (uint64_t)w * nspans;
    uint32_t carry = 0;
    for (uint32_t first = 0; first < nspans; first += 256u) {
        const uint32_t sp = first + threadIdx.x;
        const uint32_t v = sp < nspans ? sw[sp] : 0u;
        uint32_t total;
        const uint32_t at = carry + block_excl_scan(v, lds, &total);
        if (sp < nspans) sw[sp] = at;
        carry += total;
    }
    if (threadIdx.x == 0) {
        const bool fine = overflow[w] == 0u && carry == k;
        cand_total[w] = carry;
        sel[w].active = fine ? 0u : 2u;
        sel[w].T = 0u; sel[w].r = 0u; sel[w].seen = carry;
        overflow[w] = 0u;
    }
    for (uint32_t q = threadIdx.x; q < kSubs; q += blockDim.x) cand_count[(w * kSubs + q) * kSubStride] = 0u;
}

// ---- run table -> coordinate order ------------------------------------------------------
// tab[w][c].y is the run length of group c.  Three small kernels turn the lengths into
// positions in coordinate order: sums over spans of 1024 groups, a scan of the span sums that
// also decides whether the filter caught enough, and the prefixes inside a span, which drive
// the copy of the runs into coordinate order.
__global__ __launch_bounds__(1024) void k_tab_sum(const uint2* __restrict__ tab, uint32_t ngroups,
                                                  uint32_t* __restrict__ span_sum, uint32_t nspans,
                                                  const SelState* __restrict__ gate) {
    __shared__ uint32_t red[16];
    const uint32_t w = blockIdx.y, sp = blockIdx.x;
    if (gate != nullptr && gate[w].active != 3u) return;       // (the other workers' sums are offsets by now)
    const uint32_t c = sp * kSpan + threadIdx.x;
    uint32_t mine = c < ngroups ? tab[(uint64_t)w * ngroups + c].y : 0u;
    mine = wave_sum(mine);
    if (lane_id() == 0) red[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int q = 0; q < 16; ++q) t += red[q];
        span_sum[(uint64_t)w * nspans + sp] = t;
    }
}

// Start of a worker's selection (any thread count): rank 0 looks for the k-th entry of the
// view, rank 1 for the kb-th (or the last one if the view is shorter); clears the worker's
// digit histograms of all three levels.
__device__ __forceinline__ void begin_selection(SelState* sel, uint32_t w, uint32_t n, uint32_t k,
                                                uint32_t kb, uint32_t view_len, uint32_t* hist) {
    if (threadIdx.x == 0) {
        sel[w].prefix[0] = 0; sel[w].prefix[1] = 0;
        sel[w].krem[0] = k;
        sel[w].krem[1] = kb < view_len ? kb : view_len;
    }
    for (int level = 0; level < 3; ++level) {
        uint32_t* h = hist + ((uint64_t)level * n + w) * 2u * 2048u;
        for (uint32_t b = threadIdx.x; b < 4096u; b += blockDim.x) h[b] = 0u;
    }
}

// One block per worker.  The filter is usable when nothing overflowed and it caught at
// least k entries: then the top-k is among the candidates, because every entry outside the
// candidate set is smaller than every entry inside.  Otherwise sel[w].active = 1 sends the
// worker's selection over its whole row.
// With the sure / band split (sure_count non-null: the worker's kSubs slot counters of the sure
// buffer, cleared here) the candidates are the band only: usable when nothing overflowed, fewer
// than k entries are sure (S < k) and sure plus band hold at least k; the selection then looks for
// rank k - S inside the band.  sure_total[w] = S (0 when the worker falls back), msg_count[w] =
// how many entries the compaction will write to the worker's message row (k - S, or k).
__global__ __launch_bounds__(256) void k_tab_decide(uint32_t* __restrict__ span_sum, uint32_t nspans,
                                                    const uint32_t* __restrict__ overflow, uint32_t k,
                                                    uint32_t kb, uint32_t d, uint32_t n,
                                                    SelState* __restrict__ sel,
                                                    uint32_t* __restrict__ cand_total,
                                                    uint32_t* __restrict__ stat_full,
                                                    const uint32_t* __restrict__ zero_at,
                                                    uint32_t* __restrict__ hist,
                                                    uint32_t* __restrict__ sure_count,
                                                    uint32_t* __restrict__ sure_total,
                                                    uint32_t* __restrict__ msg_count) {
    __shared__ uint32_t lds[5];
    const uint32_t w = blockIdx.x;
    uint32_t* sw = span_sum + (uint64_t)w * nspans;
    uint32_t carry = 0;
    for (uint32_t first = 0; first < nspans; first += 256u) {       // span sums -> span offsets
        const uint32_t sp = first + threadIdx.x;
        const uint32_t v = sp < nspans ? sw[sp] : 0u;
        uint32_t total;
        const uint32_t at = carry + block_excl_scan(v, lds, &total);
        if (sp < nspans) sw[sp] = at;
        carry += total;
    }
    const uint32_t M = carry;
    uint32_t S = 0;
    const bool split = sure_count != nullptr;
    if (split) {                                 // blockDim.x == kSubs: one slot counter per thread
        uint32_t* mine = &sure_count[(w * kSubs + threadIdx.x) * kSubStride];
        const uint32_t v = *mine;
        *mine = 0u;
        (void)block_excl_scan(v, lds, &S);
    }
    const bool usable = overflow[w] == 0u && (split ? (S < k && M >= k - S) : M >= k);
    const uint32_t rank = usable ? k - S : k;
    if (threadIdx.x == 0) {
        cand_total[w] = M;
        sel[w].active = usable ? 0u : 1u;
        sel[w].zero_used = zero_at[w];          // what the accumulate pass zeroed ahead of time
        if (!usable) stat_full[w] += 1u;
        if (sure_total) sure_total[w] = (split && usable) ? S : 0u;
        if (msg_count) msg_count[w] = rank;
    }
    begin_selection(sel, w, n, rank, (split && usable) ? rank : kb, usable ? M : d, hist);
}

// A worker that falls back to its whole row although sure entries were recorded (and written to e
// as +0 ahead of time) gets them back: one thread per 256-coordinate group walks the group's run.
// grid (ceil(ngroups / 256), n); nothing to do for workers whose selection uses the candidates.
__global__ __launch_bounds__(256) void k_restore_sure(const SelState* __restrict__ sel, SureRuns sp,
                                                      uint32_t ngroups, float* __restrict__ e, uint64_t ld) {
    const uint32_t w = blockIdx.y;
    if (sel[w].active != 1u) return;
    const uint32_t grp = blockIdx.x * blockDim.x + threadIdx.x;
    if (grp >= ngroups) return;
    const uint2 run = sp.stab[(uint64_t)w * ngroups + grp];
    const uint2* sw = sp.sure + (uint64_t)w * sp.cap;
    float* row = e + (uint64_t)w * ld;
    for (uint32_t q = 0; q < run.y; ++q) {
        const uint2 item = sw[run.x + q];
        row[item.x] = __uint_as_float(item.y);
    }
}

// No filter in this iteration: every worker searches its whole row.
__global__ __launch_bounds__(256) void k_sel_begin_rows(SelState* __restrict__ sel, uint32_t n, uint32_t k,
                                                        uint32_t kb, uint32_t d,
                                                        uint32_t* __restrict__ cand_total,
                                                        uint32_t* __restrict__ hist) {
    const uint32_t w = blockIdx.x;
    if (threadIdx.x == 0) { sel[w].active = 1u; sel[w].zero_used = 0xffffffffu; cand_total[w] = 0u; }
    begin_selection(sel, w, n, k, kb, d, hist);
}

// ---- composed compressor: Random-k, Top-k inside the kept coordinates, 4-bit codes ---------
// (Section 5.2 "Baselines": the strongest static baseline's compressor.)  The Random-k pass above
// records the k1 kept entries as runs and leaves e = p; the radix select of S2/S3 then runs on
// those entries in coordinate order for rank k, as it does on a filter's candidates, and the
// message it writes is coded below.
//
// One block per worker, after k_tab_sum: span sums -> span offsets, then the selection of the k
// largest recorded entries starts.  exact = 1: every kept coordinate was recorded, the runs must
// hold exactly k1 entries (active = 2 flags a slot overflow).  exact = 0: only the kept entries
// above a bound were recorded, which is enough when there are at least k of them; otherwise
// active = 3 marks the worker for the repeat pass (recording every kept entry, no bound), whose
// kernels are enqueued every time and run only for such workers (gated = 1: this kernel, too, then
// looks at those workers only and leaves the others' verdict alone).  Leaves the slot counters
// and the overflow flag cleared.
__global__ __launch_bounds__(256) void k_tab_decide_composed(uint32_t* __restrict__ span_sum, uint32_t nspans,
                                                             uint32_t* __restrict__ overflow, uint32_t k1,
                                                             uint32_t k, uint32_t n, int exact,
                                                             SelState* __restrict__ sel,
                                                             uint32_t* __restrict__ cand_total,
                                                             uint32_t* __restrict__ cand_count,
                                                             uint32_t* __restrict__ hist,
                                                             uint32_t* __restrict__ stat_repeat, int gated) {
    __shared__ uint32_t lds[5];
    const uint32_t w = blockIdx.x;
    if (gated && sel[w].active != 3u) return;   // a repeat pass: the worker's first verdict stands
    uint32_t* sw = span_sum + (uint64_t)w * nspans;
    uint32_t carry = 0;
    for (uint32_t first = 0; first < nspans; first += 256u) {
        const uint32_t sp = first + threadIdx.x;
        const uint32_t v = sp < nspans ? sw[sp] : 0u;
        uint32_t total;
        const uint32_t at = carry + block_excl_scan(v, lds, &total);
        if (sp < nspans) sw[sp] = at;
        carry += total;
    }
    const bool fine = overflow[w] == 0u && (exact ? carry == k1 : carry >= k);
    __syncthreads();                            // every thread has read the flag
    if (threadIdx.x == 0) {
        cand_total[w] = fine ? carry : 0u;
        if (!fine && !exact) stat_repeat[w] += 1u;          // the pass is repeated without the bound for this worker
        sel[w].active = fine ? 0u : (exact ? 2u : 3u);
        sel[w].zero_used = 0xffffffffu;         // nothing was cleared ahead of time
        sel[w].seen = carry;
        overflow[w] = 0u;
    }
    for (uint32_t q = threadIdx.x; q < kSubs; q += blockDim.x) cand_count[(w * kSubs + q) * kSubStride] = 0u;
    begin_selection(sel, w, n, k, k, fine ? carry : 0u, hist);
}

// 4-bit stage: the message (values in coordinate order) is cut into blocks of 256 entries, one
// thread block each.  step = (largest magnitude of the block) / 7; code = value / step rounded to
// the nearest integer (halves to even) inside [-7, 7]; the message value becomes what the
// receiver decodes, code * step, and the coding error goes back into e at the entry's coordinate
// (k_chunk_emit, run with fix_e = 0, left p there).  A block whose step is zero sends zero codes.  Two codes per
// byte, even position in the low nibble, two's complement.  grid (ceil(k / 256), n).
__global__ __launch_bounds__(256) void k_quantize4(const uint32_t* __restrict__ msg_idx,
                                                   float* __restrict__ msg_val, uint64_t msg_ld, uint32_t k,
                                                   const SelState* __restrict__ sel,
                                                   float* __restrict__ e, uint64_t ld,
                                                   uint8_t* __restrict__ codes, uint64_t codes_ld,
                                                   float* __restrict__ steps, uint64_t steps_ld) {
    __shared__ float red[4];
    const uint32_t w = blockIdx.y, b = blockIdx.x;
    if (sel[w].active == 2u) return;            // broken invariant: the host reports it, nothing is coded
    const uint32_t m = b * 256u + threadIdx.x;
    const bool in = m < k;
    const float v = in ? msg_val[(uint64_t)w * msg_ld + m] : 0.0f;
    float big = fabsf(v);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) big = fmaxf(big, __shfl_xor(big, off, 64));
    if (lane_id() == 0) red[threadIdx.x >> 6] = big;
    __syncthreads();
    big = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float step = big / 7.0f;
    int q = 0;
    if (step > 0.0f) {
        float nearest = rintf(v / step);
        nearest = fminf(fmaxf(nearest, -7.0f), 7.0f);
        q = (int)nearest;
    }
    const float deq = (float)q * step;
    const uint32_t nib = (uint32_t)q & 0xfu;
    const uint32_t next_nib = (uint32_t)__shfl_down((int)nib, 1, 64);   // pairs (even, odd) never straddle a wave
    if (in) {
        msg_val[(uint64_t)w * msg_ld + m] = deq;
        e[(uint64_t)w * ld + msg_idx[(uint64_t)w * msg_ld + m]] = v - deq;
        if ((threadIdx.x & 1u) == 0u) codes[(uint64_t)w * codes_ld + (m >> 1)] = (uint8_t)(nib | (next_nib << 4));
    }
    if (threadIdx.x == 0) steps[(uint64_t)w * steps_ld + b] = step;
}

// Prefixes inside a span, and with them the candidates in coordinate order: group c's run
// cand[first .. first+len) goes to positions [at, at+len) of the ordered arrays (index,
// value; rows of out_ld entries).  The block copies its span's candidates together: thread q takes the q-th, finds
// its group by bisection over the span's prefixes in LDS, and the stores are coalesced.
// A worker whose selection falls back to its whole row (active == 1) gets its row completed
// instead: the recorded candidates that the accumulate pass had zeroed ahead of time are
// written back to e (e_row non-null; rows of e_ld floats).
__global__ __launch_bounds__(1024) void k_tab_order(const uint2* __restrict__ tab, uint32_t ngroups,
                                                    const uint32_t* __restrict__ span_off,
                                                    uint32_t nspans, const SelState* __restrict__ sel,
                                                    const uint2* __restrict__ cand, uint64_t cap,
                                                    uint32_t* __restrict__ sorted_idx,
                                                    float* __restrict__ sorted_val, uint64_t out_ld,
                                                    float* __restrict__ e_row, uint64_t e_ld) {
    __shared__ uint32_t lds[17];
    __shared__ uint32_t at_of[kSpan];        // exclusive prefix of the run lengths inside the span
    __shared__ uint32_t first_of[kSpan];     // first slot of each run
    const uint32_t w = blockIdx.y, sp = blockIdx.x;
    const uint32_t mode = sel[w].active;
    const bool restore = mode == 1u && e_row != nullptr;
    if (mode != 0u && !restore) return;
    const uint32_t zero_used = sel[w].zero_used;
    const uint32_t c = sp * kSpan + threadIdx.x;
    const uint2 run = c < ngroups ? tab[(uint64_t)w * ngroups + c] : make_uint2(0u, 0u);
    uint32_t total;
    const uint32_t at = block_excl_scan(run.y, lds, &total);
    at_of[threadIdx.x] = at;
    first_of[threadIdx.x] = run.x;
    __syncthreads();
    if (total == 0u) return;
    const uint2* cw = cand + (uint64_t)w * cap;
    const uint64_t out0 = (uint64_t)w * out_ld + span_off[(uint64_t)w * nspans + sp];
    for (uint32_t q = threadIdx.x; q < total; q += kSpan) {
        uint32_t lo = 0, hi = kSpan;           // first group in [lo, hi) whose prefix exceeds q
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (at_of[mid] > q) hi = mid; else lo = mid + 1u;
        }
        const uint32_t grp = lo - 1u;           // at_of[0] = 0 <= q, so lo >= 1; empty runs are skipped
        const uint2 item = cw[first_of[grp] + (q - at_of[grp])];
        if (restore) {
            if ((item.y & 0x7fffffffu) >= zero_used) e_row[(uint64_t)w * e_ld + item.x] = __uint_as_float(item.y);
        } else {
            sorted_idx[out0 + q] = item.x;
            sorted_val[out0 + q] = __uint_as_float(item.y);
        }
    }
}

// ------------------------------------------------------------------------------------
// S2  radix select of the k-th entry under (|v| descending, index ascending), done on the
// 31-bit magnitude pattern in three digits of 11, 10 and 10 bits, for two ranks at once:
// rank 0 is k (gives the threshold T and r), rank 1 is the candidate target used to place
// the next iteration's filter bound.  Each worker is searched through its *view*: its
// ordered candidates (active == 0) or its whole row of e (active == 1).
// ------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lvl_lo(int level) { return level == 0 ? 20u : level == 1 ? 10u : 0u; }
__device__ __forceinline__ uint32_t lvl_hi(int level) { return level == 0 ? 31u : level == 1 ? 20u : 10u; }
__device__ __forceinline__ uint32_t lvl_bins(int level) { return level == 0 ? 2048u : 1024u; }

struct View { const float* row; const uint32_t* map; uint32_t count; };

__device__ __forceinline__ View view_of(const SelViews& vs, const SelState* sel, uint32_t w) {
    View v;
    if (sel[w].active) { v.row = vs.e + (uint64_t)w * vs.ld; v.map = nullptr; v.count = vs.d; }
    else {
        v.row = vs.cand_val + (uint64_t)w * vs.cap;
        v.map = vs.cand_idx + (uint64_t)w * vs.cap;
        v.count = vs.cand_total[w];
    }
    return v;
}

// One count per lane with `on` into an LDS histogram.  The entries of a candidate view are
// close in magnitude, so on the upper digits nearly every lane of a wave names the same bin,
// and LDS atomics on one address are served one after another: the lanes that share the
// first active lane's bin are counted with a ballot and added once; the rest add singly.
// All lanes of the wave must call this together.
__device__ __forceinline__ void hist_add(uint32_t* h, uint32_t digit, bool on) {
    const uint64_t todo = __ballot(on);
    if (todo == 0ull) return;
    const uint32_t leader = (uint32_t)__builtin_ctzll(todo);
    const uint32_t lead_digit = (uint32_t)__builtin_amdgcn_readlane((int)digit, (int)leader);
    const uint64_t same = __ballot(on && digit == lead_digit);
    if (lane_id() == leader) atomicAdd(&h[lead_digit], (uint32_t)__popcll(same));
    if (on && digit != lead_digit) atomicAdd(&h[digit], 1u);
}

// Histogram of one digit over each worker's view.  Level 0 builds one histogram shared by
// both ranks; levels 1, 2 build one per rank, over the entries whose higher bits match that
// rank's prefix.  hist layout: [worker][2][2048].
__global__ __launch_bounds__(256) void k_digit_hist(SelViews vs, const SelState* __restrict__ sel,
                                                    uint32_t* __restrict__ hist, int level) {
    __shared__ uint32_t h[2][2048];
    const uint32_t w = blockIdx.y;
    const View v = view_of(vs, sel, w);
    const uint32_t quads = (v.count + 3u) >> 2;
    if (blockIdx.x * blockDim.x >= quads) return;         // nothing for this block (uniform)
    const uint32_t lo = lvl_lo(level), hi = lvl_hi(level), bins = lvl_bins(level);
    const int nrank = level == 0 ? 1 : 2;
    for (uint32_t b = threadIdx.x; b < 2048u; b += blockDim.x) { h[0][b] = 0; h[1][b] = 0; }
    __syncthreads();
    const uint32_t pre0 = sel[w].prefix[0] >> hi, pre1 = sel[w].prefix[1] >> hi;
    for (uint32_t q = blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += gridDim.x * blockDim.x) {
        const float4 x = reinterpret_cast<const float4*>(v.row)[q];
        const float vv[4] = {x.x, x.y, x.z, x.w};
        const uint32_t j = q << 2;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool in = j + c < v.count;
            const uint32_t key = mag_key(vv[c]);
            const uint32_t digit = (key >> lo) & (bins - 1u);
            if (level == 0) {
                hist_add(h[0], digit, in);
            } else {
                hist_add(h[0], digit, in && (key >> hi) == pre0);
                hist_add(h[1], digit, in && (key >> hi) == pre1);
            }
        }
    }
    __syncthreads();
    uint32_t* out = hist + (uint64_t)w * 2u * 2048u;
    for (int r = 0; r < nrank; ++r)
        for (uint32_t b = threadIdx.x; b < bins; b += blockDim.x) {
            const uint32_t c = h[r][b];
            if (c) atomicAdd(&out[r * 2048u + b], c);
        }
}

// Pick the digit holding each rank: grid (n, 2), block 256.  For rank `rk`, walks the
// histogram from the top digit down until the running count reaches krem[rk]; appends the
// digit to prefix[rk] and reduces krem[rk] by the count of the digits above it.  After the
// last level publishes T, r (rank 0) and the magnitude at the filter rank (rank 1).
__global__ __launch_bounds__(256) void k_digit_pick(SelState* __restrict__ sel,
                                                    const uint32_t* __restrict__ hist, int level) {
    __shared__ uint32_t lds[8];
    __shared__ uint32_t found_digit, found_above;
    const uint32_t w = blockIdx.x, rk = blockIdx.y;
    const uint32_t bins = lvl_bins(level), lo = lvl_lo(level);
    const uint32_t per = bins / 256u;
    // level 0 has a single histogram (slot 0) read by both ranks
    const uint32_t* hsrc = hist + (uint64_t)w * 2u * 2048u + (level == 0 ? 0u : rk * 2048u);
    const uint32_t krem = sel[w].krem[rk];
    if (threadIdx.x == 0) { found_digit = 0; found_above = 0; }
    // thread 0 owns the top `per` digits
    const uint32_t top = bins - threadIdx.x * per;      // exclusive upper digit of this thread
    uint32_t mine = 0;
    for (uint32_t q = 0; q < per; ++q) mine += hsrc[top - 1u - q];
    uint32_t total;
    const uint32_t above = block_excl_scan(mine, lds, &total);
    if (above < krem && krem <= above + mine) {
        uint32_t run = above;
        for (uint32_t q = 0; q < per; ++q) {
            const uint32_t c = hsrc[top - 1u - q];
            if (krem <= run + c) { found_digit = top - 1u - q; found_above = run; break; }
            run += c;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t pre = sel[w].prefix[rk] | (found_digit << lo);
        const uint32_t rem = krem - found_above;
        sel[w].prefix[rk] = pre;
        sel[w].krem[rk] = rem;
        if (level == 2) {
            if (rk == 0) { sel[w].T = pre; sel[w].r = rem; }
            else sel[w].next_bound = pre;
        }
    }
}

// ------------------------------------------------------------------------------------
// S3  ordered compaction of a view, given (T, r): count per 4096-entry chunk, scan over
// chunks, emit.  An entry is sent iff key > T, or key == T and fewer than r entries with
// key == T precede it in coordinate order.  Count arrays are laid out [worker][stride].
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_chunk_count(SelViews vs, const SelState* __restrict__ sel,
                                                     uint32_t* __restrict__ cnt_gt,
                                                     uint32_t* __restrict__ cnt_eq, uint32_t stride) {
    __shared__ uint32_t red[8];
    const uint32_t w = blockIdx.y;
    const View v = view_of(vs, sel, w);
    const uint32_t nchunks = (v.count + 4095u) >> 12;
    const uint32_t T = sel[w].T;
    for (uint32_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
        uint32_t gt = 0, eq = 0;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint32_t j = c * 4096u + s * 1024u + threadIdx.x * 4u;
            if (j < v.count) {
                const float4 x = *reinterpret_cast<const float4*>(v.row + j);
                const float vv[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                for (int m = 0; m < 4; ++m)
                    if (j + m < v.count) {
                        const uint32_t key = mag_key(vv[m]);
                        gt += key > T;
                        eq += key == T;
                    }
            }
        }
        const uint32_t wave_gt = wave_sum(gt), wave_eq = wave_sum(eq);
        if (lane_id() == 0) { red[threadIdx.x >> 6] = wave_gt; red[4 + (threadIdx.x >> 6)] = wave_eq; }
        __syncthreads();
        if (threadIdx.x == 0) {
            cnt_gt[(uint64_t)w * stride + c] = red[0] + red[1] + red[2] + red[3];
            cnt_eq[(uint64_t)w * stride + c] = red[4] + red[5] + red[6] + red[7];
        }
        __syncthreads();
    }
}

// Filter bound for the next iteration (one thread per worker, called from k_chunk_scan).  After a whole-row search the bound starts from the exact
// magnitude of rank kb.  After a candidate search it starts from the magnitude of rank
// min(kb, M) among the M candidates; when fewer than kb were caught it is lowered further,
// assuming the count keeps growing towards smaller magnitudes at the rate seen between T and
// the old bound.  The error buffers drift (they ramp up while the model is far from its
// optimum and relax later), so the bound is then moved by the factor the threshold is
// expected to move by: linear continuation of the last two thresholds while they rise,
// T_next / T = 2 - T_prev / T, geometric while they fall, T_next / T = T / T_prev.  Too high a bound (fewer than k caught) and too low a bound
// (buffer overflow) both cost a whole-row search, and the target kb = 2.5 k sits in the
// middle of the usable window [k, 7.5 k], so the trend is followed in full.  The bound only decides which search runs; the selection
// itself is exact either way.
__device__ __forceinline__ void next_bound(SelState* sel, uint32_t w, uint32_t k, uint32_t kb,
                                           uint32_t* bound, uint32_t* zero_at, const uint32_t* cand_total,
                                           uint32_t* overflow) {
    uint32_t nb = sel[w].next_bound;
    const uint32_t T = sel[w].T;
    uint32_t nz = T;                            // expected threshold of the next selection
    if (sel[w].active == 0u) {
        const uint32_t M = cand_total[w], L = bound[w];
        if (M < kb) {
            uint32_t drop = 1u << 19;                                   // about 6 % in magnitude
            if (M > k && T > L) {
                const float per_key = (float)(T - L) / (float)(M - k);   // pattern units per entry
                const float want = per_key * (float)(kb - M);
                drop = want >= 2097152.0f ? (1u << 21) : (uint32_t)want + 1u;
            }
            if (drop > (1u << 21)) drop = 1u << 21;
            nb = L > drop ? L - drop : 0u;
        }
    }
    if (sel[w].k_prev == k && sel[w].T_prev != 0u && T != 0u && T < 0x7f800000u && nb != 0u) {
        // rising thresholds ramp (linear continuation: T_next / T = 2 - T_prev / T), falling ones
        // decay (after k grew the accumulated residual drains by a constant factor per
        // iteration: T_next / T = T / T_prev)
        const float back = __uint_as_float(sel[w].T_prev) / __uint_as_float(T);
        float ratio = back <= 1.0f ? 2.0f - back : 1.0f / back;
        // a jump is not a trend: leave the bound where the last selection put it.  (A linear
        // ramp from the second to the third selection has ratio 1.5 and is still followed.)
        if (ratio < 0.4f || ratio > 1.5f) ratio = 1.0f;
        const float moved = __uint_as_float(nb) * ratio;
        if (moved > 0.0f && moved < 3.0e38f) nb = __float_as_uint(moved);
        const float moved_T = __uint_as_float(T) * ratio;
        if (moved_T > 0.0f && moved_T < 3.0e38f) nz = __float_as_uint(moved_T);
    }
    sel[w].T_prev = T;
    sel[w].k_prev = k;
    sel[w].seen = cand_total[w];
    bound[w] = nb;
    zero_at[w] = nz;
    overflow[w] = 0u;
}

// Filter bound from a sample.  Where no bound fits the coming selection (the first iteration, or k
// changed: Algorithm 2 re-chooses delta), one entry in `stride` of p = e + lr*g is computed ahead
// of the accumulate pass -- eight consecutive coordinates out of every 8 * stride, so that a
// sample point costs an eighth of a 32-byte access per array instead of a whole one -- and the
// radix select of S2 runs on that sample for the ranks
// k / stride and kb / stride: the patterns found there estimate the threshold and the pattern at
// the candidate target for the whole row (the count above the bound then misses its target by
// about 1 / sqrt(kb / stride), far inside the usable window [k, 3 kb]).  As always the bound only
// decides which search runs; the selection that follows is exact.
// With kFusedGrad the gradient is not read from g but generated for the sampled coordinates (the
// arithmetic of k_grad), for iterations whose gradient never reaches memory.
template <bool kFusedGrad>
__global__ __launch_bounds__(256) void k_sample_p(const float* __restrict__ e, const float* __restrict__ g,
                                                  GradSource src, uint64_t ld, uint32_t d, float lr,
                                                  uint32_t stride, uint32_t count,
                                                  float* __restrict__ sample, uint64_t sample_ld) {
    if (kFusedGrad) resolve_iteration(src);
    const uint32_t w = blockIdx.y;
    const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= count) return;
    const uint64_t coord = (uint64_t)(s >> 3) * 8u * stride + (s & 7u);
    float v = 0.0f;                            // past the end of the row: ranks last
    if (coord < (uint64_t)d) {
        const uint64_t at = (uint64_t)w * ld + coord;
        float gj;
        if (kFusedGrad) {
            const uint32_t j = (uint32_t)coord & ~3u;          // the quad the draw is made for
            float gq[4];
            grad_quad(src, grad_shared4(src, j), w, j, d, gq);
            gj = gq[(uint32_t)coord & 3u];
        } else {
            gj = g[at];
        }
        v = e[at] + lr * gj;
    }
    sample[(uint64_t)w * sample_ld + s] = v;
}
template __global__ void k_sample_p<false>(const float*, const float*, GradSource, uint64_t, uint32_t, float,
                                           uint32_t, uint32_t, float*, uint64_t);
template __global__ void k_sample_p<true>(const float*, const float*, GradSource, uint64_t, uint32_t, float,
                                          uint32_t, uint32_t, float*, uint64_t);

// One block per worker: the sample becomes the worker's view and the selection starts.
__global__ __launch_bounds__(256) void k_sample_begin(SelState* __restrict__ sel, uint32_t n, uint32_t k_s,
                                                      uint32_t kb_s, uint32_t count,
                                                      uint32_t* __restrict__ sample_total,
                                                      uint32_t* __restrict__ hist) {
    const uint32_t w = blockIdx.x;
    if (threadIdx.x == 0) { sel[w].active = 0u; sample_total[w] = count; }
    begin_selection(sel, w, n, k_s, kb_s, count, hist);
}

// One thread per worker: rank kb_s of the sample places the bound, rank k_s the expected threshold.
// sure_at (may be null): the pattern from which a candidate counts as sure to be sent, as far above the
// expected threshold as the bound lies below it (in pattern units, which follow the logarithm of the
// magnitude closely enough over a few per cent): 2 T - L, at least T + 1, at most the largest finite pattern.
__global__ __launch_bounds__(256) void k_sample_finish(const SelState* __restrict__ sel, uint32_t n,
                                                       uint32_t* __restrict__ bound,
                                                       uint32_t* __restrict__ zero_at,
                                                       uint32_t* __restrict__ sure_at, int sure_mode) {
    const uint32_t w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= n) return;
    const uint32_t L = sel[w].next_bound, T = sel[w].T;
    bound[w] = L;
    zero_at[w] = T;
    if (sure_at) {
        const uint64_t above = (uint64_t)T + (T > L ? T - L : 1u);
        uint32_t at = above > 0x7f7fffffull ? 0x7f7fffffu : (uint32_t)above;
        // test knobs: the line just above the expected threshold (k or more sure entries about every
        // other time: the selection falls back to the row), at infinity (nothing is sure), below the
        // expected threshold (always too many sure entries).  Fewer than k sure entries means the k-th
        // largest lies below the line, so every sure entry is sent: the count alone decides.
        if (sure_mode == 1) at = T + 1u;
        if (sure_mode == 2) at = 0x7f800000u;
        if (sure_mode == 3) at = T > L ? T - (T - L) / 2u : T + 1u;
        sure_at[w] = at;
    }
}

// One block of 1024 threads per worker walks the chunk counts in order and turns them into
// eq_before[c] (entries equal to T before chunk c) and out_base[c] (message offset of the
// chunk's first sent entry).  In place: cnt_eq -> eq_before, cnt_gt -> out_base.
__global__ __launch_bounds__(1024) void k_chunk_scan(SelViews vs, SelState* __restrict__ sel,
                                                     uint32_t* __restrict__ cnt_gt,
                                                     uint32_t* __restrict__ cnt_eq, uint32_t stride,
                                                     uint32_t k, uint32_t kb, uint32_t* __restrict__ bound,
                                                     uint32_t* __restrict__ zero_at,
                                                     uint32_t* __restrict__ cand_count,
                                                     uint32_t* __restrict__ overflow) {
    __shared__ uint32_t lds[17];
    const uint32_t w = blockIdx.x;
    const View v = view_of(vs, sel, w);
    const uint32_t nchunks = (v.count + 4095u) >> 12;
    const uint32_t r = sel[w].r;
    uint32_t* gtp = cnt_gt + (uint64_t)w * stride;
    uint32_t* eqp = cnt_eq + (uint64_t)w * stride;
    uint32_t eq_carry = 0, out_carry = 0;
    for (uint32_t base = 0; base < nchunks; base += 1024u) {
        const uint32_t c = base + threadIdx.x;
        const uint32_t gt = c < nchunks ? gtp[c] : 0u;
        const uint32_t eq = c < nchunks ? eqp[c] : 0u;
        uint32_t eq_total, out_total;
        const uint32_t eq_before = eq_carry + block_excl_scan(eq, lds, &eq_total);
        const uint32_t room = r > eq_before ? r - eq_before : 0u;
        const uint32_t sent = gt + (eq < room ? eq : room);
        const uint32_t out_base = out_carry + block_excl_scan(sent, lds, &out_total);
        if (c < nchunks) { eqp[c] = eq_before; gtp[c] = out_base; }
        eq_carry += eq_total;
        out_carry += out_total;
    }
    if (threadIdx.x == 0) next_bound(sel, w, k, kb, bound, zero_at, vs.cand_total, overflow);
    for (uint32_t q = threadIdx.x; q < kSubs; q += blockDim.x) cand_count[(w * kSubs + q) * kSubStride] = 0u;
}

// Writes the message (ascending coordinate) and makes e the residual: sent entries +0, all
// others their value.  In a row view the position is the coordinate and every sent entry is
// cleared.  In a candidate view map[pos] is the coordinate of entry pos, and the accumulate
// pass has already cleared the candidates at or above zero_used: only a sent entry below it
// still has to be cleared, and an unsent one at or above it gets its value back.  fix_e = 0
// leaves e alone altogether (the composed compressor's 4-bit stage writes the sent entries'
// residuals itself).
__global__ __launch_bounds__(256) void k_chunk_emit(SelViews vs, const SelState* __restrict__ sel,
                                                    const uint32_t* __restrict__ out_base,
                                                    const uint32_t* __restrict__ eq_before,
                                                    uint32_t stride, float* __restrict__ e,
                                                    uint32_t* __restrict__ msg_idx,
                                                    float* __restrict__ msg_val, uint64_t msg_ld,
                                                    uint32_t k, int fix_e) {
    __shared__ uint32_t lds[5];
    // the entries a round of the block sends are gathered here and leave with contiguous stores
    __shared__ uint32_t out_idx[1024];
    __shared__ float out_val[1024];
    const uint32_t w = blockIdx.y;
    const View v = view_of(vs, sel, w);
    const uint32_t nchunks = (v.count + 4095u) >> 12;
    const uint32_t T = sel[w].T, r = sel[w].r;
    const uint32_t zero_used = v.map ? sel[w].zero_used : 0xffffffffu;
    float* erow = e + (uint64_t)w * vs.ld;
    uint32_t* oi = msg_idx + (uint64_t)w * msg_ld;
    float* ov = msg_val + (uint64_t)w * msg_ld;
    for (uint32_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
        uint32_t eq_run = eq_before[(uint64_t)w * stride + c];
        uint32_t out_run = out_base[(uint64_t)w * stride + c];
        for (int s = 0; s < 4; ++s) {
            const uint32_t j = c * 4096u + s * 1024u + threadIdx.x * 4u;
            float vv[4] = {0.f, 0.f, 0.f, 0.f};
            uint32_t key[4] = {0, 0, 0, 0};
            bool valid[4] = {false, false, false, false};
            if (j < v.count) {
                const float4 x = *reinterpret_cast<const float4*>(v.row + j);
                vv[0] = x.x; vv[1] = x.y; vv[2] = x.z; vv[3] = x.w;
#pragma unroll
                for (int m = 0; m < 4; ++m) { valid[m] = j + m < v.count; key[m] = mag_key(vv[m]); }
            }
            uint32_t neq = 0;
#pragma unroll
            for (int m = 0; m < 4; ++m) neq += valid[m] && key[m] == T;
            uint32_t eq_total;
            uint32_t eq_rank = eq_run + block_excl_scan(neq, lds, &eq_total);
            bool send[4];
            uint32_t nsend = 0;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                bool take = false;
                if (valid[m]) {
                    if (key[m] > T) take = true;
                    else if (key[m] == T) { take = eq_rank < r; ++eq_rank; }
                }
                send[m] = take;
                nsend += take;
            }
            uint32_t send_total;
            uint32_t at = block_excl_scan(nsend, lds, &send_total);   // position inside this round
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const bool cleared = key[m] >= zero_used;          // already +0 in e
                if (send[m]) {
                    const uint32_t coord = v.map ? v.map[j + m] : j + m;
                    out_idx[at] = coord;
                    out_val[at] = vv[m];
                    ++at;
                    if (!cleared && fix_e) erow[coord] = 0.0f;
                } else if (valid[m] && cleared && fix_e) {
                    erow[v.map[j + m]] = vv[m];
                }
            }
            __syncthreads();
            for (uint32_t q = threadIdx.x; q < send_total; q += blockDim.x) {
                const uint32_t pos = out_run + q;
                if (pos < k) { oi[pos] = out_idx[q]; ov[pos] = out_val[q]; }
            }
            __syncthreads();
            eq_run += eq_total;
            out_run += send_total;
        }
    }
}

// ------------------------------------------------------------------------------------
// S4  U = sum_i Delta_i in worker order (Algorithm 1, server side), tile by tile.
// ------------------------------------------------------------------------------------
// k_msg_offsets finds, for every worker and
// every boundary b * kTile, how many of the worker's (ascending) indices lie below it; then one
// block per tile of kTile coordinates adds the workers' entries of its range into a tile in
// LDS, worker after worker (a barrier between workers keeps the summation order; indices
// inside one message are distinct, so the adds of one worker never collide), and writes the
// tile out with coalesced stores.  U is overwritten as a whole: no clearing before or after,
// and no scattered read-modify-write in HBM.
// count (may be null) gives the length of each worker's row where it is not k for all of them.
__global__ __launch_bounds__(256) void k_msg_offsets(const uint32_t* __restrict__ idx, uint64_t msg_ld,
                                                     uint32_t k, uint32_t ntiles,
                                                     uint32_t* __restrict__ off,
                                                     const uint32_t* __restrict__ count) {
    const uint32_t w = blockIdx.y;
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b > ntiles) return;
    const uint32_t* row = idx + (uint64_t)w * msg_ld;
    const uint64_t edge = (uint64_t)b * kTile;             // may exceed 2^32 at the last boundary
    uint32_t lo = 0, hi = count ? count[w] : k;            // first position with row[pos] >= edge
    while (lo < hi) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        if ((uint64_t)row[mid] < edge) lo = mid + 1u; else hi = mid;
    }
    off[(uint64_t)w * (ntiles + 1u) + b] = lo;
}

// With kApply the tile is not stored but used at once: xn = x - tile / n (S5 fused into S4), so
// the dense update never goes through HBM.  When x and xn are the same row, only the entries
// with a non-zero sum are touched.
// With the sure / band split (sv.sure non-null) a worker's message has two parts: the row idx / val
// holds what the compaction sent out of the band, and its sure entries lie in runs, one per
// 256-coordinate group, named by the run table sv.stab (kTile / 256 runs per tile).  Both are added
// in the worker's turn; the indices of one worker are distinct over both parts.
template <bool kApply>
__global__ __launch_bounds__(256) void k_aggregate_tiles(float* __restrict__ U,
                                                         const uint32_t* __restrict__ idx,
                                                         const float* __restrict__ val, uint64_t msg_ld,
                                                         const uint32_t* __restrict__ off,
                                                         uint32_t ntiles, uint32_t n, ModelRows rows,
                                                         float nf, SureView sv) {
    __shared__ __attribute__((aligned(16))) float tile[kTile];
    __shared__ uint32_t lo_s[256], hi_s[256];
    constexpr uint32_t kRuns = kTile / 256u;               // 16 runs per tile and worker
    constexpr uint32_t kHoist = 256u / kRuns;              // workers whose runs one round of loads covers
    __shared__ uint32_t run_first[256], run_at[kHoist * (kRuns + 1u)];
    const uint32_t b = blockIdx.x;
    const uint32_t base = b * kTile;
    // the tile of x_t is asked for first, so that it travels while the messages are located and summed
    // (not where one row is updated in place: there only the touched coordinates may be read at all)
    const float* x = rows.x;
    float* xn = rows.xn;
    float4 xv[kTile / 1024u];
    bool have_x = false;
    if (kApply) {
        if (rows.t_dev != nullptr) {
            const uint64_t t = *rows.t_dev;
            x = rows.ring + (t % rows.ring_slots) * rows.ring_ld;
            xn = rows.ring + ((t + 1u) % rows.ring_slots) * rows.ring_ld;
        }
        if (x != xn) {
            const float4* xin = reinterpret_cast<const float4*>(x + (uint64_t)base);
#pragma unroll
            for (uint32_t i = 0; i < kTile / 1024u; ++i) xv[i] = xin[threadIdx.x + i * 256u];
            have_x = true;
        }
    }
    for (uint32_t q = threadIdx.x; q < kTile; q += 256u) tile[q] = 0.0f;
    uint32_t entries = 0;                                  // message entries that fall into this tile
    for (uint32_t w0 = 0; w0 < n; w0 += 256u) {
        const uint32_t batch = n - w0 < 256u ? n - w0 : 256u;
        __syncthreads();                                   // tile zeroed / last batch's bounds consumed
        if (threadIdx.x < batch) {
            const uint32_t* o = off + (uint64_t)(w0 + threadIdx.x) * (ntiles + 1u) + b;
            lo_s[threadIdx.x] = o[0];
            hi_s[threadIdx.x] = o[1];
        }
        __syncthreads();
        for (uint32_t i0 = 0; i0 < batch; i0 += kHoist) {
            if (sv.sure != nullptr) {
                // the run descriptors of the next kHoist workers in one round of loads: thread t takes
                // run t % 16 of worker i0 + t / 16; prefix of the lengths inside each group of 16 lanes
                const uint32_t wi = i0 + (threadIdx.x / kRuns), r = threadIdx.x % kRuns;
                uint2 run = make_uint2(0u, 0u);
                if (wi < batch && sv.total[w0 + wi] != 0u)
                    run = sv.stab[(uint64_t)(w0 + wi) * sv.ngroups + (uint64_t)b * kRuns + r];
                uint32_t incl = run.y;
#pragma unroll
                for (uint32_t step = 1; step < kRuns; step <<= 1) {
                    const uint32_t up = __shfl_up(incl, step, kRuns);
                    if (r >= step) incl += up;
                }
                run_first[threadIdx.x] = run.x;
                run_at[(threadIdx.x / kRuns) * (kRuns + 1u) + r] = incl - run.y;
                if (r == kRuns - 1u) run_at[(threadIdx.x / kRuns) * (kRuns + 1u) + kRuns] = incl;
                __syncthreads();
            }
            const uint32_t i1 = i0 + kHoist < batch ? i0 + kHoist : batch;
            for (uint32_t i = i0; i < i1; ++i) {
                bool added = false;                        // same for the whole block
                if (sv.sure != nullptr) {
                    const uint32_t* at_of = run_at + (i - i0) * (kRuns + 1u);
                    const uint32_t* first_of = run_first + (i - i0) * kRuns;
                    const uint32_t total = at_of[kRuns];
                    entries += total;
                    added |= total != 0u;
                    const uint2* sw = sv.sure + (uint64_t)(w0 + i) * sv.cap;
                    for (uint32_t q = threadIdx.x; q < total; q += 256u) {
                        uint32_t r = 0;
#pragma unroll
                        for (uint32_t s = 1; s < kRuns; ++s) r += at_of[s] <= q;   // run holding entry q
                        const uint2 item = sw[first_of[r] + (q - at_of[r])];
                        const uint32_t at = item.x - base;
                        tile[at] = tile[at] + __uint_as_float(item.y);
                    }
                }
                const uint32_t lo = lo_s[i], hi = hi_s[i];
                if (lo != hi) {
                    const uint32_t* ri = idx + (uint64_t)(w0 + i) * msg_ld;
                    const float* rv = val + (uint64_t)(w0 + i) * msg_ld;
                    entries += hi - lo;
                    added = true;
                    for (uint32_t m = lo + threadIdx.x; m < hi; m += 256u) {
                        const uint32_t at = ri[m] - base;  // < kTile by the choice of lo, hi
                        tile[at] = tile[at] + rv[m];
                    }
                }
                // the next worker's additions come after this one's (a worker's own entries, sure and
                // band alike, name distinct coordinates and need no order among themselves)
                if (added) __syncthreads();
            }
            if (sv.sure != nullptr) __syncthreads();       // the descriptors are overwritten next round
        }
    }
    if (kApply) {
        if (x == xn && entries < kTile / 64u) {
            // one model row updated in place (message-queue form) and few entries: only the
            // coordinates some message named can change, x - (+0)/n being x itself, so only those
            // are read and written
            float* row = xn + (uint64_t)base;
            for (uint32_t q = threadIdx.x; q < kTile; q += 256u) {
                const float u = tile[q];
                if (__float_as_uint(u) != 0u) row[q] = row[q] - u / nf;
            }
            return;
        }
        const float4* xin = reinterpret_cast<const float4*>(x + (uint64_t)base);
        float4* xout = reinterpret_cast<float4*>(xn + (uint64_t)base);
#pragma unroll
        for (uint32_t i = 0; i < kTile / 1024u; ++i) {
            const uint32_t q = threadIdx.x + i * 256u;
            const float4 xq = have_x ? xv[i] : xin[q];
            const float4 uv = reinterpret_cast<const float4*>(tile)[q];
            float4 o;
            o.x = xq.x - uv.x / nf;
            o.y = xq.y - uv.y / nf;
            o.z = xq.z - uv.z / nf;
            o.w = xq.w - uv.w / nf;
            xout[q] = o;
        }
    } else {
        float4* out = reinterpret_cast<float4*>(U + (uint64_t)base);
        for (uint32_t q = threadIdx.x; q < kTile / 4u; q += 256u) out[q] = reinterpret_cast<const float4*>(tile)[q];
    }
}

template __global__ void k_aggregate_tiles<false>(float*, const uint32_t*, const float*, uint64_t, const uint32_t*,
                                                  uint32_t, uint32_t, ModelRows, float, SureView);
template __global__ void k_aggregate_tiles<true>(float*, const uint32_t*, const float*, uint64_t, const uint32_t*,
                                                 uint32_t, uint32_t, ModelRows, float, SureView);

// ---- a split message in its canonical form (inspection: ddef_get_message) -----------------------
// Worker w's message is its sure runs plus the band part of its message row; the one list in
// ascending coordinate order is put together tile by tile.  k_tile_sure_count: sure entries per
// tile; k_tile_scan: their exclusive prefix (in place); k_message_merge: a block marks its tile's
// entries of both parts in LDS, ranks them by coordinate and writes them at
// (sure entries before the tile) + (band entries before the tile).
__global__ __launch_bounds__(256) void k_tile_sure_count(SureView sv, uint32_t w, uint32_t ntiles,
                                                         uint32_t* __restrict__ tile_count) {
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= ntiles) return;
    constexpr uint32_t kRuns = kTile / 256u;
    const uint2* runs = sv.stab + (uint64_t)w * sv.ngroups + (uint64_t)b * kRuns;
    uint32_t total = 0;
    for (uint32_t r = 0; r < kRuns; ++r) total += runs[r].y;
    tile_count[b] = total;
}

__global__ __launch_bounds__(1024) void k_tile_scan(uint32_t* __restrict__ tile_count, uint32_t ntiles) {
    __shared__ uint32_t lds[17];
    uint32_t carry = 0;
    for (uint32_t base = 0; base < ntiles; base += 1024u) {
        const uint32_t b = base + threadIdx.x;
        const uint32_t v = b < ntiles ? tile_count[b] : 0u;
        uint32_t total;
        const uint32_t before = carry + block_excl_scan(v, lds, &total);
        if (b < ntiles) tile_count[b] = before;
        carry += total;
    }
}

__global__ __launch_bounds__(256) void k_message_merge(SureView sv, uint32_t w, const uint32_t* __restrict__ idx,
                                                       const float* __restrict__ val, uint64_t msg_ld,
                                                       const uint32_t* __restrict__ off, uint32_t ntiles,
                                                       const uint32_t* __restrict__ sure_before,
                                                       uint32_t* __restrict__ out_idx, float* __restrict__ out_val,
                                                       uint32_t k) {
    __shared__ float tile[kTile];
    __shared__ uint32_t present[kTile / 32u];
    __shared__ uint32_t lds[5];
    const uint32_t b = blockIdx.x, base = b * kTile;
    constexpr uint32_t kRuns = kTile / 256u;
    for (uint32_t q = threadIdx.x; q < kTile / 32u; q += 256u) present[q] = 0u;
    __syncthreads();
    const uint2* runs = sv.stab + (uint64_t)w * sv.ngroups + (uint64_t)b * kRuns;
    const uint2* sw = sv.sure + (uint64_t)w * sv.cap;
    for (uint32_t r = 0; r < kRuns; ++r) {
        const uint2 run = runs[r];
        for (uint32_t q = threadIdx.x; q < run.y; q += 256u) {
            const uint2 item = sw[run.x + q];
            const uint32_t at = item.x - base;
            tile[at] = __uint_as_float(item.y);
            atomicOr(&present[at >> 5], 1u << (at & 31u));
        }
    }
    const uint32_t* o = off + (uint64_t)w * (ntiles + 1u) + b;
    const uint32_t lo = o[0], hi = o[1];
    for (uint32_t m = lo + threadIdx.x; m < hi; m += 256u) {
        const uint32_t at = idx[(uint64_t)w * msg_ld + m] - base;
        tile[at] = val[(uint64_t)w * msg_ld + m];
        atomicOr(&present[at >> 5], 1u << (at & 31u));
    }
    __syncthreads();
    // thread t owns coordinates [16 t, 16 t + 16): half a presence word
    const uint32_t mine = (present[threadIdx.x >> 1] >> ((threadIdx.x & 1u) * 16u)) & 0xffffu;
    uint32_t total;
    uint32_t pos = sure_before[b] + lo + block_excl_scan((uint32_t)__popc(mine), lds, &total);
    for (uint32_t c = 0; c < 16u; ++c)
        if ((mine >> c) & 1u) {
            if (pos < k) { out_idx[pos] = base + threadIdx.x * 16u + c; out_val[pos] = tile[threadIdx.x * 16u + c]; }
            ++pos;
        }
}

// Last node of a captured iteration: t <- t + 1 in device memory.
__global__ void k_advance(uint64_t* t_dev) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *t_dev += 1u;
}

// S5  x_{t+1} = x_t - U / n, written into the next ring slot (may alias x_t when the ring
// has a single slot: element-wise, so in place is fine).  One quad per thread, single-wave
// blocks in address order.
__global__ __launch_bounds__(64) void k_apply(const float* x, const float* __restrict__ U, float* xn,
                                              uint32_t d, float nf) {
    const uint32_t q = blockIdx.x * 64u + threadIdx.x;
    if (q >= ((d + 3u) >> 2)) return;
    const float4 xv = reinterpret_cast<const float4*>(x)[q];
    const float4 uv = load_stream4(U + ((uint64_t)q << 2));
    float4 o;
    o.x = xv.x - uv.x / nf;
    o.y = xv.y - uv.y / nf;
    o.z = xv.z - uv.z / nf;
    o.w = xv.w - uv.w / nf;
    reinterpret_cast<float4*>(xn)[q] = o;
}

// Dense zero fill of a row (one quad per thread, single-wave blocks).
__global__ __launch_bounds__(64) void k_fill_f4(float* __restrict__ p, uint64_t quads) {
    const uint64_t q = (uint64_t)blockIdx.x * 64u + threadIdx.x;
    if (q < quads) reinterpret_cast<float4*>(p)[q] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// Plain copy of known size (one quad per thread, single-wave blocks): the yardstick that the
// hardware byte counters are scaled by.  src may equal dst.
__global__ __launch_bounds__(64) void k_copy_f4(const float* src, float* dst, uint64_t quads) {
    const uint64_t q = (uint64_t)blockIdx.x * 64u + threadIdx.x;
    if (q < quads) reinterpret_cast<float4*>(dst)[q] = reinterpret_cast<const float4*>(src)[q];
}

}  // namespace ddef
