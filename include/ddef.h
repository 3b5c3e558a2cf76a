/*
 * ddef — the data-parallel hot path of DD-EF-SGD / DeCo-SGD on one AMD MI355X (gfx950).
 *
 * One context simulates the n workers and the server of Algorithm 1 of the paper
 * ("DD-EF-SGD") with every worker's share resident in the GPU's HBM.  One iteration t is
 * the four calls, in this order,
 *
 *     ddef_grad            g_i = grad f_i(x_{t-tau}) + xi_i      (Assumption 2, Section 2.2.3)
 *     ddef_ef_compress     Delta_i = C_delta(e_i + gamma g_i),
 *                          e_i <- e_i + gamma g_i - Delta_i       (Algorithm 1, worker side)
 *     ddef_aggregate       U = sum_i Delta_i                      (Algorithm 1, server side)
 *     ddef_apply_delayed   x_{t+1} = x_t - U / n                  (Algorithm 1, server side)
 *
 * The delay tau lives in a ring of tau_max+1 parameter snapshots: iteration t takes its
 * gradient at the snapshot x_{t-tau} and applies the resulting update at once, which gives
 * the same iterates x_t as a server that holds every message for tau iterations.  While
 * t - tau < 0 nothing has arrived yet (the paper's convention Delta_{t-tau} = 0, Section
 * 3.2): those iterations leave x and every e_i unchanged and only advance t.
 *
 * C_delta is Top-k (Section 5.2: keep the k largest-magnitude entries) with
 * k = ceil(delta * d) clamped to [1, d].  The order is total: larger |v| first, compared on
 * the IEEE-754 bit pattern with the sign cleared, then lower index.  A message is the k
 * pairs (index, value) in ascending index order.
 *
 * Conventions for every function
 *   - returns DDEF_OK (0) or a negative DDEF_E* code; never throws, aborts or prints;
 *   - pointers named host_* are host memory owned by the caller, read or filled before the
 *     call returns; the library owns all device memory;
 *   - a context is bound to the HIP device that was current at ddef_init and to one stream;
 *     the four step calls only enqueue work on that stream, the getters and ddef_sync wait
 *     for it.  A context is not thread-safe;
 *   - all arithmetic of the method is IEEE fp32 with every operation rounded separately (no
 *     fused multiply-add; the fused steps inside the noise generator are part of its
 *     definition), indices are uint32, d < 2^32 - 8192 (so that rounding a length up to whole
 *     groups, chunks or tiles never leaves 32 bits).
 */
#ifndef DDEF_H
#define DDEF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DDEF_OK 0
#define DDEF_EINVAL (-1)     /* argument outside its domain, null pointer                 */
#define DDEF_ESTATE (-2)     /* call order violated                                       */
#define DDEF_ENOMEM (-3)     /* device or host allocation failed                          */
#define DDEF_EHIP (-4)       /* a HIP runtime call failed; sticky for the context         */
#define DDEF_ENONFINITE (-5) /* NaN/Inf appeared in e + lr*g; sticky until ddef_set_problem  */
#define DDEF_EINTERNAL (-6)  /* an invariant of the library broke on the device; sticky   */

#define DDEF_COMPRESSOR_TOPK 0  /* keep the k largest magnitudes (default)                  */
#define DDEF_COMPRESSOR_RANDK 1 /* keep k coordinates drawn at random per worker, iteration */
#define DDEF_COMPRESSOR_COMPOSED 2 /* Random-k, then Top-k of the kept ones, then 4-bit codes */

#define DDEF_NOISE_NONE 0
#define DDEF_NOISE_GAUSS 1      /* N(0,1) * noise_scale                                    */
#define DDEF_NOISE_STUDENT_T3 2 /* Student-t, 3 degrees of freedom, * noise_scale          */

typedef struct ddef_ctx ddef_ctx;

/* Problem statement of Algorithm 1: x in R^d, n workers, staleness at most tau_max.
 * Allocates e[n][d] = 0, g[n][d], the snapshot ring [tau_max+1][d], U[d] and work buffers
 * on the current device; tau starts at tau_max.  d in [1, 2^32 - 8192), n in [1, 65535], tau_max <= 4096.
 * On failure *out is NULL.  ENOMEM when the device cannot hold the state. */
int ddef_init(uint64_t d, uint32_t n, uint32_t tau_max, ddef_ctx** out);

/* The same problem with the server state of Algorithm 1 held literally: one model x_t, updated
 * in place, and a queue of the messages of the last tau_max+1 iterations in place of the
 * snapshot ring.  The four calls keep their order and meaning, except that in iteration t
 *   ddef_grad            takes the gradient at the current x_t (no iteration is empty) and
 *                        draws the noise keyed by t + tau, the iteration at which the message
 *                        is due, so that a constant tau gives bit for bit the iterates of
 *                        the ring form.  Keys never repeat: when tau falls and t + tau names an
 *                        iteration already used, the key is the last one plus one,
 *                        key_t = max(t + tau_t, key_{t-1} + 1);
 *   ddef_ef_compress     queues the messages Delta_{i,t} (these are what ddef_get_message
 *                        returns);
 *   ddef_aggregate       sums the messages Delta_{i,t-tau} sent tau iterations earlier; U = 0
 *                        while t < tau (Section 3.2's convention).
 * tau may change between iterations within [0, tau_max]: the server then applies whatever was
 * sent tau_t iterations before t, so a message can be applied twice or never, as with a real
 * queue whose delay changes.  Top-k only: ddef_set_compressor rejects the others with EINVAL.
 * Memory: x[d] and messages [tau_max+1][n][k] (index, value), not [tau_max+1][d] snapshots;
 * the gradient prefetch option has no effect (the next gradient needs x_{t+1}). */
int ddef_init_queue(uint64_t d, uint32_t n, uint32_t tau_max, ddef_ctx** out);
int ddef_destroy(ddef_ctx* ctx);

/* Use a caller-provided hipStream_t (passed as void*) for all later work; NULL restores
 * the context's own stream.  The caller keeps the stream alive.  Only between iterations. */
int ddef_set_stream(ddef_ctx* ctx, void* hip_stream);

/* The synthetic objective f(x) = 1/2 sum_j lambda_j (x_j - xstar_j)^2 shared by all workers
 * (IID data) and the start point: copies three host arrays of d floats, sets every snapshot
 * to x0, every error buffer to 0 and t to 0.  Gradient noise xi = noise_scale * z with z a
 * counter-based draw keyed by (seed, t, worker, j): Philox4x32-10 words turned into normals by
 * Box-Muller (four coordinates to a block) or into Student-t(3) draws (three words each, four
 * coordinates to three blocks), out of exactly rounded fp32 operations only, so that any
 * implementation of the same definition reproduces every draw bit for bit. */
int ddef_set_problem(ddef_ctx* ctx, const float* host_lambda, const float* host_xstar,
                     const float* host_x0, uint64_t seed, int noise_kind, float noise_scale);

/* The sparsifier C_delta of the following iterations.  Top-k is the paper's default
 * (Section 5.2); Random-k is its other sparsifier (appendix "Experiment Results with other
 * sparsifiers": k entries chosen at random).  Random-k keeps the coordinates pi(0..k-1) of a
 * permutation pi of [0, d) keyed by (seed, t, worker): a 4-round Feistel network over the
 * smallest even-width bit field holding d, round function MurmurHash3's 32-bit finaliser of
 * (half XOR round key), cycle-walked into [0, d), round keys from Philox4x32-10 with counter
 * (0xFFFFFFFF, worker, t).  Messages, error feedback and k = ceil(delta*d) are as for Top-k;
 * ddef_get_threshold reports (0, 0).
 * Composed is the compressor the paper gives for its strongest static baseline (Section 5.2
 * "Baselines": Random-k with 20 %, Top-k with 10 %, 4-bit quantisation); the paper describes it no
 * further, the stages below are this library's reading.  (1) Random-k as above keeps
 * k1 = ceil(rand_ratio * d) coordinates (ddef_set_composed, default 0.2).  (2) Top-k keeps the
 * k = ceil(delta * k1) largest of those under the same total order (magnitude descending,
 * coordinate ascending); delta is ddef_ef_compress's argument, and ddef_get_threshold reports
 * this selection.  (3) The k values, in ascending coordinate order, are cut into blocks of 256:
 * step = (largest magnitude in the block) / 7, code = value / step rounded to the nearest integer
 * (halves to even) inside [-7, 7], all codes 0 where step is 0.  Delta holds what the receiver
 * decodes, code * step (that is what ddef_get_message returns and the aggregation sums), so
 * e' = p - Delta keeps the coding error with everything not sent.  Ring form only.
 * Only between iterations. */
int ddef_set_compressor(ddef_ctx* ctx, int kind);
/* Share of the coordinates the Random-k stage of the composed compressor keeps, in (0, 1].
 * Between iterations. */
int ddef_set_composed(ddef_ctx* ctx, double rand_ratio);

/* Heterogeneous local objectives (Assumption 3; the paper's non-IID experiments): worker i's
 * quadratic has the optimum xstar + zeta * u_i instead of xstar, u_i a standard normal vector
 * fixed by (seed, i) -- the same counter-based draw as the gradient noise, under the step key
 * 2^64 - 2 that no iteration reaches.  zeta = 0 (default) is the IID case.  Between iterations. */
int ddef_set_heterogeneity(ddef_ctx* ctx, float zeta);

/* Staleness for the following iterations, 0..tau_max (Algorithm 2 re-chooses it every E
 * iterations).  Only between iterations, else ESTATE. */
int ddef_set_tau(ddef_ctx* ctx, uint32_t tau);

/* Stochastic gradient of every worker at the stale iterate:
 * g_i[j] = lambda[j] * (x_{t-tau}[j] - xstar[j]) + noise_scale * z(seed, t, i, j).
 * While t - tau < 0 the iteration is marked empty and no gradient is produced. */
int ddef_grad(ddef_ctx* ctx);

/* Test hook: replace worker `worker`'s gradient by d host floats (instead of, or after,
 * ddef_grad) and mark the iteration as non-empty. */
int ddef_load_grad(ddef_ctx* ctx, uint32_t worker, const float* host_g);

/* Error feedback and Top-k for every worker: p = e + lr*g (two roundings), the k entries of
 * p first in the order above become the message, e <- p with the sent entries set to +0.
 * delta in (0, 1] (double, so that k = ceil(delta*d) is the intended integer); lr is the
 * stepsize gamma.  On an empty iteration the messages are empty and e is untouched. */
int ddef_ef_compress(ddef_ctx* ctx, double delta, float lr);

/* Dense sum of the n messages, U[j] = ((0 + Delta_0[j]) + Delta_1[j]) + ..., in worker
 * order, which makes the fp32 result reproducible.  The sum is formed tile by tile in on-chip
 * memory, and that is carried out by ddef_apply_delayed in the same pass that updates the
 * model, so the dense U never travels through device memory; this call only locates each
 * tile's entries in the (index-ordered) messages.  ddef_get_update returns U all the same (it
 * computes the sum on its own when asked), from this call until the next ddef_ef_compress. */
int ddef_aggregate(ddef_ctx* ctx);

/* x_{t+1} = x_t - U / (float)n, stored as the next snapshot; t <- t + 1.  lr must be the
 * value given to ddef_ef_compress in this iteration (the stepsize acts inside the error
 * feedback, as in Algorithm 1; it is checked, not applied a second time), else EINVAL. */
int ddef_apply_delayed(ddef_ctx* ctx, float lr);

/* One whole iteration: the four calls above in order, with the same results and errors.
 * With DDEF_OPT_GRAPH set, a steady iteration (ring form, Top-k, t >= tau, the same k, lr and
 * tau as the iteration before, no buffer to grow, profiling and prefetch off) is recorded once
 * as a HIP graph and replayed from then on: one graph launch instead of some sixteen kernel
 * launches, which is what small problems are bound by.  Inside the graph the iteration number
 * is read from device memory, so nothing in it changes from replay to replay.  Any change of
 * k, lr, tau, an option, the stream or the problem drops the recording; the next steady
 * iteration records a new one.  Iterations that do not qualify run the four calls as usual. */
int ddef_step(ddef_ctx* ctx, double delta, float lr);
int ddef_graph_replays(ddef_ctx* ctx, uint64_t* count);   /* iterations served by a replay so far */

/* Wait for the context's stream.  Also reports what the kernels flagged meanwhile:
 * DDEF_ENONFINITE when some e + lr*g was Inf or NaN (the method needs finite values; the
 * context then refuses further work until ddef_set_problem), DDEF_EINTERNAL when a device-side
 * invariant broke.  ddef_get_message reports the same. */
int ddef_sync(ddef_ctx* ctx);

/* ---- inspection / checkpoint hooks (each waits for the stream) ------------------------ */
int ddef_step_index(ddef_ctx* ctx, uint64_t* t);
int ddef_get_model(ddef_ctx* ctx, float* host_x);                       /* x_t, d floats  */
/* The objective the method minimises, at the current iterate (Section 2.1, problem (1)):
 * f(x_t) = (1/n) sum_i f_i(x_t), f_i(x) = 1/2 sum_j lambda_j (x_j - x*_ij)^2 with worker i's optimum
 * x*_i = xstar + zeta u_i (ddef_set_heterogeneity).  Computed on the device in double from the
 * fp32 state (the order of the additions is fixed for a given d and device, so the value is reproducible);
 * waits for the stream.  *host_f: host pointer.  ESTATE before ddef_set_problem. */
int ddef_objective(ddef_ctx* ctx, double* host_f);
int ddef_set_model(ddef_ctx* ctx, const float* host_x);                 /* overwrite x_t  */
/* Checkpoint and resume (ring form, between iterations): the state of a run is t, the
 * snapshots x_{t-age} for age = 0 .. min(t, tau_max) and the error buffers (the problem, tau and
 * the options are the caller's to set again).  ddef_get_snapshot / ddef_set_snapshot copy one
 * snapshot (EINVAL when age > tau_max or, for the getter, age > t); ddef_set_step_index sets t.
 * Restore in this order: ddef_set_problem, ddef_set_step_index, every snapshot, every error
 * buffer.  A resumed run continues bit for bit like the uninterrupted one (the candidate filter
 * starts afresh, which only decides which search runs).  The message-queue form keeps state in
 * its queue that these calls do not cover: ESTATE there. */
int ddef_get_snapshot(ddef_ctx* ctx, uint32_t age, float* host_x);
int ddef_set_snapshot(ddef_ctx* ctx, uint32_t age, const float* host_x);
int ddef_set_step_index(ddef_ctx* ctx, uint64_t t);
int ddef_get_error(ddef_ctx* ctx, uint32_t worker, float* host_e);
int ddef_set_error(ddef_ctx* ctx, uint32_t worker, const float* host_e);
int ddef_get_grad(ddef_ctx* ctx, uint32_t worker, float* host_g);
int ddef_get_update(ddef_ctx* ctx, float* host_U);   /* U of the last ddef_aggregate; valid until the next ddef_ef_compress */
/* Last message of a worker: *k entries (0 on an empty iteration), ascending index.
 * host_idx / host_val may be NULL to query k only; otherwise they hold at least k items. */
int ddef_get_message(ddef_ctx* ctx, uint32_t worker, uint32_t* host_idx, float* host_val,
                     uint64_t* k);
/* Wire form of a worker's last message under the composed compressor (Section 5.2 "Baselines",
 * 4-bit stage as read in ddef_set_compressor's comment): (k+1)/2 bytes of codes, entry 2m in the
 * low and entry 2m+1 in the high nibble of byte m, two's complement, a missing last entry 0; and
 * (k+255)/256 block steps.  Entry m decodes to code * steps[m / 256] at coordinate idx[m] of
 * ddef_get_message.  host_codes / host_steps may be NULL to query k.  ESTATE under another
 * compressor. */
int ddef_get_message_codes(ddef_ctx* ctx, uint32_t worker, uint8_t* host_codes, float* host_steps,
                           uint64_t* k);
/* Threshold of the last selection: T = smallest selected magnitude pattern, r = how many
 * selected entries carry exactly T. */
int ddef_get_threshold(ddef_ctx* ctx, uint32_t worker, uint32_t* T, uint64_t* r);

/* ---- host-side scalar pieces ------------------------------------------------------------ */
/* k = ceil(delta*d) clamped to [1, d]; 0 when delta is outside (0, 1] or d is 0. */
uint64_t ddef_k_from_delta(double delta, uint64_t d);
/* DeCo (Algorithm 3): scan tau from ceil((b + V_g/a)/T_comp) down to ceil(b/T_comp) with
 * delta = min{(tau T_comp - b) a / V_g, T_comp a / V_g, 1}, skip candidates with
 * delta <= 0, keep the minimal phi, smallest tau on ties.  v_g_bits, a_bps (bits/s),
 * t_comp_s > 0, b_s >= 0.  EINVAL when no candidate exists. */
int ddef_deco(double v_g_bits, double a_bps, double b_s, double t_comp_s, uint32_t* tau,
              double* delta);
/* The same scan minimising phi' = phi / delta, the key factor when data is non-IID (Remark on
 * phi; Section 5.6 replaces phi by it). */
int ddef_deco_noniid(double v_g_bits, double a_bps, double b_s, double t_comp_s, uint32_t* tau,
                     double* delta);
double ddef_phi_prime(double delta, double tau);
/* The two corners of the (tau, delta) plane that Algorithm 3's joint choice is measured against
 * (Section 2.2: compression alone, delayed aggregation alone), placed by the same two quantities
 * the algorithm scans between.  Compression only: tau = 0 and the ratio whose transfer takes one
 * computation time, delta = min{T_comp a / V_g, 1}.  Delay only: delta = 1 and the staleness at
 * which Algorithm 3's scan starts, tau = ceil((b + V_g / a) / T_comp), at most tau_max. */
int ddef_corner_compression_only(double v_g_bits, double a_bps, double t_comp_s, double* delta);
int ddef_corner_delay_only(double v_g_bits, double a_bps, double b_s, double t_comp_s, uint32_t tau_max,
                           uint32_t* tau);
/* DeCo's objective phi(delta, tau) = (1 - delta) / (delta (1 - delta/2)^tau) (Theorems 1 and 2,
 * Algorithm 3); NaN outside 0 < delta <= 1, tau >= 0. */
double ddef_phi(double delta, double tau);
/* Theorem 3: T_avg ~ max{(T_comp + b + delta V_g / a) / (tau + 1), delta V_g / a, T_comp}. */
double ddef_t_avg_model(uint32_t tau, double delta, double v_g_bits, double a_bps, double b_s,
                        double t_comp_s);
/* The pipeline recurrence the theorem is proved from (Section 4.1 and the proof of Theorem 3:
 * computation k+1 starts when computation k is done and message k - tau has arrived; a
 * message takes delta V_g / a on the wire, one at a time, plus the latency b), run for
 * `iterations` iterations; returns the arrival time of the last message divided by their
 * number, the quantity the theorem's error bound (b + min{T_comp, delta V_g/a}) / E is for. */
double ddef_t_avg_simulate(uint32_t tau, double delta, double v_g_bits, double a_bps, double b_s,
                           double t_comp_s, uint64_t iterations);
/* Look-up table of Section 4.5: DeCo precomputed at `points` bandwidths spaced evenly over
 * [a_min, a_max] for a measured latency b.  A query inside the range returns the entry of the
 * nearest sample point (*from_table = 1); outside it DeCo is evaluated online
 * (*from_table = 0; from_table may be NULL).  The caller destroys the table. */
typedef struct ddef_lut ddef_lut;
int ddef_lut_build(double v_g_bits, double a_min_bps, double a_max_bps, uint32_t points, double b_s,
                   double t_comp_s, ddef_lut** out);
int ddef_lut_query(const ddef_lut* lut, double a_bps, uint32_t* tau, double* delta, int* from_table);
int ddef_lut_destroy(ddef_lut* lut);

/* ---- measurement hooks ------------------------------------------------------------------ */
/* With profiling on, every kernel launch is bracketed by HIP events on the context's
 * stream; ddef_profile_read waits for the stream and returns, for kernel slot `slot`
 * (0 .. ddef_profile_slots()-1), its name, the launches since profiling was switched on and
 * their summed duration in milliseconds. */
int ddef_profile_enable(ddef_ctx* ctx, int on);
int ddef_profile_slots(void);
int ddef_profile_read(ddef_ctx* ctx, int slot, const char** name, uint64_t* launches,
                      double* total_ms);
/* What the device of this context reports about itself (hipGetDeviceProperties): compute
 * units, wavefront width, LDS bytes per compute unit, device memory in bytes, shader and memory
 * clocks in kHz, memory bus width in bits, and the architecture name (at most name_len - 1
 * characters, NUL-terminated).  Any pointer may be NULL. */
int ddef_device_info(ddef_ctx* ctx, uint32_t* compute_units, uint32_t* wave_size, uint64_t* lds_bytes_per_cu,
                     uint64_t* memory_bytes, uint32_t* clock_khz, uint32_t* memory_clock_khz,
                     uint32_t* memory_bus_bits, char* arch_name, uint32_t name_len);

/* Yardstick for hardware byte counters: one launch of a plain copy kernel (k_copy_f4) that
 * reads and rewrites the gradient scratch row of worker 0 in place; *bytes_each_way is the
 * number of bytes it reads (= writes).  Between iterations only; the gradient scratch is
 * rewritten by the next ddef_grad anyway. */
int ddef_copy_probe(ddef_ctx* ctx, uint64_t* bytes_each_way);
/* How many worker selections so far took the multi-pass path over the whole vector
 * (counted over all workers and iterations since ddef_set_problem), plus one for every worker and
 * iteration of the composed compressor whose recording pass had to be repeated without its bound. */
int ddef_full_select_count(ddef_ctx* ctx, uint64_t* count);
/* Diagnostics of a worker's last selection: the magnitude bound its candidate filter will use
 * next, how many candidates the filter caught this time, and whether the selection had to
 * search the whole row (1) or found the top-k among the candidates (0). */
int ddef_get_filter_state(ddef_ctx* ctx, uint32_t worker, uint32_t* next_bound, uint32_t* candidates,
                          uint32_t* searched_row);
/* Tuning / test knobs; see DDEF_OPT_*.  Only between iterations. */
#define DDEF_OPT_FORCE_FULL_SELECT 1 /* 1: never use the candidate filter                 */
#define DDEF_OPT_CANDIDATE_SLACK_X16 2 /* candidate target = k * value / 16 (default 40)  */
#define DDEF_OPT_PREFETCH_GRAD 3 /* 1: ddef_grad also starts the gradient of the NEXT iteration
                                  * on a second stream (it only needs x_{t+1-tau}, tau >= 1), so
                                  * that its arithmetic overlaps the memory-bound rest of the
                                  * iteration; results are unchanged.  Costs a second gradient
                                  * buffer of n*d floats.  Default 0: measured on MI355X the two
                                  * kernels share the chip poorly (the whole step gains about
                                  * 10 %, the streaming pass loses most of its bandwidth while
                                  * they overlap).                                              */
#define DDEF_OPT_GRAPH 5     /* 1: ddef_step records steady iterations as a HIP graph and replays it */
#define DDEF_OPT_FUSE_GRAD 4 /* 1: ddef_grad launches nothing; ddef_ef_compress generates the gradient
                              * inside the accumulate pass, so it never touches HBM (8 bytes less per
                              * worker and element).  Results are unchanged.  ddef_get_grad then works
                              * only between ddef_grad and ddef_apply_delayed (it regenerates the
                              * values); ddef_load_grad and Random-k fall back to a stored gradient.
                              * Default 0: the pass becomes bound by the generator's arithmetic.      */
#define DDEF_OPT_RANDK_BUCKET_PERCENT 6 /* Random-k with k >= 2^20 sorts the kept coordinates into
                              * buckets by coordinate region before it sets their bits; a bucket
                              * holds its expected fill plus 8 standard deviations (value 0,
                              * default), and what does not fit is set bit by bit.  A value of
                              * 1..400 sizes the buckets at that percentage of the expected fill
                              * instead (tests use it to exercise the overflow path).  Results are
                              * unchanged.                                                          */
#define DDEF_OPT_COMPOSED_BOUND 7 /* composed compressor: 1 (default) records only the kept entries above a
                              * bound placed from a sample of e + lr*g, which a few more than k of them
                              * are expected to pass; for a worker where fewer than k did, the pass is
                              * repeated without the bound (the repeat is enqueued every time and decided
                              * on the device, so ddef_ef_compress does not wait for the stream); 0 always
                              * records every kept entry; 2 places the bound too high on purpose (tests of
                              * the repeat).  Results are unchanged.                                 */
#define DDEF_OPT_DENSE_SPLIT 8 /* 1 (default): where messages are dense (k/d > 1/32; ring form, Top-k; the filter
                              * bound is then placed from a sample of e + lr*g in every iteration), the
                              * candidates a margin above the expected threshold count as
                              * sure to be sent: they are recorded once, in runs, and go to the aggregation as
                              * they are, and only the band around the threshold is ordered, searched and
                              * compacted.  A worker's message then lies in device memory in two parts;
                              * ddef_get_message puts them together.  0: one part, every candidate searched.
                              * 2, 3, 4 (tests): the line between sure and band is put just above the expected
                              * threshold (about every other selection then counts k or more sure entries and
                              * falls back to its row), at infinity (nothing is sure), or below the expected
                              * threshold (always too many sure entries).  Results are unchanged.           */
int ddef_set_option(ddef_ctx* ctx, int option, int64_t value);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The work of ddef_ef_compress (Top-k compressor) on
 * buffers the caller owns, with no allocation of any kind and no context: for each of the n
 * workers, p = e + lr*g is written over e, the k = ceil(delta*d) entries first in the total order
 * become the message (ascending coordinate) and are cleared in e.  Same results, bit for bit, as
 * ddef_ef_compress on the same e and g.
 *   dev_e, dev_g     device pointers, n rows of ld floats each, 16-byte aligned; ld >= d and a
 *                    multiple of 4; entries [d, ld) of a row are read and rewritten but never
 *                    selected.  Finite values are required (nothing reports Inf/NaN here).
 *   dev_msg_idx/val  device pointers, n rows of msg_ld >= k entries; row w receives worker w's
 *                    message, entries beyond k are left alone.
 *   hip_stream       hipStream_t (as void*) of the current device; NULL is the null stream.  The
 *                    call only enqueues kernels (eleven launches, no memset or copy nodes), so it
 *                    may be recorded into a HIP graph.
 * The selection always searches the whole rows (no candidate filter: that needs buffers sized by
 * k).  Its work memory -- selection state, histograms, per-chunk counts -- is a fixed array of
 * about 21 MiB in the library's device image, one copy per GPU for the life of the process,
 * which bounds the size: n <= 64 and n * ceil(d/4096) <= 2^21 (8 workers of 10^9 coordinates,
 * 64 of 1.3*10^8), else EINVAL.  Every call on a GPU shares that array: calls that overlap on
 * one GPU (two streams, two threads) race; calls on one stream are safe back to back.
 * EINVAL also for null or misaligned pointers, delta outside (0, 1], d = 0, msg_ld < k. */
int ddef_ef_compress_static(float* dev_e, const float* dev_g, uint64_t ld, uint64_t d, uint32_t n,
                            double delta, float lr, uint32_t* dev_msg_idx, float* dev_msg_val,
                            uint64_t msg_ld, void* hip_stream);

const char* ddef_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* DDEF_H */
