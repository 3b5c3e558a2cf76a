// CPU oracle for the DD-EF-SGD step (test infrastructure, not part of the product).
//
// A plain, slow, single-pass-per-idea statement of what one iteration of DD-EF-SGD
// (Algorithm 1 of the paper) computes for n simulated workers on the synthetic
// diagonal quadratic f(x) = 1/2 sum_j lambda_j (x_j - x*_j)^2.  It exists so that the
// GPU library can be checked against it; only the tests, the smoke check and the
// benchmark's cpu_baseline leg may call it.  It shares no code with the GPU library.
//
// Arithmetic is fp32 with every operation rounded on its own (build with
// -ffp-contract=off, no fast-math): the acceptance bar is bit-exact indices and error
// buffers, which a wider oracle could not decide.
//
// What follows what:
//   gradient          g = grad f_i(x) + xi                    Assumption 2 (bounded noise)
//   stale iterate     gradient taken at x_{t-tau}             Section 2.2.3
//   EF accumulate     p = e + gamma*g                         Algorithm 1, worker side
//   compressor        Top-k of p, k = ceil(delta*d)           Section 5.2 "Baselines"; Top-k lemma
//   other sparsifier  Random-k: k entries chosen at random    Appendix "Experiment Results with other sparsifiers"
//   composed          Random-k, Top-k inside it, 4-bit codes  Section 5.2 "Baselines" (the strongest static baseline's compressor)
//   residual          e' = e + gamma*g - Delta                Algorithm 1, worker side
//   server update     x' = x - (1/n) sum_i Delta_i            Algorithm 1, server side
//   start-up          Delta_{t-tau} = 0 while t-tau < 0       Section 3.2, boundary convention
//   DeCo              (tau*, delta*) minimising phi           Algorithm 3, Remark on delta*(tau)
//   timing            TS/TM/TC recurrence, T_avg closed form  Section 4.1, Theorem 3 and its proof
//   objective         f(x) = (1/n) sum_i f_i(x)               Section 2.1, problem (1)
//
// Two forms of the delay are coded.  The normative one keeps a ring of parameter
// snapshots and takes the gradient at the old iterate x_{t-tau}; the literal one
// (queue_run) is Algorithm 1 as printed: workers at the current x_t, the server holding
// messages for tau steps.  For constant tau they must give the same x_t for every t.
//
// Pins (tests/test_oracle_*.py): brute-force top-k on tiny d, exhaustive subsets, the
// bit-exact EF identity Delta + e' = p, conservation, the nested-virtual-sequence
// identity, the Top-k contraction bound, delta=1/tau=0 -> D-SGD, delta=1 -> delayed SGD,
// the closed form (1-lr*lambda)^t on the noiseless quadratic, ring form == queue form,
// Philox known answers, the noise transform against libm, DeCo's degenerate values and
// Theorem 3 against the recurrence.  The composed compressor (tests/test_oracle_composed.py):
// its selection against a numpy sort of the Random-k subset, its quantiser against a hand-worked
// block, the nearest-level property by brute force over all 15 levels, the case whose values lie
// on the 4-bit grid (lossless: equals plain Top-k), conservation and the contraction.  Under a *changing* (tau, delta) -- Algorithm 2
// re-chooses both while Algorithm 1 runs; the paper prints no trajectory for it -- both forms are
// pinned against numpy replays written from the reading "iteration t uses what lies tau_t iterations
// back": at delta = 1 (SGD with a time-varying delay) and at delta < 1 (error feedback and Top-k by a
// full stable sort), messages, error buffers and iterates bit for bit (tests/test_oracle_step.py).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <thread>
#include <vector>

namespace {

inline uint32_t bits_of(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float float_of(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }
inline uint32_t magnitude_key(float f) { return bits_of(f) & 0x7fffffffu; }

// ---------------------------------------------------------------------------------
// Counter-based noise.  Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random
// numbers: as easy as 1, 2, 3", SC'11) keyed by the seed, counter = (j, worker, step).
// ---------------------------------------------------------------------------------
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// -2 ln(u) for u = ((w >> 8) + 1) / 2^24 in (0, 1], from +,-,* and fused multiply-add
// (std::fmaf: one rounding, the same on every IEEE machine):
// u = 2^(e-24) * m, m folded into (sqrt(1/2), sqrt(2)], f = m - 1,
// ln(1 + f) = f + f^2 g(f) with g a degree-7 polynomial (the Chebyshev interpolant of
// (ln(1+f) - f) / f^2 on that interval, coefficients rounded to fp32; |error of ln m| < 4e-8).
float neg2ln_uniform(uint32_t w) {
    uint32_t a = (w >> 8) + 1u;                       // 1 .. 2^24, exact as a float
    uint32_t fb = bits_of((float)a);
    int e = (int)(fb >> 23) - 127;                    // 0 .. 24
    uint32_t mant = fb & 0x7fffffu;
    float m = float_of(mant | 0x3f800000u);           // [1, 2)
    if (mant > 0x3504f3u) { m = m * 0.5f; e += 1; }   // fold above sqrt(2)
    float f = m - 1.0f;
    float g = 0x1.67ed28p-4f;
    g = std::fmaf(g, f, -0x1.21fd54p-3f);
    g = std::fmaf(g, f, 0x1.2fd102p-3f);
    g = std::fmaf(g, f, -0x1.53bb74p-3f);
    g = std::fmaf(g, f, 0x1.99071p-3f);
    g = std::fmaf(g, f, -0x1.000302p-2f);
    g = std::fmaf(g, f, 0x1.555638p-2f);
    g = std::fmaf(g, f, -0x1.fffffep-2f);
    float lnm = std::fmaf(f * f, g, f);
    float v = std::fmaf((float)(24 - e), 0x1.62e43p-1f, -lnm);   // (24-e) ln 2 - ln m = -ln u >= 0
    v = v < 0.0f ? 0.0f : v;
    return 2.0f * v;
}

// cos and sin of the angle 2*pi*((w >> 8) + 1/2) / 2^24: quadrant from the top bits after
// an eighth-turn shift, Taylor polynomials on (-pi/4, pi/4) for the rest (Horner with fmaf).
void unit_circle_point(uint32_t w, float* cos_out, float* sin_out) {
    uint32_t b = ((w >> 8) + 0x200000u) & 0xffffffu;
    uint32_t q = b >> 22;
    int r = (int)(b & 0x3fffffu) - 0x200000;          // [-2^21, 2^21)
    float phi = (float)(2 * r + 1) * 0x1.921fb6p-23f;   // pi / 2^24 rounded to fp32
    float p2 = phi * phi;
    float sp = 1.0f / 362880.0f;
    sp = std::fmaf(sp, p2, -1.0f / 5040.0f);
    sp = std::fmaf(sp, p2, 1.0f / 120.0f);
    sp = std::fmaf(sp, p2, -1.0f / 6.0f);
    sp = std::fmaf(sp, p2, 1.0f);
    float s = phi * sp;
    float cp = -1.0f / 3628800.0f;
    cp = std::fmaf(cp, p2, 1.0f / 40320.0f);
    cp = std::fmaf(cp, p2, -1.0f / 720.0f);
    cp = std::fmaf(cp, p2, 1.0f / 24.0f);
    cp = std::fmaf(cp, p2, -0.5f);
    float c = std::fmaf(cp, p2, 1.0f);
    switch (q) {
        case 0: *cos_out = c;  *sin_out = s;  break;
        case 1: *cos_out = -s; *sin_out = c;  break;
        case 2: *cos_out = -c; *sin_out = -s; break;
        default: *cos_out = s; *sin_out = -c; break;
    }
}

// Standard draw z(seed, t, worker, j) from one Philox block (w0..w3).
// kind 1: Box-Muller normals, four coordinates to a block: the block of counter (j >> 2, worker,
//   t) serves coordinates 4q .. 4q+3 with the two independent pairs
//   (sqrt(-2 ln u(w0)) cos(angle(w1)), the same radius times sin) and likewise from (w2, w3).
// kind 2: Student-t with 3 degrees of freedom, z0 / sqrt(chi2_3 / 3), where chi2_3 is the
//   square of the second Box-Muller normal z1 = sqrt(-2 ln u(w0)) sin(angle(w1)) plus an
//   independent chi-square with 2 degrees of freedom, -2 ln u(w2) (the squared radius of a
//   second Box-Muller pair, which needs no angle).  With R2 = -2 ln u(w0), z0 = sqrt(R2) cos and
//   z1^2 = R2 sin^2, the quotient is cos * sqrt(3 R2 / (R2 sin^2 + chi2_2)): one division and
//   one square root.  A draw takes three words; the four coordinates 4q .. 4q+3 take the twelve
//   words of the three blocks with counters (3q, worker, t), (3q+1, ..), (3q+2, ..) in order:
//   coordinate 4q+c uses words 3c, 3c+1, 3c+2 of that sequence as (radius, angle, chi-square).
// kind 0: no noise.
float noise_z(uint64_t seed, uint64_t t, uint32_t worker, uint32_t j, int kind) {
    if (kind == 0) return 0.0f;
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    float c01, s01;
    if (kind == 1) {
        uint32_t ctr[4] = {j >> 2, worker, (uint32_t)t, (uint32_t)(t >> 32)};
        philox4x32_10(ctr, key, w);
        uint32_t pair = (j >> 1) & 1u;
        float radius = std::sqrt(neg2ln_uniform(w[2 * pair]));
        unit_circle_point(w[2 * pair + 1], &c01, &s01);
        return (j & 1u) ? radius * s01 : radius * c01;
    }
    uint32_t word[3];
    for (uint32_t m = 0; m < 3; ++m) {
        uint32_t at = 3u * (j & 3u) + m;                   // position among the quad's twelve words
        uint32_t ctr[4] = {3u * (j >> 2) + (at >> 2), worker, (uint32_t)t, (uint32_t)(t >> 32)};
        philox4x32_10(ctr, key, w);
        word[m] = w[at & 3u];
    }
    float r2 = neg2ln_uniform(word[0]);
    unit_circle_point(word[1], &c01, &s01);
    float chi2_2 = neg2ln_uniform(word[2]);
    float chi2_3 = std::fmaf(r2, s01 * s01, chi2_2);
    if (chi2_3 == 0.0f) return 0.0f;
    float ratio = (3.0f * r2) / chi2_3;
    return c01 * std::sqrt(ratio);
}

// ---------------------------------------------------------------------------------
// Top-k under the total order (|v| descending, index ascending); |v| compared on the
// bit pattern with the sign cleared, so +0 and -0 tie and denormals order correctly.
// Writes the chosen indices in ascending order.  T = smallest chosen magnitude key,
// r = how many chosen entries carry exactly that key.
// ---------------------------------------------------------------------------------
void topk_select(const float* p, uint64_t d, uint64_t k, uint32_t* idx_out,
                 uint32_t* T_out, uint64_t* r_out) {
    std::vector<uint32_t> order(d);
    for (uint64_t j = 0; j < d; ++j) order[j] = (uint32_t)j;
    auto before = [p](uint32_t a, uint32_t b) {
        uint32_t ka = magnitude_key(p[a]), kb = magnitude_key(p[b]);
        if (ka != kb) return ka > kb;
        return a < b;
    };
    if (k < d) std::nth_element(order.begin(), order.begin() + k, order.end(), before);
    std::sort(order.begin(), order.begin() + k);
    uint32_t T = 0xffffffffu;
    for (uint64_t m = 0; m < k; ++m) T = std::min(T, magnitude_key(p[order[m]]));
    uint64_t r = 0;
    for (uint64_t m = 0; m < k; ++m) {
        idx_out[m] = order[m];
        if (magnitude_key(p[order[m]]) == T) ++r;
    }
    if (T_out) *T_out = T;
    if (r_out) *r_out = r;
}

// ---------------------------------------------------------------------------------
// Random-k: the k coordinates pi(0), ..., pi(k-1) of a keyed pseudo-random permutation pi
// of [0, d).  pi is a 4-round Feistel network on 2w bits (w = smallest with 4^w >= d) whose
// round function is the MurmurHash3 32-bit finaliser of (half XOR round key), cut to w
// bits, walked until the value falls below d (cycle walking keeps it a bijection of
// [0, d)).  Round keys: the Philox block with counter (0xFFFFFFFF, worker, t) under the
// seed -- a counter word no noise draw uses, since coordinates stay below 2^32 - 8192.
// ---------------------------------------------------------------------------------
uint32_t murmur_fmix32(uint32_t h) {
    h ^= h >> 16; h *= 0x85ebca6bu; h ^= h >> 13; h *= 0xc2b2ae35u; h ^= h >> 16;
    return h;
}

struct RandkKey { uint32_t round_key[4]; uint32_t w; uint64_t d; };

RandkKey randk_key(uint64_t seed, uint64_t t, uint32_t worker, uint64_t d) {
    RandkKey key;
    uint32_t ctr[4] = {0xffffffffu, worker, (uint32_t)t, (uint32_t)(t >> 32)};
    uint32_t sk[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    philox4x32_10(ctr, sk, key.round_key);
    key.w = 1;
    while (((uint64_t)1 << (2 * key.w)) < d) ++key.w;
    key.d = d;
    return key;
}

uint64_t feistel_forward(const RandkKey& key, uint64_t x) {
    const uint32_t mask = (uint32_t)(((uint64_t)1 << key.w) - 1);
    uint32_t left = (uint32_t)(x >> key.w), right = (uint32_t)x & mask;
    for (int r = 0; r < 4; ++r) {
        uint32_t f = murmur_fmix32(right ^ key.round_key[r]) & mask;
        uint32_t new_right = left ^ f;
        left = right;
        right = new_right;
    }
    return ((uint64_t)left << key.w) | right;
}

uint64_t randk_permute(const RandkKey& key, uint64_t m) {
    uint64_t y = feistel_forward(key, m);
    while (y >= key.d) y = feistel_forward(key, y);
    return y;
}

// the chosen coordinates in ascending order
void randk_select(uint64_t seed, uint64_t t, uint32_t worker, uint64_t d, uint64_t k, uint32_t* idx_out) {
    RandkKey key = randk_key(seed, t, worker, d);
    for (uint64_t m = 0; m < k; ++m) idx_out[m] = (uint32_t)randk_permute(key, m);
    std::sort(idx_out, idx_out + k);
}

// ---------------------------------------------------------------------------------
// 4-bit quantiser of a message (composed compressor, third stage).  The paper names the stage
// and nothing else, so this is a reading: the values, in message order (ascending coordinate),
// are cut into blocks of 256; a block's step is (largest magnitude in the block) / 7, a value's
// code the integer nearest to value / step (halves to the even one) kept inside [-7, 7], and
// the receiver's value is code * step.  A block whose step comes out as zero (all values zero,
// or so tiny that max/7 rounds to zero) sends only zero codes.  Two codes share a byte: the
// even position in the low nibble, two's complement.
// codes: (count+1)/2 bytes, steps: (count+255)/256 floats, deq: count floats.
// ---------------------------------------------------------------------------------
constexpr uint64_t kQuantBlock = 256;

void quantize4(const float* v, uint64_t count, uint8_t* codes, float* steps, float* deq) {
    for (uint64_t m = 0; m < (count + 1) / 2; ++m) codes[m] = 0;
    for (uint64_t b0 = 0; b0 < count; b0 += kQuantBlock) {
        const uint64_t b1 = std::min(count, b0 + kQuantBlock);
        float largest = 0.0f;
        for (uint64_t m = b0; m < b1; ++m) largest = std::max(largest, std::fabs(v[m]));
        const float step = largest / 7.0f;
        steps[b0 / kQuantBlock] = step;
        for (uint64_t m = b0; m < b1; ++m) {
            int q = 0;
            if (step > 0.0f) {
                float ratio = v[m] / step;
                float nearest = std::nearbyint(ratio);          // default rounding mode: halves to even
                if (nearest > 7.0f) nearest = 7.0f;
                if (nearest < -7.0f) nearest = -7.0f;
                q = (int)nearest;
            }
            deq[m] = (float)q * step;
            codes[m / 2] |= (uint8_t)((q & 0xf) << ((m & 1) * 4));
        }
    }
}

uint64_t k_from_delta(double delta, uint64_t d) {
    double kd = std::ceil(delta * (double)d);
    if (kd < 1.0) kd = 1.0;
    if (kd > (double)d) kd = (double)d;
    return (uint64_t)kd;
}

// ---------------------------------------------------------------------------------
// Normative state: ring of snapshots, one error buffer per worker.
// ---------------------------------------------------------------------------------
struct Oracle {
    uint64_t d = 0;
    uint32_t n = 0, tau_max = 0, tau = 0;
    uint64_t t = 0;
    uint64_t seed = 0;
    int noise_kind = 0;
    float noise_scale = 0.0f;
    int threads = 1;
    int compressor = 0;                 // 0: Top-k, 1: Random-k, 2: composed (Random-k, Top-k inside, 4-bit)
    double rand_ratio = 0.2;            // composed: share of the coordinates the Random-k stage keeps
    std::vector<std::vector<uint8_t>> msg_codes;   // composed: the 4-bit codes and block steps of the last message
    std::vector<std::vector<float>> msg_steps;
    float zeta = 0.0f;                  // non-IID: worker i's optimum is x* + zeta * u_i
    bool step_is_noop = false;
    std::vector<float> lambda, xstar, U;
    std::vector<std::vector<float>> ring, e, g;
    std::vector<std::vector<uint32_t>> msg_idx;
    std::vector<std::vector<float>> msg_val;
    std::vector<uint32_t> thr_T;
    std::vector<uint64_t> thr_r;

    std::vector<float>& slot(uint64_t step) { return ring[step % (tau_max + 1)]; }
};

template <class F>
void for_each_worker(Oracle* o, F fn) {
    if (o->threads <= 1 || o->n == 1) {
        for (uint32_t i = 0; i < o->n; ++i) fn(i);
        return;
    }
    std::vector<std::thread> pool;
    uint32_t nt = std::min<uint32_t>((uint32_t)o->threads, o->n);
    for (uint32_t w = 0; w < nt; ++w)
        pool.emplace_back([=]() { for (uint32_t i = w; i < o->n; i += nt) fn(i); });
    for (auto& th : pool) th.join();
}

constexpr uint64_t kHeterogeneityKey = 0xfffffffffffffffeull;

// Worker i's gradient at the coordinates [j0, j1) (every coordinate is computed on its own).
void grad_worker(Oracle* o, uint32_t i, uint64_t j0, uint64_t j1) {
    const std::vector<float>& xs = o->slot(o->t - o->tau);
    std::vector<float>& g = o->g[i];
    for (uint64_t j = j0; j < j1; ++j) {
        // heterogeneous local objectives (Assumption 3): f_i has its own optimum, shifted from x*
        // by zeta times a fixed standard normal vector u_i (drawn under a step key no iteration uses)
        float optimum = o->xstar[j];
        if (o->zeta != 0.0f) optimum = o->xstar[j] + o->zeta * noise_z(o->seed, kHeterogeneityKey, i, (uint32_t)j, 1);
        float diff = xs[j] - optimum;
        float mean = o->lambda[j] * diff;
        float xi = o->noise_scale * noise_z(o->seed, o->t, i, (uint32_t)j, o->noise_kind);
        g[j] = mean + xi;
    }
}

void compress_worker(Oracle* o, uint32_t i, uint64_t k, float lr) {
    const uint64_t d = o->d;
    std::vector<float> p(d);
    for (uint64_t j = 0; j < d; ++j) {
        float scaled = lr * o->g[i][j];
        p[j] = o->e[i][j] + scaled;
    }
    o->msg_idx[i].assign(k, 0u);
    o->msg_val[i].assign(k, 0.0f);
    if (o->compressor == 1) {
        randk_select(o->seed, o->t, i, d, k, o->msg_idx[i].data());
        o->thr_T[i] = 0; o->thr_r[i] = 0;
    } else {
        topk_select(p.data(), d, k, o->msg_idx[i].data(), &o->thr_T[i], &o->thr_r[i]);
    }
    std::vector<float> dense(d, 0.0f);                  // Delta as a dense vector
    for (uint64_t m = 0; m < k; ++m) {
        uint32_t j = o->msg_idx[i][m];
        o->msg_val[i][m] = p[j];
        dense[j] = p[j];
    }
    for (uint64_t j = 0; j < d; ++j) o->e[i][j] = p[j] - dense[j];
}

// Composed compressor: Random-k keeps k1 = ceil(rand_ratio * d) coordinates, Top-k keeps the
// k = ceil(delta * k1) largest of those (same total order; among the kept coordinates a lower
// coordinate wins a tie), the 4-bit quantiser codes their values.  Delta is what the receiver
// decodes, so the quantisation error stays in the error buffer with everything not sent.
void compress_worker_composed(Oracle* o, uint32_t i, double delta, float lr) {
    const uint64_t d = o->d;
    std::vector<float> p(d);
    for (uint64_t j = 0; j < d; ++j) {
        float scaled = lr * o->g[i][j];
        p[j] = o->e[i][j] + scaled;
    }
    const uint64_t k1 = k_from_delta(o->rand_ratio, d);
    const uint64_t k = k_from_delta(delta, k1);
    std::vector<uint32_t> subset(k1);
    randk_select(o->seed, o->t, i, d, k1, subset.data());          // ascending coordinates
    std::vector<float> kept(k1);
    for (uint64_t m = 0; m < k1; ++m) kept[m] = p[subset[m]];
    std::vector<uint32_t> pos(k);
    topk_select(kept.data(), k1, k, pos.data(), &o->thr_T[i], &o->thr_r[i]);
    o->msg_idx[i].assign(k, 0u);
    o->msg_val[i].assign(k, 0.0f);
    std::vector<float> chosen(k);
    for (uint64_t m = 0; m < k; ++m) {
        o->msg_idx[i][m] = subset[pos[m]];
        chosen[m] = kept[pos[m]];
    }
    o->msg_codes[i].assign((k + 1) / 2, 0);
    o->msg_steps[i].assign((k + kQuantBlock - 1) / kQuantBlock, 0.0f);
    quantize4(chosen.data(), k, o->msg_codes[i].data(), o->msg_steps[i].data(), o->msg_val[i].data());
    std::vector<float> dense(d, 0.0f);
    for (uint64_t m = 0; m < k; ++m) dense[o->msg_idx[i][m]] = o->msg_val[i][m];
    for (uint64_t j = 0; j < d; ++j) o->e[i][j] = p[j] - dense[j];
}

// DeCo's objective and the timing model (double precision, host scalars).
double phi_value(double delta, double tau) {
    return (1.0 - delta) / (delta * std::pow(1.0 - 0.5 * delta, tau));
}

}  // namespace

extern "C" {

void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    philox4x32_10(ctr, key, out);
}
float oracle_neg2ln_uniform(uint32_t w) { return neg2ln_uniform(w); }
void oracle_unit_circle_point(uint32_t w, float* c, float* s) { unit_circle_point(w, c, s); }
float oracle_noise_z(uint64_t seed, uint64_t t, uint32_t worker, uint32_t j, int kind) {
    return noise_z(seed, t, worker, j, kind);
}
void oracle_noise_fill(uint64_t seed, uint64_t t, uint32_t worker, uint64_t j0, uint64_t count,
                       int kind, float* out) {
    for (uint64_t m = 0; m < count; ++m) out[m] = noise_z(seed, t, worker, (uint32_t)(j0 + m), kind);
}
uint64_t oracle_k_from_delta(double delta, uint64_t d) { return k_from_delta(delta, d); }
void oracle_topk(const float* p, uint64_t d, uint64_t k, uint32_t* idx_out, uint32_t* T_out,
                 uint64_t* r_out) {
    topk_select(p, d, k, idx_out, T_out, r_out);
}

void oracle_randk_indices(uint64_t seed, uint64_t t, uint32_t worker, uint64_t d, uint64_t k, uint32_t* idx_out) {
    randk_select(seed, t, worker, d, k, idx_out);
}
uint64_t oracle_randk_permute(uint64_t seed, uint64_t t, uint32_t worker, uint64_t d, uint64_t m) {
    return randk_permute(randk_key(seed, t, worker, d), m);
}
uint32_t oracle_murmur_fmix32(uint32_t h) { return murmur_fmix32(h); }
void oracle_set_compressor(void* h, int kind) { ((Oracle*)h)->compressor = kind; }
void oracle_set_composed(void* h, double rand_ratio) { ((Oracle*)h)->rand_ratio = rand_ratio; }
void oracle_quantize4(const float* v, uint64_t count, uint8_t* codes, float* steps, float* deq) {
    quantize4(v, count, codes, steps, deq);
}
void oracle_set_heterogeneity(void* h, float zeta) { ((Oracle*)h)->zeta = zeta; }

void* oracle_create(uint64_t d, uint32_t n, uint32_t tau_max) {
    Oracle* o = new Oracle;
    o->d = d; o->n = n; o->tau_max = tau_max; o->tau = tau_max;
    o->lambda.assign(d, 0.0f);
    o->xstar.assign(d, 0.0f);
    o->U.assign(d, 0.0f);
    o->ring.assign(tau_max + 1, std::vector<float>(d, 0.0f));
    o->e.assign(n, std::vector<float>(d, 0.0f));
    o->g.assign(n, std::vector<float>(d, 0.0f));
    o->msg_idx.assign(n, {});
    o->msg_val.assign(n, {});
    o->msg_codes.assign(n, {});
    o->msg_steps.assign(n, {});
    o->thr_T.assign(n, 0u);
    o->thr_r.assign(n, 0u);
    return o;
}
void oracle_destroy(void* h) { delete (Oracle*)h; }
void oracle_set_threads(void* h, int threads) { ((Oracle*)h)->threads = threads; }

void oracle_set_problem(void* h, const float* lambda, const float* xstar, const float* x0,
                        uint64_t seed, int noise_kind, float noise_scale) {
    Oracle* o = (Oracle*)h;
    std::copy(lambda, lambda + o->d, o->lambda.begin());
    std::copy(xstar, xstar + o->d, o->xstar.begin());
    for (auto& s : o->ring) std::copy(x0, x0 + o->d, s.begin());
    for (auto& e : o->e) std::fill(e.begin(), e.end(), 0.0f);
    o->seed = seed; o->noise_kind = noise_kind; o->noise_scale = noise_scale;
    o->t = 0;
}
void oracle_set_tau(void* h, uint32_t tau) { ((Oracle*)h)->tau = tau; }
uint64_t oracle_step_index(void* h) { return ((Oracle*)h)->t; }

// Gradient at the stale iterate.  While t - tau < 0 there is nothing to apply yet
// (Delta_{t-tau} := 0), the step is a no-op and no gradient is produced.
void oracle_grad(void* h) {
    Oracle* o = (Oracle*)h;
    o->step_is_noop = o->t < o->tau;
    if (o->step_is_noop) return;
    if (o->threads > (int)o->n) {
        // more threads than workers (one worker of a very long vector): the threads share each
        // worker's coordinates in contiguous ranges instead
        const uint64_t nt = (uint64_t)o->threads, per = (o->d + nt - 1) / nt;
        for (uint32_t i = 0; i < o->n; ++i) {
            std::vector<std::thread> pool;
            for (uint64_t j0 = 0; j0 < o->d; j0 += per)
                pool.emplace_back([=]() { grad_worker(o, i, j0, std::min(o->d, j0 + per)); });
            for (auto& th : pool) th.join();
        }
        return;
    }
    for_each_worker(o, [o](uint32_t i) { grad_worker(o, i, 0, o->d); });
}
// Replace worker i's gradient by a given vector (unit tests); marks the step as real.
void oracle_load_grad(void* h, uint32_t worker, const float* g) {
    Oracle* o = (Oracle*)h;
    o->step_is_noop = false;
    std::copy(g, g + o->d, o->g[worker].begin());
}
void oracle_ef_compress(void* h, double delta, float lr) {
    Oracle* o = (Oracle*)h;
    if (o->step_is_noop) {
        for (uint32_t i = 0; i < o->n; ++i) { o->msg_idx[i].clear(); o->msg_val[i].clear(); }
        return;
    }
    if (o->compressor == 2) {
        for_each_worker(o, [o, delta, lr](uint32_t i) { compress_worker_composed(o, i, delta, lr); });
        return;
    }
    uint64_t k = k_from_delta(delta, o->d);
    for_each_worker(o, [o, k, lr](uint32_t i) { compress_worker(o, i, k, lr); });
}
void oracle_aggregate(void* h) {
    Oracle* o = (Oracle*)h;
    std::fill(o->U.begin(), o->U.end(), 0.0f);
    for (uint32_t i = 0; i < o->n; ++i)
        for (size_t m = 0; m < o->msg_idx[i].size(); ++m)
            o->U[o->msg_idx[i][m]] = o->U[o->msg_idx[i][m]] + o->msg_val[i][m];
}
void oracle_apply_delayed(void* h) {
    Oracle* o = (Oracle*)h;
    const std::vector<float>& x = o->slot(o->t);
    std::vector<float>& xn = o->slot(o->t + 1);
    float nf = (float)o->n;
    for (uint64_t j = 0; j < o->d; ++j) {
        float avg = o->U[j] / nf;
        xn[j] = x[j] - avg;
    }
    o->t += 1;
}
void oracle_step(void* h, double delta, float lr) {
    oracle_grad(h);
    oracle_ef_compress(h, delta, lr);
    oracle_aggregate(h);
    oracle_apply_delayed(h);
}

// The objective the method minimises (Section 2.1, problem (1)) at the current iterate:
// f(x_t) = (1/n) sum_i f_i(x_t) with the synthetic quadratics f_i(x) = 1/2 sum_j lambda_j (x_j - x*_ij)^2,
// x*_i = x* + zeta u_i as in the gradient.  Evaluated in double from the fp32 state.
double oracle_objective(void* h) {
    Oracle* o = (Oracle*)h;
    const std::vector<float>& x = o->slot(o->t);
    double total = 0.0;
    for (uint64_t j = 0; j < o->d; ++j) {
        double squares = 0.0;
        for (uint32_t i = 0; i < o->n; ++i) {
            float optimum = o->xstar[j];
            if (o->zeta != 0.0f) optimum = o->xstar[j] + o->zeta * noise_z(o->seed, kHeterogeneityKey, i, (uint32_t)j, 1);
            double diff = (double)x[j] - (double)optimum;
            squares += diff * diff;
        }
        total += (double)o->lambda[j] * (squares / (double)o->n);
    }
    return 0.5 * total;
}

void oracle_get_model(void* h, float* x) {
    Oracle* o = (Oracle*)h;
    const std::vector<float>& s = o->slot(o->t);
    std::copy(s.begin(), s.end(), x);
}
void oracle_set_model(void* h, const float* x) {
    Oracle* o = (Oracle*)h;
    std::copy(x, x + o->d, o->slot(o->t).begin());
}
void oracle_get_snapshot(void* h, uint64_t step, float* x) {
    Oracle* o = (Oracle*)h;
    const std::vector<float>& s = o->slot(step);
    std::copy(s.begin(), s.end(), x);
}
void oracle_get_error(void* h, uint32_t w, float* e) {
    Oracle* o = (Oracle*)h;
    std::copy(o->e[w].begin(), o->e[w].end(), e);
}
void oracle_set_error(void* h, uint32_t w, const float* e) {
    Oracle* o = (Oracle*)h;
    std::copy(e, e + o->d, o->e[w].begin());
}
void oracle_get_grad(void* h, uint32_t w, float* g) {
    Oracle* o = (Oracle*)h;
    std::copy(o->g[w].begin(), o->g[w].end(), g);
}
uint64_t oracle_message_size(void* h, uint32_t w) { return ((Oracle*)h)->msg_idx[w].size(); }
void oracle_get_message(void* h, uint32_t w, uint32_t* idx, float* val) {
    Oracle* o = (Oracle*)h;
    std::copy(o->msg_idx[w].begin(), o->msg_idx[w].end(), idx);
    std::copy(o->msg_val[w].begin(), o->msg_val[w].end(), val);
}
// composed compressor: the wire form of the last message ((k+1)/2 code bytes, (k+255)/256 steps)
void oracle_get_message_codes(void* h, uint32_t w, uint8_t* codes, float* steps) {
    Oracle* o = (Oracle*)h;
    std::copy(o->msg_codes[w].begin(), o->msg_codes[w].end(), codes);
    std::copy(o->msg_steps[w].begin(), o->msg_steps[w].end(), steps);
}
void oracle_get_update(void* h, float* U) {
    Oracle* o = (Oracle*)h;
    std::copy(o->U.begin(), o->U.end(), U);
}
void oracle_get_threshold(void* h, uint32_t w, uint32_t* T, uint64_t* r) {
    Oracle* o = (Oracle*)h;
    *T = o->thr_T[w]; *r = o->thr_r[w];
}

// Algorithm 1 as printed: every worker takes its gradient at the current x_u, compresses,
// and sends; the server applies the message sent tau iterations earlier.  The gradient
// taken at time u is consumed at server step u + tau, which is the step index the noise
// draw is keyed by, so that this form and the ring form see the same random numbers.
// x_traj receives x_0 .. x_T ((T+1)*d floats) when not null; x_final receives x_T.
void oracle_queue_run(uint64_t d, uint32_t n, uint32_t tau, uint64_t T, double delta, float lr,
                      const float* lambda, const float* xstar, const float* x0, uint64_t seed,
                      int noise_kind, float noise_scale, float* x_traj, float* x_final) {
    uint64_t k = k_from_delta(delta, d);
    std::vector<float> x(x0, x0 + d), g(d), p(d), dense(d);
    std::vector<std::vector<float>> e(n, std::vector<float>(d, 0.0f));
    struct Msg { std::vector<uint32_t> idx; std::vector<float> val; };
    std::vector<std::vector<Msg>> sent(T, std::vector<Msg>(n));   // sent[u][i] = Delta_u^i
    if (x_traj) std::copy(x.begin(), x.end(), x_traj);
    float nf = (float)n;
    for (uint64_t u = 0; u < T; ++u) {
        for (uint32_t i = 0; i < n; ++i) {                         // worker side
            for (uint64_t j = 0; j < d; ++j) {
                float diff = x[j] - xstar[j];
                float mean = lambda[j] * diff;
                float xi = noise_scale * noise_z(seed, u + tau, i, (uint32_t)j, noise_kind);
                g[j] = mean + xi;
                float scaled = lr * g[j];
                p[j] = e[i][j] + scaled;
            }
            Msg& m = sent[u][i];
            m.idx.assign(k, 0u); m.val.assign(k, 0.0f);
            topk_select(p.data(), d, k, m.idx.data(), nullptr, nullptr);
            std::fill(dense.begin(), dense.end(), 0.0f);
            for (uint64_t q = 0; q < k; ++q) { m.val[q] = p[m.idx[q]]; dense[m.idx[q]] = p[m.idx[q]]; }
            for (uint64_t j = 0; j < d; ++j) e[i][j] = p[j] - dense[j];
        }
        std::vector<float> U(d, 0.0f);                             // server side
        if (u >= tau) {
            for (uint32_t i = 0; i < n; ++i) {
                const Msg& m = sent[u - tau][i];
                for (uint64_t q = 0; q < k; ++q) U[m.idx[q]] = U[m.idx[q]] + m.val[q];
            }
        }
        for (uint64_t j = 0; j < d; ++j) { float avg = U[j] / nf; x[j] = x[j] - avg; }
        if (x_traj) std::copy(x.begin(), x.end(), x_traj + (u + 1) * d);
    }
    if (x_final) std::copy(x.begin(), x.end(), x_final);
}

// The same literal form, one iteration at a time, so that its error buffers and messages can be
// inspected: state = x_u, e_i (already advanced to time u), and the messages sent so far.
struct QueueOracle {
    uint64_t d = 0, u = 0, seed = 0;
    // Noise key of the gradient taken at iteration u: the iteration u + tau_u at which its message
    // is due, moved up where needed so that the keys increase strictly (a falling tau would
    // otherwise name the same iteration twice and draw the same noise twice):
    // key_u = max(u + tau_u, key_{u-1} + 1).  For a constant tau this is u + tau.
    uint64_t next_key_floor = 0;
    uint32_t n = 0, tau = 0;
    int noise_kind = 0;
    float noise_scale = 0.0f;
    float zeta = 0.0f;                  // non-IID: worker i's optimum is x* + zeta * u_i
    std::vector<float> lambda, xstar, x, U;
    std::vector<std::vector<float>> e;
    std::vector<std::vector<std::vector<uint32_t>>> sent_idx;   // [iteration][worker]
    std::vector<std::vector<std::vector<float>>> sent_val;
};

void* oracle_queue_create(uint64_t d, uint32_t n, uint32_t tau) {
    QueueOracle* q = new QueueOracle;
    q->d = d; q->n = n; q->tau = tau;
    q->lambda.assign(d, 0.0f); q->xstar.assign(d, 0.0f); q->x.assign(d, 0.0f); q->U.assign(d, 0.0f);
    q->e.assign(n, std::vector<float>(d, 0.0f));
    return q;
}
void oracle_queue_destroy(void* h) { delete (QueueOracle*)h; }
// tau may change between iterations: the server applies what was sent tau iterations earlier
void oracle_queue_set_tau(void* h, uint32_t tau) { ((QueueOracle*)h)->tau = tau; }
void oracle_queue_set_heterogeneity(void* h, float zeta) { ((QueueOracle*)h)->zeta = zeta; }
void oracle_queue_set_problem(void* h, const float* lambda, const float* xstar, const float* x0, uint64_t seed,
                              int noise_kind, float noise_scale) {
    QueueOracle* q = (QueueOracle*)h;
    std::copy(lambda, lambda + q->d, q->lambda.begin());
    std::copy(xstar, xstar + q->d, q->xstar.begin());
    std::copy(x0, x0 + q->d, q->x.begin());
    for (auto& e : q->e) std::fill(e.begin(), e.end(), 0.0f);
    q->sent_idx.clear(); q->sent_val.clear();
    q->seed = seed; q->noise_kind = noise_kind; q->noise_scale = noise_scale; q->u = 0;
    q->next_key_floor = 0;
}
void oracle_queue_step(void* h, double delta, float lr) {
    QueueOracle* q = (QueueOracle*)h;
    const uint64_t d = q->d, k = k_from_delta(delta, d), u = q->u;
    q->sent_idx.emplace_back(q->n); q->sent_val.emplace_back(q->n);
    const uint64_t key = std::max(u + q->tau, q->next_key_floor);
    q->next_key_floor = key + 1;
    std::vector<float> p(d), dense(d);
    for (uint32_t i = 0; i < q->n; ++i) {                          // worker side, at the current x_u
        for (uint64_t j = 0; j < d; ++j) {
            float optimum = q->xstar[j];
            if (q->zeta != 0.0f) optimum = q->xstar[j] + q->zeta * noise_z(q->seed, kHeterogeneityKey, i, (uint32_t)j, 1);
            float diff = q->x[j] - optimum;
            float mean = q->lambda[j] * diff;
            float xi = q->noise_scale * noise_z(q->seed, key, i, (uint32_t)j, q->noise_kind);
            float g = mean + xi;
            float scaled = lr * g;
            p[j] = q->e[i][j] + scaled;
        }
        std::vector<uint32_t>& idx = q->sent_idx[u][i];
        std::vector<float>& val = q->sent_val[u][i];
        idx.assign(k, 0u); val.assign(k, 0.0f);
        topk_select(p.data(), d, k, idx.data(), nullptr, nullptr);
        std::fill(dense.begin(), dense.end(), 0.0f);
        for (uint64_t m = 0; m < k; ++m) { val[m] = p[idx[m]]; dense[idx[m]] = p[idx[m]]; }
        for (uint64_t j = 0; j < d; ++j) q->e[i][j] = p[j] - dense[j];
    }
    std::fill(q->U.begin(), q->U.end(), 0.0f);                      // server side: the message of u - tau
    if (u >= q->tau)
        for (uint32_t i = 0; i < q->n; ++i) {
            const std::vector<uint32_t>& idx = q->sent_idx[u - q->tau][i];
            const std::vector<float>& val = q->sent_val[u - q->tau][i];
            for (size_t m = 0; m < idx.size(); ++m) q->U[idx[m]] = q->U[idx[m]] + val[m];
        }
    float nf = (float)q->n;
    for (uint64_t j = 0; j < d; ++j) { float avg = q->U[j] / nf; q->x[j] = q->x[j] - avg; }
    q->u += 1;
}
void oracle_queue_get_model(void* h, float* x) { QueueOracle* q = (QueueOracle*)h; std::copy(q->x.begin(), q->x.end(), x); }
void oracle_queue_get_update(void* h, float* U) { QueueOracle* q = (QueueOracle*)h; std::copy(q->U.begin(), q->U.end(), U); }
void oracle_queue_get_error(void* h, uint32_t w, float* e) {
    QueueOracle* q = (QueueOracle*)h;
    std::copy(q->e[w].begin(), q->e[w].end(), e);
}
uint64_t oracle_queue_message_size(void* h, uint32_t w) {
    QueueOracle* q = (QueueOracle*)h;
    return q->u == 0 ? 0 : q->sent_idx[q->u - 1][w].size();
}
// the message worker w sent in the last iteration
void oracle_queue_get_message(void* h, uint32_t w, uint32_t* idx, float* val) {
    QueueOracle* q = (QueueOracle*)h;
    if (q->u == 0) return;
    std::copy(q->sent_idx[q->u - 1][w].begin(), q->sent_idx[q->u - 1][w].end(), idx);
    std::copy(q->sent_val[q->u - 1][w].begin(), q->sent_val[q->u - 1][w].end(), val);
}

// ---- DeCo (Algorithm 3) and the timing model (Section 4, Theorem 3) ----------------
double oracle_phi(double delta, double tau) { return phi_value(delta, tau); }

// Key factor of the non-IID analysis (Remark on phi): phi' = (1-delta) / (delta^2 (1-delta/2)^tau).
double oracle_phi_prime(double delta, double tau) {
    return (1.0 - delta) / (delta * delta * std::pow(1.0 - 0.5 * delta, tau));
}

// delta*(tau) of the Remark following Theorem 3.
double oracle_delta_star(double tau, double v_g, double a, double b, double t_comp) {
    double first = std::max(0.0, (tau * t_comp - b) * a / v_g);
    return std::min(std::min(first, t_comp * a / v_g), 1.0);
}

// Scan tau from ceil((b + V_g/a)/T_comp) down to ceil(b/T_comp); delta = delta*(tau);
// candidates with delta <= 0 have no phi and are skipped; "<=" keeps the smallest tau
// among equal phi.  Returns 0 when a candidate was found, -1 otherwise.
int oracle_deco(double v_g, double a, double b, double t_comp, uint32_t* tau_out, double* delta_out) {
    long hi = (long)std::ceil((b + v_g / a) / t_comp);
    long lo = (long)std::ceil(b / t_comp);
    double best = std::numeric_limits<double>::infinity();
    int found = -1;
    for (long tau = hi; tau >= lo; --tau) {
        double delta = std::min(std::min((tau * t_comp - b) * a / v_g, t_comp * a / v_g), 1.0);
        if (!(delta > 0.0)) continue;
        double phi = phi_value(delta, (double)tau);
        if (phi <= best) { best = phi; *tau_out = (uint32_t)tau; *delta_out = delta; found = 0; }
    }
    return found;
}

// The same scan with phi' as the objective (Section 5.6: "In non-IID scenarios, we replace phi").
int oracle_deco_noniid(double v_g, double a, double b, double t_comp, uint32_t* tau_out, double* delta_out) {
    long hi = (long)std::ceil((b + v_g / a) / t_comp);
    long lo = (long)std::ceil(b / t_comp);
    double best = std::numeric_limits<double>::infinity();
    int found = -1;
    for (long tau = hi; tau >= lo; --tau) {
        double delta = std::min(std::min((tau * t_comp - b) * a / v_g, t_comp * a / v_g), 1.0);
        if (!(delta > 0.0)) continue;
        double obj = oracle_phi_prime(delta, (double)tau);
        if (obj <= best) { best = obj; *tau_out = (uint32_t)tau; *delta_out = delta; found = 0; }
    }
    return found;
}

double oracle_t_avg_closed_form(double tau, double delta, double v_g, double a, double b, double t_comp) {
    double xfer = delta * v_g / a;
    return std::max(std::max((t_comp + b + xfer) / (tau + 1.0), xfer), t_comp);
}

// TC_E / E (the quantity the theorem's error bound is stated for) from the recurrence
// in the proof of Theorem 3:
//   TC_k = TM_k + b;  TS_{k+1} = T_comp + max(TC_{k-tau}, TS_k);
//   TM_{k+1} = delta*V_g/a + max(TM_k, TS_{k+1});  TS_0 = TM_0 = 0, TC_k = 0 for k <= 0.
double oracle_t_avg_recurrence(uint32_t tau, double delta, double v_g, double a, double b,
                               double t_comp, uint64_t E) {
    std::vector<double> TS(E + 1, 0.0), TM(E + 1, 0.0);
    double xfer = delta * v_g / a;
    for (uint64_t k = 0; k < E; ++k) {
        double tc_old = 0.0;
        if (k >= tau && k - tau >= 1) tc_old = TM[k - tau] + b;
        TS[k + 1] = t_comp + std::max(tc_old, TS[k]);
        TM[k + 1] = xfer + std::max(TM[k], TS[k + 1]);
    }
    return (TM[E] + b) / (double)E;
}

}  // extern "C"
