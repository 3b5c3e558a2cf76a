// Short runs of every part of the CPU oracle (oracle/ddef_oracle.cpp) for a build with
// AddressSanitizer and UBSan: the step in all three compressors, tiny and ragged sizes, more
// threads than workers, the literal queue form with a changing tau, the 4-bit coder, DeCo and the
// timing recurrence.  Exit status 0 and a clean sanitizer report are the test; values are pinned
// elsewhere (tests/test_oracle_*.py).
#include <cstdint>
#include <cstdio>
#include <initializer_list>
#include <vector>

extern "C" {
void* oracle_create(uint64_t d, uint32_t n, uint32_t tau_max);
void oracle_destroy(void*);
void oracle_set_threads(void*, int);
void oracle_set_problem(void*, const float*, const float*, const float*, uint64_t, int, float);
void oracle_set_tau(void*, uint32_t);
void oracle_set_compressor(void*, int);
void oracle_set_composed(void*, double);
void oracle_set_heterogeneity(void*, float);
void oracle_step(void*, double, float);
double oracle_objective(void*);
void oracle_get_model(void*, float*);
void oracle_get_error(void*, uint32_t, float*);
void oracle_get_update(void*, float*);
uint64_t oracle_message_size(void*, uint32_t);
void oracle_get_message(void*, uint32_t, uint32_t*, float*);
void oracle_get_message_codes(void*, uint32_t, uint8_t*, float*);
void oracle_get_threshold(void*, uint32_t, uint32_t*, uint64_t*);
void oracle_quantize4(const float*, uint64_t, uint8_t*, float*, float*);
void oracle_topk(const float*, uint64_t, uint64_t, uint32_t*, uint32_t*, uint64_t*);
void oracle_randk_indices(uint64_t, uint64_t, uint32_t, uint64_t, uint64_t, uint32_t*);
void oracle_noise_fill(uint64_t, uint64_t, uint32_t, uint64_t, uint64_t, int, float*);
void oracle_queue_run(uint64_t, uint32_t, uint32_t, uint64_t, double, float, const float*, const float*, const float*,
                      uint64_t, int, float, float*, float*);
void* oracle_queue_create(uint64_t d, uint32_t n, uint32_t tau);
void oracle_queue_destroy(void*);
void oracle_queue_set_problem(void*, const float*, const float*, const float*, uint64_t, int, float);
void oracle_queue_set_tau(void*, uint32_t);
void oracle_queue_step(void*, double, float);
void oracle_queue_get_model(void*, float*);
uint64_t oracle_queue_message_size(void*, uint32_t);
void oracle_queue_get_message(void*, uint32_t, uint32_t*, float*);
int oracle_deco(double, double, double, double, uint32_t*, double*);
int oracle_deco_noniid(double, double, double, double, uint32_t*, double*);
double oracle_t_avg_recurrence(uint32_t, double, double, double, double, double, uint64_t);
double oracle_t_avg_closed_form(double, double, double, double, double, double);
}

static std::vector<float> ramp(uint64_t d, float a) {
    std::vector<float> v(d);
    for (uint64_t j = 0; j < d; ++j) v[j] = a + 0.01f * (float)((j * 37u) % 101u);
    return v;
}

int main() {
    for (uint64_t d : {1ull, 2ull, 3ull, 7ull, 33ull, 257ull, 4099ull})
        for (uint32_t n : {1u, 3u}) for (int kind : {0, 1, 2}) for (int comp : {0, 1, 2}) {
            const std::vector<float> lam = ramp(d, 0.1f), xs = ramp(d, -0.5f), x0 = ramp(d, 0.5f);
            void* o = oracle_create(d, n, 2);
            oracle_set_threads(o, (int)(d % 5u) + 1);             // fewer, as many and more threads than workers
            oracle_set_problem(o, lam.data(), xs.data(), x0.data(), 11, kind, 0.1f);
            oracle_set_compressor(o, comp);
            oracle_set_composed(o, 0.5);
            if (kind == 2) oracle_set_heterogeneity(o, 0.3f);
            const uint32_t taus[6] = {2, 2, 0, 1, 2, 0};
            const double deltas[6] = {0.1, 0.1, 1.0, 0.3, 0.01, 0.5};
            for (int it = 0; it < 6; ++it) {
                oracle_set_tau(o, taus[it]);
                oracle_step(o, deltas[it], 0.05f);
                std::vector<float> row(d);
                oracle_get_model(o, row.data());
                oracle_get_update(o, row.data());
                for (uint32_t w = 0; w < n; ++w) {
                    oracle_get_error(o, w, row.data());
                    const uint64_t k = oracle_message_size(o, w);
                    std::vector<uint32_t> idx(k);
                    std::vector<float> val(k);
                    oracle_get_message(o, w, idx.data(), val.data());
                    if (comp == 2 && k) {
                        std::vector<uint8_t> codes((k + 1) / 2);
                        std::vector<float> steps((k + 255) / 256);
                        oracle_get_message_codes(o, w, codes.data(), steps.data());
                    }
                    uint32_t T;
                    uint64_t r;
                    oracle_get_threshold(o, w, &T, &r);
                }
            }
            (void)oracle_objective(o);
            oracle_destroy(o);
        }
    for (uint64_t count : {1ull, 2ull, 255ull, 256ull, 257ull, 1000ull}) {
        const std::vector<float> v = ramp(count, -0.4f);
        std::vector<uint8_t> codes((count + 1) / 2);
        std::vector<float> steps((count + 255) / 256), deq(count);
        oracle_quantize4(v.data(), count, codes.data(), steps.data(), deq.data());
        std::vector<uint32_t> idx(count);
        uint32_t T;
        uint64_t r;
        for (uint64_t k : {(uint64_t)1, (count + 1) / 2, count}) oracle_topk(v.data(), count, k, idx.data(), &T, &r);
        oracle_randk_indices(3, 9, 1, count, (count + 1) / 2, idx.data());
        for (int kind : {1, 2}) oracle_noise_fill(5, 1ull << 40, 2, 0xfffffff0ull - count, count, kind, deq.data());
    }
    {
        const uint64_t d = 300;
        const std::vector<float> lam = ramp(d, 0.1f), xs = ramp(d, -0.5f), x0 = ramp(d, 0.5f);
        std::vector<float> traj((9 + 1) * d), last(d);
        oracle_queue_run(d, 2, 3, 9, 0.05, 0.05f, lam.data(), xs.data(), x0.data(), 4, 1, 0.1f, traj.data(), last.data());
        oracle_queue_run(d, 2, 0, 9, 1.0, 0.05f, lam.data(), xs.data(), x0.data(), 4, 2, 0.1f, nullptr, last.data());
        void* q = oracle_queue_create(d, 2, 0);
        oracle_queue_set_problem(q, lam.data(), xs.data(), x0.data(), 4, 1, 0.1f);
        const uint32_t taus[8] = {0, 3, 3, 1, 0, 2, 2, 5};
        for (int u = 0; u < 8; ++u) {
            oracle_queue_set_tau(q, taus[u]);
            oracle_queue_step(q, u % 2 ? 0.2 : 0.02, 0.05f);
            const uint64_t k = oracle_queue_message_size(q, 1);
            std::vector<uint32_t> idx(k);
            std::vector<float> val(k);
            oracle_queue_get_message(q, 1, idx.data(), val.data());
            oracle_queue_get_model(q, last.data());
        }
        oracle_queue_destroy(q);
    }
    for (double a : {5e7, 1e9, 1e10}) for (double b : {0.0, 0.05, 0.3}) {
        uint32_t tau = 0;
        double delta = 0.0;
        if (oracle_deco(32.0 * 124e6, a, b, 0.02, &tau, &delta) == 0) {
            (void)oracle_t_avg_recurrence(tau, delta, 32.0 * 124e6, a, b, 0.02, 200);
            (void)oracle_t_avg_recurrence(tau, delta, 32.0 * 124e6, a, b, 0.02, 1);
            (void)oracle_t_avg_closed_form(tau, delta, 32.0 * 124e6, a, b, 0.02);
        }
        (void)oracle_deco_noniid(32.0 * 124e6, a, b, 0.02, &tau, &delta);
    }
    std::printf("ok\n");
    return 0;
}
