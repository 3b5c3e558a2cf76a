// Host-only exercise of the C-ABI layer (csrc/ddef_api.hip built against the stand-in HIP runtime
// of this folder), meant to run under AddressSanitizer and UBSan: call-order state machine,
// argument checks, buffer sizes of every getter and setter, and what the lazy set-ups leave behind
// when an allocation, a stream or an event fails half-way.  No kernel runs, so nothing is said
// about results; exit status 0 and a clean sanitizer report are the test.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <initializer_list>
#include <vector>

#include "ddef.h"

static int failures = 0;
#define CHECK(cond)                                                                   \
    do {                                                                              \
        if (!(cond)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
    } while (0)

static std::vector<float> ramp(uint64_t d, float a) {
    std::vector<float> v(d);
    for (uint64_t j = 0; j < d; ++j) v[j] = a + 0.001f * (float)(j % 97);
    return v;
}

static void set_problem(ddef_ctx* c, uint64_t d) {
    const std::vector<float> lam = ramp(d, 0.5f), xs = ramp(d, -1.0f), x0 = ramp(d, 1.0f);
    CHECK(ddef_set_problem(c, lam.data(), xs.data(), x0.data(), 7, DDEF_NOISE_GAUSS, 0.1f) == DDEF_OK);
}

static int step(ddef_ctx* c, double delta, float lr) {
    int rc = ddef_grad(c);
    if (rc == DDEF_OK) rc = ddef_ef_compress(c, delta, lr);
    if (rc == DDEF_OK) rc = ddef_aggregate(c);
    if (rc == DDEF_OK) rc = ddef_apply_delayed(c, lr);
    return rc;
}

// every getter with buffers of exactly the documented size (a byte more read or written is a report)
static void read_everything(ddef_ctx* c, uint64_t d, uint32_t n, bool fused = false) {
    std::vector<float> row(d);
    CHECK(ddef_get_model(c, row.data()) == DDEF_OK);
    CHECK(ddef_get_update(c, row.data()) == DDEF_OK);
    for (uint32_t w = 0; w < n; ++w) {
        CHECK(ddef_get_error(c, w, row.data()) == DDEF_OK);
        // a fused gradient exists only while its iteration is in progress
        CHECK(ddef_get_grad(c, w, row.data()) == (fused ? DDEF_ESTATE : DDEF_OK));
        uint64_t k = 0;
        CHECK(ddef_get_message(c, w, nullptr, nullptr, &k) == DDEF_OK);
        std::vector<uint32_t> idx(k);
        std::vector<float> val(k);
        CHECK(ddef_get_message(c, w, idx.data(), val.data(), &k) == DDEF_OK);
        uint32_t T = 0, nb = 0, cand = 0, rowsearch = 0;
        uint64_t r = 0;
        if (k) {
            CHECK(ddef_get_threshold(c, w, &T, &r) == DDEF_OK);
            CHECK(ddef_get_filter_state(c, w, &nb, &cand, &rowsearch) == DDEF_OK);
        }
    }
    double f = 0.0;
    uint64_t count = 0, t = 0;
    CHECK(ddef_objective(c, &f) == DDEF_OK);
    CHECK(ddef_full_select_count(c, &count) == DDEF_OK);
    CHECK(ddef_step_index(c, &t) == DDEF_OK);
    CHECK(ddef_sync(c) == DDEF_OK);
}

static void plain_runs() {
    for (uint64_t d : {1ull, 5ull, 4096ull, 4097ull, 70001ull}) for (uint32_t n : {1u, 3u}) for (int queue : {0, 1}) {
        ddef_ctx* c = nullptr;
        CHECK((queue ? ddef_init_queue(d, n, 3, &c) : ddef_init(d, n, 3, &c)) == DDEF_OK);
        if (!c) continue;
        set_problem(c, d);
        CHECK(ddef_set_tau(c, 2) == DDEF_OK);
        for (int it = 0; it < 6; ++it) {
            const double delta = it < 3 ? 0.01 : 0.3;         // the message rows grow mid-run
            if (it == 4) CHECK(ddef_set_tau(c, 1) == DDEF_OK);
            CHECK(step(c, delta, 0.05f) == DDEF_OK);
            read_everything(c, d, n);
        }
        if (!queue) {
            for (int kind : {DDEF_COMPRESSOR_RANDK, DDEF_COMPRESSOR_COMPOSED, DDEF_COMPRESSOR_TOPK}) {
                CHECK(ddef_set_compressor(c, kind) == DDEF_OK);
                CHECK(step(c, 0.2, 0.05f) == DDEF_OK);
                read_everything(c, d, n);
                if (kind == DDEF_COMPRESSOR_COMPOSED) {
                    uint64_t k = 0;
                    CHECK(ddef_get_message_codes(c, 0, nullptr, nullptr, &k) == DDEF_OK);
                    std::vector<uint8_t> codes((k + 1) / 2);
                    std::vector<float> steps((k + 255) / 256);
                    CHECK(ddef_get_message_codes(c, 0, codes.data(), steps.data(), &k) == DDEF_OK);
                }
            }
            // checkpoint hooks
            std::vector<float> row(d);
            for (uint32_t age = 0; age <= 3; ++age) {
                CHECK(ddef_get_snapshot(c, age, row.data()) == DDEF_OK);
                CHECK(ddef_set_snapshot(c, age, row.data()) == DDEF_OK);
            }
            CHECK(ddef_get_snapshot(c, 4, row.data()) == DDEF_EINVAL);
            CHECK(ddef_set_step_index(c, 100) == DDEF_OK);
            CHECK(ddef_set_model(c, row.data()) == DDEF_OK);
            CHECK(ddef_set_error(c, n - 1, row.data()) == DDEF_OK);
            for (int opt : {DDEF_OPT_FUSE_GRAD, DDEF_OPT_GRAPH, DDEF_OPT_FORCE_FULL_SELECT}) {
                CHECK(ddef_set_option(c, opt, 1) == DDEF_OK);
                for (int it = 0; it < 4; ++it) CHECK(ddef_step(c, 0.01, 0.05f) == DDEF_OK);
                read_everything(c, d, n, opt == DDEF_OPT_FUSE_GRAD);
                CHECK(ddef_set_option(c, opt, 0) == DDEF_OK);
            }
            uint64_t bytes = 0;
            CHECK(ddef_copy_probe(c, &bytes) == DDEF_OK && bytes >= d * 4);
            CHECK(ddef_profile_enable(c, 1) == DDEF_OK);
            CHECK(step(c, 0.01, 0.05f) == DDEF_OK);
            for (int s = 0; s < ddef_profile_slots(); ++s) {
                const char* name = nullptr;
                uint64_t launches = 0;
                double ms = 0.0;
                CHECK(ddef_profile_read(c, s, &name, &launches, &ms) == DDEF_OK && name != nullptr);
            }
            CHECK(ddef_profile_enable(c, 0) == DDEF_OK);
        }
        char arch[8];
        uint32_t cus = 0;
        CHECK(ddef_device_info(c, &cus, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, arch, sizeof arch) == DDEF_OK);
        CHECK(ddef_destroy(c) == DDEF_OK);
    }
}

static void call_order_and_arguments() {
    ddef_ctx* c = nullptr;
    CHECK(ddef_init(0, 1, 0, &c) == DDEF_EINVAL && c == nullptr);
    CHECK(ddef_init(10, 0, 0, &c) == DDEF_EINVAL);
    CHECK(ddef_init(0xFFFFE000ull, 1, 0, &c) == DDEF_EINVAL);
    CHECK(ddef_init(10, 1, 5000, &c) == DDEF_EINVAL);
    CHECK(ddef_init(10, 1, 0, nullptr) == DDEF_EINVAL);
    CHECK(ddef_init(1000, 2, 2, &c) == DDEF_OK);
    CHECK(ddef_grad(c) == DDEF_ESTATE);                       // no problem yet
    set_problem(c, 1000);
    CHECK(ddef_ef_compress(c, 0.1, 0.05f) == DDEF_ESTATE);
    CHECK(ddef_aggregate(c) == DDEF_ESTATE);
    CHECK(ddef_apply_delayed(c, 0.05f) == DDEF_ESTATE);
    CHECK(ddef_set_tau(c, 3) == DDEF_EINVAL);
    CHECK(ddef_set_tau(c, 0) == DDEF_OK);
    CHECK(ddef_grad(c) == DDEF_OK);
    CHECK(ddef_grad(c) == DDEF_ESTATE);
    CHECK(ddef_set_tau(c, 1) == DDEF_ESTATE);
    CHECK(ddef_set_option(c, DDEF_OPT_FUSE_GRAD, 1) == DDEF_ESTATE);
    CHECK(ddef_ef_compress(c, 0.0, 0.05f) == DDEF_EINVAL);
    CHECK(ddef_ef_compress(c, 1.5, 0.05f) == DDEF_EINVAL);
    CHECK(ddef_ef_compress(c, 0.1, 0.05f) == DDEF_OK);
    CHECK(ddef_apply_delayed(c, 0.05f) == DDEF_ESTATE);
    CHECK(ddef_aggregate(c) == DDEF_OK);
    CHECK(ddef_apply_delayed(c, 0.06f) == DDEF_EINVAL);       // not the stepsize of this iteration
    CHECK(ddef_apply_delayed(c, 0.05f) == DDEF_OK);
    std::vector<float> row(1000);
    CHECK(ddef_get_error(c, 2, row.data()) == DDEF_EINVAL);
    CHECK(ddef_load_grad(c, 2, row.data()) == DDEF_EINVAL);
    CHECK(ddef_get_model(c, nullptr) == DDEF_EINVAL);
    CHECK(ddef_set_option(c, 99, 1) == DDEF_EINVAL);
    CHECK(ddef_set_option(c, DDEF_OPT_CANDIDATE_SLACK_X16, 3) == DDEF_EINVAL);
    CHECK(ddef_set_compressor(c, 7) == DDEF_EINVAL);
    CHECK(ddef_set_composed(c, 0.0) == DDEF_EINVAL);
    CHECK(ddef_destroy(c) == DDEF_OK);
    CHECK(ddef_destroy(nullptr) == DDEF_EINVAL);
    CHECK(ddef_grad(nullptr) == DDEF_EINVAL);
}

// ddef_init with its i-th allocation failing: ENOMEM, no handle, nothing left behind
static void init_failures() {
    for (long at = 0; at < 40; ++at) {
        const long live_before = fake_hip::state().live;
        fake_hip::state().fail_malloc_in = at;
        ddef_ctx* c = nullptr;
        const int rc = ddef_init(9000, 2, 2, &c);
        fake_hip::state().fail_malloc_in = -1;
        if (rc == DDEF_OK) { CHECK(c != nullptr); CHECK(ddef_destroy(c) == DDEF_OK); CHECK(at >= 10); break; }
        CHECK(rc == DDEF_ENOMEM && c == nullptr);
        CHECK(fake_hip::state().live == live_before);
        CHECK(hipGetLastError() == hipSuccess);               // the failure was reported, not left behind
    }
    fake_hip::state().fail_stream_in = 0;
    ddef_ctx* c = nullptr;
    CHECK(ddef_init(9000, 2, 2, &c) == DDEF_EHIP && c == nullptr);
    fake_hip::state().fail_stream_in = -1;
}

static bool launched_with_null(const char* kernel, size_t pointer_index, size_t from) {
    const std::vector<fake_hip::Launch>& all = fake_hip::state().launches;
    for (size_t i = from; i < all.size(); ++i)
        if (all[i].kernel == kernel && all[i].pointers.size() > pointer_index && all[i].pointers[pointer_index] == nullptr)
            return true;
    return false;
}

// The second stream, its events and the second gradient buffer of the prefetch option, with each
// of the four failing in turn: the call reports it, the next call sets everything up afresh and
// never launches the generator on a null buffer.
static void prefetch_setup_failures() {
    for (int which = 0; which < 4; ++which) {
        ddef_ctx* c = nullptr;
        CHECK(ddef_init(5000, 2, 2, &c) == DDEF_OK);
        set_problem(c, 5000);
        CHECK(ddef_set_tau(c, 1) == DDEF_OK);
        CHECK(ddef_set_option(c, DDEF_OPT_PREFETCH_GRAD, 1) == DDEF_OK);
        CHECK(step(c, 0.01, 0.05f) == DDEF_OK);               // t = 0 < tau: empty, no prefetch yet
        const size_t from = fake_hip::state().launches.size();
        if (which == 0) fake_hip::state().fail_stream_in = 0;
        if (which == 1) fake_hip::state().fail_event_in = 0;
        if (which == 2) fake_hip::state().fail_event_in = 1;
        if (which == 3) fake_hip::state().fail_malloc_in = 0;
        const int rc = ddef_grad(c);
        fake_hip::state().fail_stream_in = fake_hip::state().fail_event_in = fake_hip::state().fail_malloc_in = -1;
        CHECK(rc == (which == 3 ? DDEF_ENOMEM : DDEF_EHIP));
        if (which == 3) {
            // out of memory is not sticky: the same call again must work, with a real buffer
            CHECK(ddef_grad(c) == DDEF_OK);
            CHECK(ddef_ef_compress(c, 0.01, 0.05f) == DDEF_OK);
            CHECK(ddef_aggregate(c) == DDEF_OK);
            CHECK(ddef_apply_delayed(c, 0.05f) == DDEF_OK);
            for (int it = 0; it < 3; ++it) { const int rs = step(c, 0.01, 0.05f); if (rs) std::printf("step -> %d\n", rs); CHECK(rs == DDEF_OK); }
        } else {
            CHECK(ddef_grad(c) == DDEF_EHIP);                 // a failed runtime call is sticky
        }
        CHECK(!launched_with_null("k_grad", 4, from));        // GradSource is no pointer: lambda.. are inside it; dest is pointer 0
        CHECK(!launched_with_null("k_grad", 0, from));
        CHECK(ddef_destroy(c) == DDEF_OK);
    }
}

// The sample buffers of the filter bound (two allocations) and the candidate and message rows
// (several): a failure in the middle is reported and the next call recovers.
static void compress_setup_failures() {
    for (long at = 0; at < 12; ++at) {
        ddef_ctx* c = nullptr;
        CHECK(ddef_init(300000, 2, 0, &c) == DDEF_OK);
        set_problem(c, 300000);
        CHECK(ddef_grad(c) == DDEF_OK);
        const size_t from = fake_hip::state().launches.size();
        fake_hip::state().fail_malloc_in = at;
        const int rc = ddef_ef_compress(c, 0.01, 0.05f);
        const bool fired = fake_hip::state().fail_malloc_in == -1;
        fake_hip::state().fail_malloc_in = -1;
        if (fired) {
            CHECK(rc == DDEF_ENOMEM);
            CHECK(ddef_ef_compress(c, 0.01, 0.05f) == DDEF_OK);
        } else {
            CHECK(rc == DDEF_OK);
        }
        CHECK(!launched_with_null("k_sample_begin", 1, from));       // sel, sample_total, hist
        CHECK(!launched_with_null("k_sample_p<false>", 3, from));    // e, g, sample (GradSource holds the rest)
        CHECK(ddef_aggregate(c) == DDEF_OK);
        CHECK(ddef_apply_delayed(c, 0.05f) == DDEF_OK);
        for (int kind : {DDEF_COMPRESSOR_COMPOSED, DDEF_COMPRESSOR_RANDK}) {
            CHECK(ddef_set_compressor(c, kind) == DDEF_OK);
            CHECK(ddef_grad(c) == DDEF_OK);
            fake_hip::state().fail_malloc_in = at % 4;
            const int rc2 = ddef_ef_compress(c, 0.3, 0.05f);
            const bool fired2 = fake_hip::state().fail_malloc_in == -1;
            fake_hip::state().fail_malloc_in = -1;
            if (fired2) { CHECK(rc2 == DDEF_ENOMEM); CHECK(ddef_ef_compress(c, 0.3, 0.05f) == DDEF_OK); }
            else CHECK(rc2 == DDEF_OK);
            CHECK(ddef_aggregate(c) == DDEF_OK);
            CHECK(ddef_apply_delayed(c, 0.05f) == DDEF_OK);
        }
        read_everything(c, 300000, 2);
        CHECK(ddef_destroy(c) == DDEF_OK);
    }
}

// host scalars: Algorithm 3, its look-up table, the timing model
static void deco_calls() {
    const double v_g = 32.0 * 124e6;
    for (double a : {5e7, 1e8, 1e9, 1e10}) for (double b : {0.0, 0.01, 0.1, 0.3}) {
        uint32_t tau = 0, tau2 = 0;
        double delta = 0.0, delta2 = 0.0;
        CHECK(ddef_deco(v_g, a, b, 0.02, &tau, &delta) == DDEF_OK);
        CHECK(ddef_deco_noniid(v_g, a, b, 0.02, &tau2, &delta2) == DDEF_OK);
        CHECK(delta > 0.0 && delta <= 1.0 && ddef_phi(delta, tau) >= 0.0 && ddef_phi_prime(delta2, tau2) >= 0.0);
        CHECK(ddef_t_avg_model(tau, delta, v_g, a, b, 0.02) > 0.0);
        CHECK(ddef_t_avg_simulate(tau, delta, v_g, a, b, 0.02, 500) > 0.0);
        CHECK(ddef_t_avg_simulate(tau, delta, v_g, a, b, 0.02, 1) > 0.0);
    }
    double only = 0.0;
    uint32_t hide = 0;
    CHECK(ddef_corner_compression_only(v_g, 1e8, 0.02, &only) == DDEF_OK && only > 0.0 && only < 1.0);
    CHECK(ddef_corner_compression_only(v_g, 1e12, 0.02, &only) == DDEF_OK && only == 1.0);
    CHECK(ddef_corner_delay_only(v_g, 1e8, 0.1, 0.02, 16, &hide) == DDEF_OK && hide == 16);
    CHECK(ddef_corner_delay_only(v_g, 1e12, 0.01, 0.02, 16, &hide) == DDEF_OK && hide == 1);
    CHECK(ddef_corner_delay_only(v_g, 0.0, 0.1, 0.02, 16, &hide) == DDEF_EINVAL);
    CHECK(ddef_corner_compression_only(v_g, 1e8, 0.02, nullptr) == DDEF_EINVAL);
    ddef_lut* lut = nullptr;
    CHECK(ddef_lut_build(v_g, 1e8, 1e10, 20, 0.1, 0.02, &lut) == DDEF_OK);
    for (double a : {5e7, 1e8, 1.234e9, 9.99e9, 1e10, 2e10}) {
        uint32_t tau = 0;
        double delta = 0.0;
        int from = -1;
        CHECK(ddef_lut_query(lut, a, &tau, &delta, &from) == DDEF_OK && (from == 0 || from == 1));
        CHECK(ddef_lut_query(lut, a, &tau, &delta, nullptr) == DDEF_OK);
    }
    CHECK(ddef_lut_destroy(lut) == DDEF_OK);
    CHECK(ddef_lut_build(v_g, 1e8, 2e8, 2, 0.1, 0.02, &lut) == DDEF_OK);       // the smallest table
    CHECK(ddef_lut_destroy(lut) == DDEF_OK);
    CHECK(ddef_lut_build(v_g, 1e8, 2e8, 1, 0.1, 0.02, &lut) == DDEF_EINVAL && lut == nullptr);
    uint32_t tau = 0;
    double delta = 0.0;
    CHECK(ddef_deco(v_g, -1.0, 0.1, 0.02, &tau, &delta) == DDEF_EINVAL);
    CHECK(ddef_deco(v_g, 1e9, 0.1, 0.02, nullptr, &delta) == DDEF_EINVAL);
    CHECK(ddef_lut_build(v_g, 1e9, 1e8, 20, 0.1, 0.02, &lut) == DDEF_EINVAL);
    CHECK(ddef_lut_build(v_g, 1e8, 1e9, 0, 0.1, 0.02, &lut) == DDEF_EINVAL);
    CHECK(ddef_lut_query(nullptr, 1e9, &tau, &delta, nullptr) == DDEF_EINVAL);
    CHECK(ddef_k_from_delta(0.001, 124000000) == 124000 && ddef_k_from_delta(1.0, 5) == 5 &&
          ddef_k_from_delta(1e-12, 5) == 1 && ddef_k_from_delta(0.5, 0) == 0 && ddef_k_from_delta(2.0, 5) == 0);
}

// the allocation-free entry point: what it accepts, what it refuses, and that it never allocates
static void static_entry_point() {
    const uint64_t d = 10001, ld = 10004;
    std::vector<float> e(2 * ld + 4, 0.5f), g(2 * ld + 4, 1.0f), val(2 * 200);
    std::vector<uint32_t> idx(2 * 200);
    float* ep = e.data() + ((16 - (reinterpret_cast<uintptr_t>(e.data()) & 15u)) & 15u) / 4;     // 16-byte aligned
    float* gp = g.data() + ((16 - (reinterpret_cast<uintptr_t>(g.data()) & 15u)) & 15u) / 4;
    const long mallocs_before = fake_hip::state().mallocs;
    CHECK(ddef_ef_compress_static(ep, gp, ld, d, 2, 0.01, 0.05f, idx.data(), val.data(), 200, nullptr) == DDEF_OK);
    CHECK(ddef_ef_compress_static(ep, gp, ld, d, 1, 0.001, 0.05f, idx.data(), val.data(), 200, nullptr) == DDEF_OK);
    CHECK(fake_hip::state().mallocs == mallocs_before);
    CHECK(ddef_ef_compress_static(ep, gp, ld, d, 65, 0.01, 0.05f, idx.data(), val.data(), 200, nullptr) == DDEF_EINVAL);
    CHECK(ddef_ef_compress_static(ep, gp, 4000000000ull, 3999999999ull, 3, 0.01, 0.05f, idx.data(), val.data(), 1ull << 30, nullptr) == DDEF_EINVAL);
    CHECK(ddef_ef_compress_static(ep, gp, ld - 4, d, 2, 0.01, 0.05f, idx.data(), val.data(), 200, nullptr) == DDEF_EINVAL);
    CHECK(ddef_ef_compress_static(ep, gp, ld + 1, d, 2, 0.01, 0.05f, idx.data(), val.data(), 200, nullptr) == DDEF_EINVAL);
    CHECK(ddef_ef_compress_static(ep + 1, gp, ld, d, 2, 0.01, 0.05f, idx.data(), val.data(), 200, nullptr) == DDEF_EINVAL);
    CHECK(ddef_ef_compress_static(ep, gp, ld, d, 2, 0.01, 0.05f, idx.data(), val.data(), 100, nullptr) == DDEF_EINVAL);
    CHECK(ddef_ef_compress_static(ep, gp, ld, d, 2, 0.0, 0.05f, idx.data(), val.data(), 200, nullptr) == DDEF_EINVAL);
    CHECK(ddef_ef_compress_static(nullptr, gp, ld, d, 2, 0.01, 0.05f, idx.data(), val.data(), 200, nullptr) == DDEF_EINVAL);
    CHECK(ddef_ef_compress_static(ep, gp, ld, 0, 2, 0.01, 0.05f, idx.data(), val.data(), 200, nullptr) == DDEF_EINVAL);
}

// the buffers of the sure / band split of dense messages (records, run table, slot counters) and the
// canonical-message buffers of the getter, each allocation failing in turn
static void dense_split_setup_failures() {
    for (long at = 0; at < 8; ++at) {
        ddef_ctx* c = nullptr;
        CHECK(ddef_init(70001, 2, 0, &c) == DDEF_OK);
        set_problem(c, 70001);
        CHECK(ddef_grad(c) == DDEF_OK);
        fake_hip::state().fail_malloc_in = at;
        const int rc = ddef_ef_compress(c, 0.3, 0.05f);
        const bool fired = fake_hip::state().fail_malloc_in == -1;
        fake_hip::state().fail_malloc_in = -1;
        if (fired) { CHECK(rc == DDEF_ENOMEM); CHECK(ddef_ef_compress(c, 0.3, 0.05f) == DDEF_OK); }
        else CHECK(rc == DDEF_OK);
        CHECK(ddef_aggregate(c) == DDEF_OK);
        CHECK(ddef_apply_delayed(c, 0.05f) == DDEF_OK);
        read_everything(c, 70001, 2);
        CHECK(step(c, 0.3, 0.05f) == DDEF_OK);
        CHECK(ddef_destroy(c) == DDEF_OK);
    }
}

int main() {
    deco_calls();
    dense_split_setup_failures();
    static_entry_point();
    plain_runs();
    call_order_and_arguments();
    init_failures();
    prefetch_setup_failures();
    compress_setup_failures();
    CHECK(fake_hip::state().live == 0);                       // every device allocation was freed
    CHECK(hipGetLastError() == hipSuccess);                   // no launch with an empty grid or an oversized block
    std::printf("%s: %zu launches logged, %ld allocations\n", failures ? "FAILED" : "ok",
                fake_hip::state().launches.size(), fake_hip::state().mallocs);
    return failures ? 1 : 0;
}
