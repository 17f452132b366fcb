// Drives the C ABI of the library on the CPU (device side replaced by stubs.cpp) under AddressSanitizer / UBSan.
// Reads one model per line from stdin:
//   structure K channels family max_batch num_vars depth num_replica seed height width num_deltas d0 d1 axes leaf_param
// and for each: create, sizes, structure (every table walked to its stated length), bind with host buffers standing in
// for device memory, the compute calls (their host side: argument checks, layer loops, profiling records), the error
// paths, destroy.  Prints one line per model; exit status 0 unless an invariant of the tables is broken.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/einet.h"

#define REQUIRE(c) do { if (!(c)) { std::printf("FAILED %s line %d\n", #c, __LINE__); return 1; } } while (0)

static int run_model(const einet_spec& s, long long* checksum) {
    einet_t* h = nullptr;
    int rc = einet_create(&s, &h);
    if (rc != EINET_OK) {
        REQUIRE(h == nullptr);
        REQUIRE(std::strlen(einet_last_error(nullptr)) > 0);
        std::printf("create rc=%d (%s)\n", rc, einet_last_error(nullptr));
        return 0;
    }
    size_t n_params = 0, n_stats = 0, ws = 0;
    REQUIRE(einet_sizes(h, &n_params, &n_stats, &ws) == EINET_OK);
    einet_structure_view v;
    REQUIRE(einet_structure(h, &v) == EINET_OK);
    long long sum = 0;
    for (int r = 0; r <= v.num_regions; ++r) sum += v.scope_ptr[r];
    for (int i = 0; i < v.scope_ptr[v.num_regions]; ++i) { REQUIRE(v.scope_var[i] >= 0 && v.scope_var[i] < v.num_vars); sum += v.scope_var[i]; }
    for (int r = 0; r < v.num_regions; ++r) { REQUIRE(v.region_replica[r] >= -1 && v.region_replica[r] < v.num_replica); sum += v.v_offset[r]; }
    for (int p = 0; p < v.num_partitions; ++p) {
        for (int q = 0; q < 3; ++q) REQUIRE(v.partition[3 * p + q] >= 0 && v.partition[3 * p + q] < v.num_regions);
        REQUIRE(v.w_offset[p] >= 0 && (size_t)v.w_offset[p] < n_params);
        sum += v.w_offset[p];
    }
    REQUIRE(v.layer_ptr[0] == 0 && v.layer_ptr[v.num_layers] == v.num_partitions);
    for (int i = 0; i < v.num_partitions; ++i) REQUIRE(v.layer_partition[i] >= 0 && v.layer_partition[i] < v.num_partitions);
    REQUIRE(v.phi_offset > 0 && (size_t)v.phi_offset <= n_params && (size_t)v.tot_offset < n_stats);
    *checksum += sum;

    // calls before bind are refused
    const int B = s.max_batch;
    std::vector<float> x((size_t)B * v.num_vars * v.channels, 0.f), logp(B), out(x.size());
    REQUIRE(einet_logp(h, x.data(), nullptr, EINET_MASK_NONE, B, logp.data(), nullptr) == EINET_ERR_NOT_BOUND);
    REQUIRE(einet_em_update(h, 0.5f, 1e-6f, 1.f, 0.f, nullptr) == EINET_ERR_NOT_BOUND);

    // host buffers stand in for device memory (256-byte aligned)
    float* params = static_cast<float*>(std::aligned_alloc(256, (n_params * 4 + 255) / 256 * 256));
    float* stats = static_cast<float*>(std::aligned_alloc(256, (n_stats * 4 + 255) / 256 * 256));
    char* wsp = static_cast<char*>(std::aligned_alloc(256, (ws + 255) / 256 * 256));
    REQUIRE(params && stats && wsp);
    std::memset(params, 0, n_params * 4); std::memset(stats, 0, n_stats * 4); std::memset(wsp, 0, ws);
    REQUIRE(einet_bind(h, params + 1, stats, wsp, nullptr) == EINET_ERR_INVALID_ARG);      // misaligned
    REQUIRE(einet_bind(h, params, stats, wsp, nullptr) == EINET_OK);
    REQUIRE(einet_refresh(h, nullptr) == EINET_OK);
    REQUIRE(einet_init_params(h, 7, 0.1f, 0.9f, nullptr) == EINET_OK);
    REQUIRE(einet_init_params(h, 7, 0.9f, 0.1f, nullptr) == EINET_ERR_INVALID_ARG);
    std::vector<uint8_t> mask((size_t)B * v.num_vars, 1);
    REQUIRE(einet_profile_enable(h, 1) == EINET_OK);
    REQUIRE(einet_logp(h, x.data(), nullptr, EINET_MASK_NONE, B, logp.data(), nullptr) == EINET_OK);
    REQUIRE(einet_logp(h, x.data(), mask.data(), EINET_MASK_PER_SAMPLE, B, logp.data(), nullptr) == EINET_OK);
    REQUIRE(einet_logp(h, x.data(), mask.data(), EINET_MASK_NONE, B, logp.data(), nullptr) == EINET_ERR_INVALID_ARG);
    REQUIRE(einet_logp(h, x.data(), nullptr, EINET_MASK_NONE, B + 1, logp.data(), nullptr) == EINET_ERR_BATCH_TOO_LARGE);
    REQUIRE(einet_logp(h, x.data(), nullptr, EINET_MASK_NONE, 0, logp.data(), nullptr) == EINET_ERR_INVALID_ARG);
    rc = einet_logp_static(h, x.data(), nullptr, EINET_MASK_NONE, B, logp.data(), nullptr);
    REQUIRE(rc == EINET_OK || rc == EINET_ERR_BATCH_TOO_LARGE);
    REQUIRE(einet_em_accumulate(h, x.data(), mask.data(), EINET_MASK_SHARED, B, logp.data(), nullptr) == EINET_OK);
    REQUIRE(einet_em_update(h, 0.5f, 1e-6f, 1.f, 1e-9f, nullptr) == EINET_OK);
    REQUIRE(einet_em_update(h, 1.5f, 1e-6f, 1.f, 1e-9f, nullptr) == EINET_ERR_INVALID_ARG);
    REQUIRE(einet_em_accumulate(h, x.data(), nullptr, EINET_MASK_NONE, 1, nullptr, nullptr) == EINET_OK);
    REQUIRE(einet_em_reset(h, nullptr) == EINET_OK);
    std::vector<float> xs((size_t)(2 * B + 1) * v.num_vars * v.channels, 0.f), lps(2 * B + 1);
    REQUIRE(einet_em_epoch(h, xs.data(), nullptr, EINET_MASK_NONE, 2 * B + 1, B, 0.5f, 1e-6f, 1.f, 1e-9f, lps.data(), nullptr) == EINET_OK);
    std::vector<float> u((size_t)(v.num_partitions + v.num_regions) * B, 0.5f);
    REQUIRE(einet_sample(h, B, nullptr, nullptr, EINET_MASK_NONE, u.data(), nullptr, out.data(), nullptr) == EINET_OK);
    REQUIRE(einet_sample(h, B, x.data(), mask.data(), EINET_MASK_SHARED, u.data(), x.data(), out.data(), nullptr) == EINET_OK);
    REQUIRE(einet_sample(h, B, x.data(), nullptr, EINET_MASK_NONE, u.data(), nullptr, out.data(), nullptr) < 0);
    int ncls = 0; const char* names[16]; double ms[16]; int64_t cnt[16];
    REQUIRE(einet_profile_read(h, 16, &ncls, names, ms, cnt) == EINET_OK);
    int64_t nl = 0;
    REQUIRE(einet_profile_launches(h, 0, &nl, nullptr, nullptr, nullptr) == EINET_OK);
    std::vector<int32_t> cls(nl); std::vector<float> lms(nl); std::vector<int64_t> work(nl);
    REQUIRE(einet_profile_launches(h, nl, &nl, cls.data(), lms.data(), work.data()) == EINET_OK);
    for (int64_t i = 0; i < nl; ++i) REQUIRE(cls[i] >= 0 && cls[i] < ncls);
    // binding again (same buffers, then others) and a second handle alive at the same time
    REQUIRE(einet_bind(h, params, stats, wsp, nullptr) == EINET_OK);
    einet_t* h2 = nullptr;
    REQUIRE(einet_create(&s, &h2) == EINET_OK);
    einet_destroy(h2);
    std::printf("ok regions %d partitions %d layers %d params %zu workspace %zu launches %lld\n", v.num_regions, v.num_partitions,
                v.num_layers, n_params, ws, (long long)nl);
    einet_destroy(h);
    std::free(params); std::free(stats); std::free(wsp);
    return 0;
}

int main() {
    // NULL arguments
    einet_t* h = nullptr;
    if (einet_create(nullptr, &h) != EINET_ERR_INVALID_ARG) return 2;
    einet_destroy(nullptr);
    size_t a, b, c;
    if (einet_sizes(nullptr, &a, &b, &c) == EINET_OK) return 2;
    long long checksum = 0;
    char line[512];
    int n = 0;
    while (std::fgets(line, sizeof line, stdin)) {
        einet_spec s;
        std::memset(&s, 0, sizeof s);
        long long seed;
        int d0, d1;
        if (std::sscanf(line, "%d %d %d %d %d %d %d %d %lld %d %d %d %d %d %d %d", &s.structure, &s.K, &s.channels, &s.leaf_family,
                        &s.max_batch, &s.num_vars, &s.depth, &s.num_replica, &seed, &s.height, &s.width, &s.num_deltas, &d0, &d1,
                        &s.axes, &s.leaf_param) != 16)
            continue;
        s.seed = (uint64_t)seed; s.deltas[0] = d0; s.deltas[1] = d1;
        std::printf("model %d: ", n++);
        if (run_model(s, &checksum)) return 1;
    }
    std::printf("models %d checksum %lld\n", n, checksum);
    return 0;
}
