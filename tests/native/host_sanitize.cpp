// Host-side exercise of the library's packer (alcs_pack.cpp), latency model (alcs_latency.cpp) and
// of the C oracle (oracle/alcs_oracle.c), meant to be built with -fsanitize=address,undefined and
// run without a GPU: every layout the packer can build is packed, self-checked, exported and
// compared bit for bit with the oracle's grouped CSR; handles are made from canonical arrays;
// malformed arguments must come back as error codes.  Prints "host sanitize OK" and returns 0.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "alcs.h"

extern "C" {
int64_t oracle_pack_count(const uint8_t *mask, int Cout, int Cin, int k, int V);
int oracle_pack(const float *W, const uint8_t *mask, int Cout, int Cin, int k, int V, int32_t *row_ptr,
                int32_t *col_idx, float *vals);
int oracle_unpack(const int32_t *row_ptr, const int32_t *col_idx, const float *vals, int Cout, int Cin, int k,
                  int V, float *Wd);
int oracle_densify(const float *W, const uint8_t *mask, int Cout, int Cin, int k, int V, float *Wd);
int oracle_conv(const float *Wd, const float *X, const float *bias, float *Y, int N, int Cin, int Cout, int H,
                int Wi, int k, int stride, int nthreads);
int oracle_conv_csr(const int32_t *row_ptr, const int32_t *col_idx, const float *vals, const float *X,
                    const float *bias, float *Y, int N, int Cin, int Cout, int H, int Wi, int k, int stride, int V,
                    float *scratch, double *accbuf);
double oracle_latency_estimate(const double *k, const double *t, int n, double s);
double oracle_network_latency(double tau, const double *k, const double *t, const int *n, int L, const double *s);
}

static unsigned long long rng_state = 0x9E3779B97F4A7C15ull;
static unsigned next_u32() {
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (unsigned)(rng_state >> 33);
}
static float next_f() { return (float)(int)(next_u32() % 2001 - 1000) / 250.0f; }

#define CHECK(cond)                                                                 \
    do {                                                                            \
        if (!(cond)) {                                                              \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            return 1;                                                               \
        }                                                                           \
    } while (0)

static int one_layer(int Cout, int Cin, int k, int V, int density_pct, const alcs_options *opt) {
    const int G = (Cout + V - 1) / V, K = Cin * k * k;
    std::vector<float> W((size_t)Cout * K);
    for (float &w : W) w = next_f();
    std::vector<uint8_t> mask((size_t)G * K);
    for (uint8_t &m : mask) m = (int)(next_u32() % 100) < density_pct;
    const uint8_t *mp = density_pct >= 100 ? nullptr : mask.data();
    const int64_t nnzb = oracle_pack_count(mp, Cout, Cin, k, V);
    std::vector<int32_t> rp((size_t)G + 1), ci((size_t)nnzb + 1);
    std::vector<float> vals((size_t)nnzb * V + 1);
    CHECK(oracle_pack(W.data(), mp, Cout, Cin, k, V, rp.data(), ci.data(), vals.data()) == 0);

    alcs_packed_t *p = nullptr;
    CHECK(alcs_pack_weights_opt(W.data(), mp, Cout, Cin, k, V, opt, &p) == ALCS_OK && p);
    int g2 = 0, k2 = 0;
    int64_t n2 = 0;
    CHECK(alcs_packed_info(p, &g2, &k2, &n2) == ALCS_OK && g2 == G && k2 == K && n2 == nnzb);
    CHECK(alcs_packed_selfcheck(p) == ALCS_OK);
    std::vector<int32_t> rp2((size_t)G + 1), ci2((size_t)nnzb + 1);
    std::vector<float> vals2((size_t)nnzb * V + 1);
    CHECK(alcs_packed_export(p, rp2.data(), ci2.data(), vals2.data()) == ALCS_OK);
    CHECK(!std::memcmp(rp.data(), rp2.data(), sizeof(int32_t) * (G + 1)));
    CHECK(!std::memcmp(ci.data(), ci2.data(), sizeof(int32_t) * nnzb));
    CHECK(!std::memcmp(vals.data(), vals2.data(), sizeof(float) * nnzb * V));
    alcs_options back;
    CHECK(alcs_packed_get_options(p, &back) == ALCS_OK);
    CHECK(alcs_packed_set_options(p, &back) == ALCS_OK);
    // a handle from the canonical arrays is the same handle
    alcs_packed_t *q = nullptr;
    CHECK(alcs_pack_from_csr(rp.data(), ci.data(), vals.data(), Cout, Cin, k, V, &q) == ALCS_OK && q);
    CHECK(alcs_packed_selfcheck(q) == ALCS_OK);
    CHECK(alcs_packed_export(q, rp2.data(), ci2.data(), vals2.data()) == ALCS_OK);
    CHECK(!std::memcmp(ci.data(), ci2.data(), sizeof(int32_t) * nnzb));
    // the launch is refused cleanly without a device copy / with bad shapes (no GPU needed)
    float x[16] = {0};
    const int rc = alcs_sparse_conv(p, x, nullptr, x, 1, Cin + 1, Cout, 2, 2, k, 1, nullptr);
    CHECK(rc == ALCS_E_INVALID_ARG);
    alcs_packed_free(q);
    alcs_packed_free(p);

    // the oracle's two evaluators agree on a tiny input (integer-valued data: exact)
    if ((long long)Cout * K <= 4096) {
        const int N = 2, H = 5, Wi = 4;
        for (int stride = 1; stride <= 2; ++stride) {
            const int pad = (k - 1) / 2, Ho = (H + 2 * pad - k) / stride + 1, Wo = (Wi + 2 * pad - k) / stride + 1;
            std::vector<float> X((size_t)N * Cin * H * Wi), Wd(W.size()), Y1((size_t)N * Cout * Ho * Wo), Y2(Y1.size());
            for (float &v : X) v = (float)(int)(next_u32() % 7) - 3.0f;
            std::vector<float> Wi_(W.size());
            for (size_t i = 0; i < W.size(); ++i) Wi_[i] = (float)(int)(next_u32() % 5) - 2.0f;
            CHECK(oracle_densify(Wi_.data(), mp, Cout, Cin, k, V, Wd.data()) == 0);
            CHECK(oracle_pack(Wi_.data(), mp, Cout, Cin, k, V, rp.data(), ci.data(), vals.data()) == 0);
            CHECK(oracle_conv(Wd.data(), X.data(), nullptr, Y1.data(), N, Cin, Cout, H, Wi, k, stride, 1) == 0);
            std::vector<float> scratch((size_t)K * Ho * Wo);
            std::vector<double> accbuf((size_t)V * Ho * Wo);
            CHECK(oracle_conv_csr(rp.data(), ci.data(), vals.data(), X.data(), nullptr, Y2.data(), N, Cin, Cout, H, Wi,
                                  k, stride, V, scratch.data(), accbuf.data()) == 0);
            CHECK(!std::memcmp(Y1.data(), Y2.data(), sizeof(float) * Y1.size()));
            std::vector<float> Wu(W.size());
            CHECK(oracle_unpack(rp.data(), ci.data(), vals.data(), Cout, Cin, k, V, Wu.data()) == 0);
            CHECK(!std::memcmp(Wu.data(), Wd.data(), sizeof(float) * Wd.size()));
        }
    }
    return 0;
}

int main() {
    // every group size, both kernels, ragged output channels, all densities incl. empty and full
    const int shapes[][3] = {{8, 5, 1}, {10, 3, 3}, {33, 7, 1}, {44, 70, 1}, {20, 37, 1}, {17, 9, 3}, {24, 640, 1}, {24, 1300, 1}};
    for (const auto &sh : shapes)
        for (int V : {1, 2, 4, 8, 16})
            for (int d : {0, 10, 35, 100}) {
                if (sh[1] >= 640 && d == 100 && V < 4) continue;  // keep the run short
                if (one_layer(sh[0], sh[1], sh[2], V, d, nullptr)) return 1;
            }
    // layouts chosen by options: channel chunks and several groups per wavefront
    for (int kc : {1, 5, 8, 36, 64}) {
        alcs_options o = {};
        o.chunk_channels = kc;
        if (one_layer(20, 37, 1, 4, 30, &o)) return 1;
        if (one_layer(12, 19, 3, 2, 40, &o)) return 1;
    }
    for (int gs : {1, 2, 4})
        for (int V : {4, 8, 16}) {
            alcs_options o = {};
            o.group_slots = gs;
            if (one_layer(50, 70, 1, V, 35, &o)) return 1;
            if (one_layer(44, 600, 1, V, 10, &o)) return 1;
        }
    // refused arguments
    {
        alcs_packed_t *p = nullptr;
        float w[32] = {0};
        CHECK(alcs_pack_weights(nullptr, nullptr, 8, 4, 1, 4, &p) == ALCS_E_INVALID_ARG);
        CHECK(alcs_pack_weights(w, nullptr, 8, 4, 2, 4, &p) == ALCS_E_UNSUPPORTED);
        CHECK(alcs_pack_weights(w, nullptr, 8, 4, 1, 3, &p) == ALCS_E_UNSUPPORTED);
        alcs_options o = {};
        o.waves = -1;
        CHECK(alcs_pack_weights_opt(w, nullptr, 8, 4, 1, 4, &o, &p) == ALCS_E_INVALID_ARG);
        o.waves = 0;
        o.measure_skip = 1;
        CHECK(alcs_pack_weights_opt(w, nullptr, 8, 4, 1, 4, &o, &p) == ALCS_E_INVALID_ARG);
        const int32_t rp[3] = {0, 2, 3};
        const int32_t bad_ci[3] = {1, 1, 0};  // not ascending inside group 0
        const float v[12] = {0};
        CHECK(alcs_pack_from_csr(rp, bad_ci, v, 8, 4, 1, 4, &p) == ALCS_E_INVALID_ARG);
        CHECK(alcs_packed_selfcheck(nullptr) == ALCS_E_INVALID_ARG);
        alcs_packed_free(nullptr);
    }
    // latency model against the oracle
    {
        const double k[5] = {0, 10, 20, 40, 80}, t[5] = {3, 4, 6, 6.5, 9};
        for (double s : {-1.0, 0.0, 5.0, 10.0, 33.0, 80.0, 1e9}) {
            double e = 0;
            CHECK(alcs_latency_estimate(k, t, 5, s, &e) == ALCS_OK);
            const double want = oracle_latency_estimate(k, t, 5, s);
            CHECK(e - want < 1e-12 && want - e < 1e-12);
        }
        const int n[2] = {3, 2};
        const double s2[2] = {12.0, 50.0};
        double net = 0;
        CHECK(alcs_network_latency(1.5, k, t, n, 2, s2, &net) == ALCS_OK);
        const double want = oracle_network_latency(1.5, k, t, n, 2, s2);
        CHECK(net - want < 1e-12 && want - net < 1e-12);
        double e = 0;
        CHECK(alcs_latency_estimate(k, t, 1, 1.0, &e) == ALCS_E_INVALID_ARG);
        const double kbad[3] = {0, 0, 1};
        CHECK(alcs_latency_estimate(kbad, t, 3, 1.0, &e) == ALCS_E_INVALID_ARG);
    }
    std::puts("host sanitize OK");
    return 0;
}
