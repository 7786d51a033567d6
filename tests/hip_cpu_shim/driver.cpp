// Runs every entry point of the library, compiled for the host against the HIP stand-in, on
// small shapes, under AddressSanitizer / UBSan.  Checks the outputs against the plain sum of
// eq. (1) of the paper and the coded packets of the different paths against each other.
// Usage: driver K r Q N T mode jobs [cus blocks_per_cu]      (mode: 0 f32, 1 u32, 2 h32, 3 bf16, 4 f16)
// Test infrastructure only.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <vector>

#include "ccdc.h"

#define CHECK(call)                                                                              \
    do {                                                                                         \
        const int rc_ = (call);                                                                  \
        if (rc_ != CCDC_OK) {                                                                    \
            std::fprintf(stderr, "%s -> %d (%s)\n", #call, rc_, ccdc_strerror(rc_));            \
            return 2;                                                                            \
        }                                                                                        \
    } while (0)

static int64_t query(const ccdc_plan_t *p, int what)
{
    int64_t v = -1;
    if (ccdc_plan_query(p, what, &v, sizeof v) != CCDC_OK) std::abort();
    return v;
}

static uint64_t mix(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static float widen16(uint16_t b, bool bf)
{
    if (bf) return __uint_as_float((uint32_t)b << 16);
    _Float16 h;
    std::memcpy(&h, &b, 2);
    return (float)h;
}

// A shape whose work items fit 32 bits with four-element packs but not with one-element packs:
// ccdc_plan_bind accepts it; a call with pointers that are only 4-byte aligned falls back to
// one-element packs and must be refused with CCDC_ESIZE before anything is launched (the
// pointers given here point nowhere: a launch would be caught by the sanitizer).
static int limits()
{
    const int K = 4, r = 2, Q = 4, N = 6;
    const int64_t T = 200000000;
    ccdc_plan_t *p = nullptr;
    CHECK(ccdc_plan(K, r, Q, N, &p));
    CHECK(ccdc_plan_bind(p, T, CCDC_U32_XOR));
    CHECK(ccdc_plan_upload(p));
    const long before = shim::launches.load();
    void *a = reinterpret_cast<void *>(0x1004), *b = reinterpret_cast<void *>(0x2004), *c = reinterpret_cast<void *>(0x3004);
    int bad = 0;
    // combine and decode have one work item per pack of a W-long packet: 12 * 2e8 > 2^31 - 1
    // (the encoders have one per pack of a segment, r times fewer: those still fit)
    bad += ccdc_combine(p, a, b, nullptr) != CCDC_ESIZE;
    bad += ccdc_decode(p, a, b, c, nullptr) != CCDC_ESIZE;
    bad += shim::launches.load() != before;
    // a value length past what any pack width indexes is refused when the plan is bound
    bad += ccdc_plan_bind(p, (int64_t)1 << 38, CCDC_U32_XOR) != CCDC_ESIZE;
    ccdc_plan_destroy(p);
    std::printf(bad ? "limits FAILED (%d)\n" : "limits ok\n", bad);
    return bad ? 1 : 0;
}

int main(int argc, char **argv)
{
    if (argc == 2 && std::strcmp(argv[1], "limits") == 0) return limits();
    if (argc < 8) return 64;
    const int K = atoi(argv[1]), r = atoi(argv[2]), Q = atoi(argv[3]), N = atoi(argv[4]);
    const int64_t T = atoll(argv[5]);
    const int mode = atoi(argv[6]), jobs = atoi(argv[7]);
    if (argc > 9) {
        shim::compute_units = atoi(argv[8]);
        shim::blocks_per_cu = atoi(argv[9]);
    }
    const bool half = mode >= 3, real = mode != 1;
    const size_t eb = half ? 2 : 4;

    ccdc_plan_t *p = nullptr;
    CHECK(jobs ? ccdc_plan_jobs(K, r, Q, N, &p) : ccdc_plan(K, r, Q, N, &p));
    CHECK(ccdc_plan_bind(p, T, mode));
    CHECK(ccdc_plan_upload(p));
    const int64_t nv = query(p, CCDC_Q_V_ELEMS), nvb = query(p, CCDC_Q_VBAR_ELEMS), nx = query(p, CCDC_Q_X_ELEMS),
                  nd = query(p, CCDC_Q_D_ELEMS), nphi = query(p, CCDC_Q_PHI_ELEMS), J = query(p, CCDC_Q_J);

    // exact-size heap blocks: any access outside them is reported by the sanitizer
    auto dev = [&](int64_t n) { return static_cast<unsigned char *>(std::malloc((size_t)n * eb)); };
    unsigned char *V = dev(nv), *Vbar = dev(nvb), *X = dev(nx), *D = dev(nd), *Phi = dev(nphi);
    unsigned char *X2 = dev(nx), *D2 = dev(nd), *Phi2 = dev(nphi), *X3 = dev(nx), *Phi3 = dev(nphi), *X4 = dev(nx),
                  *Phi4 = dev(nphi), *X5 = dev(nx), *Phi5 = dev(nphi);
    for (int64_t i = 0; i < nv; i++) {
        const uint64_t h = mix(0x9E3779B97F4A7C15ull * (uint64_t)(i + 1));
        if (half) {
            // small integers in the format: exact in every summation order
            const int v = (int)(h % 7) - 3;
            uint16_t b;
            if (mode == 3) {
                b = (uint16_t)(__float_as_uint((float)v) >> 16);
            } else {
                const _Float16 hh = (_Float16)(float)v;
                std::memcpy(&b, &hh, 2);
            }
            std::memcpy(V + i * 2, &b, 2);
        } else if (real) {
            const float v = (float)((int)(h % 2001) - 1000);        // integers: exact sums in fp32
            std::memcpy(V + i * 4, &v, 4);
        } else {
            const uint32_t v = (uint32_t)(h >> 32);
            std::memcpy(V + i * 4, &v, 4);
        }
    }
    // eq. (1): Phi[j][q][t] = sum over the N files of V[j][n][q][t]
    std::vector<double> want_r(real ? nphi : 0);
    std::vector<uint32_t> want_x(real ? 0 : nphi);
    for (int64_t j = 0; j < J; j++)
        for (int64_t n = 0; n < N; n++)
            for (int64_t q = 0; q < Q; q++)
                for (int64_t t = 0; t < T; t++) {
                    const int64_t src = ((j * N + n) * Q + q) * T + t, dst = (j * Q + q) * T + t;
                    if (half) {
                        uint16_t b;
                        std::memcpy(&b, V + src * 2, 2);
                        want_r[dst] += widen16(b, mode == 3);
                    } else if (real) {
                        float v;
                        std::memcpy(&v, V + src * 4, 4);
                        want_r[dst] += v;
                    } else {
                        uint32_t v;
                        std::memcpy(&v, V + src * 4, 4);
                        want_x[dst] ^= v;
                    }
                }
    int bad = 0;
    auto check_phi = [&](const unsigned char *got, const char *name) {
        for (int64_t i = 0; i < nphi; i++) {
            bool ok;
            if (half) {
                uint16_t b;
                std::memcpy(&b, got + i * 2, 2);
                const double g = widen16(b, mode == 3), w = want_r[i];
                ok = std::fabs(g - w) <= std::fabs(w) * (mode == 3 ? 1.0 / 256 : 1.0 / 2048) + 1e-9;
            } else if (real) {
                float g;
                std::memcpy(&g, got + i * 4, 4);
                ok = (double)g == want_r[i];
            } else {
                uint32_t g;
                std::memcpy(&g, got + i * 4, 4);
                ok = g == want_x[i];
            }
            if (!ok) {
                if (bad < 5) std::fprintf(stderr, "%s: output %lld differs from the plain sum\n", name, (long long)i);
                bad++;
            }
        }
    };
    auto same = [&](const unsigned char *a, const unsigned char *b, int64_t n, const char *name) {
        if (std::memcmp(a, b, (size_t)n * eb) != 0) {
            std::fprintf(stderr, "%s differs\n", name);
            bad++;
        }
    };

    // SHIM_ONLY_PIPELINE=1: only the one-pass pipeline, checked against the plain sum (for shapes
    // at which the staged kernels, one emulated thread per work item, would take too long)
    if (std::getenv("SHIM_ONLY_PIPELINE")) {
        CHECK(ccdc_pipeline_fused(p, V, X3, Phi3, nullptr));
        check_phi(Phi3, "pipeline Phi");
        ccdc_plan_destroy(p);
        for (unsigned char *q : {V, Vbar, X, D, Phi, X2, D2, Phi2, X3, Phi3, X4, Phi4, X5, Phi5}) std::free(q);
        std::printf("K=%d r=%d Q=%d N=%d T=%lld mode=%d: pipeline only, %ld launches, %d mismatches\n", K, r, Q, N,
                    (long long)T, mode, shim::launches.load(), bad);
        std::fflush(stdout);
        return bad ? 1 : 0;
    }
    CHECK(ccdc_combine(p, V, Vbar, nullptr));
    CHECK(ccdc_encode(p, Vbar, X, nullptr));
    CHECK(ccdc_decode(p, X, Vbar, D, nullptr));
    CHECK(ccdc_reduce(p, V, D, Phi, nullptr));
    check_phi(Phi, "staged Phi");
    same(D, Vbar, nd, "decoded packets vs pre-combined packets");

    CHECK(ccdc_shuffle_fused(p, V, X2, D2, nullptr));
    CHECK(ccdc_reduce(p, V, D2, Phi2, nullptr));
    same(X2, X, nx, "fused X");
    same(D2, D, nd, "fused D");
    check_phi(Phi2, "fused Phi");

    const int rc = ccdc_pipeline_fused(p, V, X3, Phi3, nullptr);
    if (rc == CCDC_OK) {
        same(X3, X, nx, "pipeline X");
        check_phi(Phi3, "pipeline Phi");
        CHECK(ccdc_pipeline_fused_noalloc(p, V, X4, Phi4, nullptr));
        same(X4, X, nx, "no-alloc pipeline X");
        same(Phi4, Phi3, nphi, "no-alloc pipeline Phi");
    } else if (rc != CCDC_ESIZE) {
        std::fprintf(stderr, "ccdc_pipeline_fused -> %d\n", rc);
        return 2;
    }

    CHECK(ccdc_node_encode(p, -1, V, X5, nullptr));
    CHECK(ccdc_node_decode_reduce(p, -1, V, X5, Phi5, nullptr));
    same(X5, X, nx, "node-local X");
    check_phi(Phi5, "node-local Phi");

    // Map stand-in: out = theta - files (XOR in the field), separate buffer and in place
    {
        unsigned char *theta = dev(nphi), *out = dev(nv), *inpl = dev(nv);
        for (int64_t i = 0; i < nphi; i++) std::memcpy(theta + i * eb, V + ((i * 7) % nv) * eb, eb);   // any valid patterns
        std::memcpy(inpl, V, (size_t)nv * eb);
        CHECK(ccdc_map(p, V, theta, out, nullptr));
        CHECK(ccdc_map(p, inpl, theta, inpl, nullptr));
        same(inpl, out, nv, "map in place");
        for (int64_t j = 0; j < J; j++)
            for (int64_t n = 0; n < N; n++)
                for (int64_t e = 0; e < (int64_t)Q * T; e++) {
                    const int64_t at = (j * N + n) * Q * T + e, th = j * Q * T + e;
                    bool ok;
                    if (half) {
                        uint16_t a, b, g;
                        std::memcpy(&a, theta + th * 2, 2);
                        std::memcpy(&b, V + at * 2, 2);
                        std::memcpy(&g, out + at * 2, 2);
                        ok = widen16(g, mode == 3) == widen16(a, mode == 3) - widen16(b, mode == 3);   // small integers: exact
                    } else if (real) {
                        float a, b, g;
                        std::memcpy(&a, theta + th * 4, 4);
                        std::memcpy(&b, V + at * 4, 4);
                        std::memcpy(&g, out + at * 4, 4);
                        ok = g == a - b;
                    } else {
                        uint32_t a, b, g;
                        std::memcpy(&a, theta + th * 4, 4);
                        std::memcpy(&b, V + at * 4, 4);
                        std::memcpy(&g, out + at * 4, 4);
                        ok = g == (a ^ b);
                    }
                    if (!ok && bad++ < 5) std::fprintf(stderr, "map: element %lld is wrong\n", (long long)at);
                }
        for (unsigned char *q : {theta, out, inpl}) std::free(q);
    }

    ccdc_plan_destroy(p);
    for (unsigned char *q : {V, Vbar, X, D, Phi, X2, D2, Phi2, X3, Phi3, X4, Phi4, X5, Phi5}) std::free(q);
    std::printf("K=%d r=%d Q=%d N=%d T=%lld mode=%d jobs=%d: %ld launches, pipeline %s, %d mismatches\n", K, r, Q, N,
                (long long)T, mode, jobs, shim::launches.load(), rc == CCDC_OK ? "ran" : "refused (size)", bad);
    return bad ? 1 : 0;
}
