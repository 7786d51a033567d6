// Host code under AddressSanitizer + UBSan: the library's planner (csrc/plan.cpp, no GPU code in it)
// and the whole oracle (oracle/ccdc_oracle.c) are compiled with the sanitizers into this program,
// which walks K <= kmax, every r, both schedules, c and m in {1, 2}, several value lengths and all
// payload algebras.  Every buffer is a heap block of exactly the size the interfaces state, so an
// index that leaves its table or its artefact stops the run.  The planner's tables are compared
// with the oracle's on the way (the two are written independently).  Test infrastructure only.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ccdc_oracle.h"
#include "plan.hpp"

static long long binom(int n, int k)
{
    long long c = 1;
    for (int i = 1; i <= k; i++) c = c * (n - k + i) / i;
    return c;
}

template <class T>
static T *exact(size_t n)
{
    return static_cast<T *>(std::malloc((n ? n : 1) * sizeof(T)));
}

static int fail(const char *what, int K, int r, int c, int m, int jobs)
{
    std::fprintf(stderr, "MISMATCH %s at K=%d r=%d c=%d m=%d jobs=%d\n", what, K, r, c, m, jobs);
    return 1;
}

int main(int argc, char **argv)
{
    const int kmax = argc > 1 ? atoi(argv[1]) : 7;
    long plans = 0, stage_runs = 0;
    for (int K = 2; K <= kmax; K++)
        for (int r = 1; r < K; r++)
            for (int jobs = 0; jobs < 2; jobs++)
                for (int c = 1; c <= 2; c++)
                    for (int m0 = 1; m0 <= 2; m0++) {
                        const long long nb = jobs ? r + 1 : binom(K, r);
                        int m = m0;
                        while (m * nb < K) m++;
                        const int Q = c * K, N = (int)(m * nb);
                        ccdc_plan_t *p = nullptr;
                        if (ccdc::build_plan(K, r, Q, N, jobs != 0, 1, &p) != CCDC_OK) return fail("build_plan", K, r, c, m, jobs);
                        orc_plan *o = orc_plan_build(K, r, Q, N, jobs ? ORC_PAPER_JOBS : ORC_SINGLE_JOB, nullptr, 0);
                        if (!o) return fail("orc_plan_build", K, r, c, m, jobs);
                        plans++;
                        const int r1 = r + 1;
                        if (p->nbatch != o->n_batch || p->nround != o->n_round || p->J != o->J || p->m != o->m)
                            return fail("counts", K, r, c, m, jobs);
                        if (std::memcmp(p->batch_label.data(), o->batch_label, sizeof(int) * p->nbatch * r) ||
                            std::memcmp(p->batch_job.data(), o->batch_job, sizeof(int) * p->nbatch) ||
                            std::memcmp(p->batch_file0.data(), o->batch_file0, sizeof(int) * p->nbatch) ||
                            std::memcmp(p->round_member.data(), o->round_member, sizeof(int) * p->nround * r1) ||
                            std::memcmp(p->round_batch.data(), o->round_batch, sizeof(int) * p->nround * r1))
                            return fail("tables", K, r, c, m, jobs);
                        for (int64_t T : {1, 3, 4, 8, 10, 12, 40}) {
                            for (int mode = 0; mode <= 4; mode++) {
                                if (ccdc::bind_plan(p, T, mode) != CCDC_OK) return fail("bind_plan", K, r, c, m, jobs);
                                const int64_t W = (int64_t)c * T;
                                if (p->ell != orc_segment_len(W, r) || p->scheduled != orc_scheduled_elems(o, T))
                                    return fail("segment split / scheduled elements", K, r, c, m, jobs);
                                for (int a = 0; a < r1; a++)
                                    if (p->packet_len[a] != orc_packet_len(W, r, a)) return fail("packet length", K, r, c, m, jobs);
                            }
                            if (K > 5 && T > 12) continue;             // keep the stage runs short
                            const int64_t W = (int64_t)c * T, ell = orc_segment_len(W, r), R = o->n_round;
                            const size_t nv = (size_t)o->J * N * Q * T, nvb = (size_t)R * r1 * W, nx = (size_t)R * r1 * ell,
                                         nphi = (size_t)o->J * Q * T;
                            {   // real algebra
                                float *V = exact<float>(nv);
                                for (size_t i = 0; i < nv; i++) V[i] = (float)((int)(i * 2654435761u % 101) - 50);
                                double *Vb = exact<double>(nvb), *X = exact<double>(nx), *D = exact<double>(nvb),
                                       *Phi = exact<double>(nphi), *Ref = exact<double>(nphi);
                                std::memset(D, 0, nvb * sizeof(double));
                                orc_combine_f64(o, T, V, Vb);
                                orc_encode_f64(o, T, Vb, X);
                                orc_decode_f64(o, T, X, Vb, D);
                                orc_reduce_f64(o, T, V, D, Phi);
                                orc_direct_f64(o, T, V, Ref);
                                if (std::memcmp(Phi, Ref, nphi * sizeof(double))) return fail("f64 Phi vs eq. (1)", K, r, c, m, jobs);
                                // hybrid: fp32 sums, XOR-coded patterns
                                float *Vbf = exact<float>(nvb), *Df = exact<float>(nvb);
                                uint32_t *Xu = exact<uint32_t>(nx);
                                std::memset(Df, 0, nvb * sizeof(float));
                                orc_combine_h32(o, T, V, Vbf);
                                orc_encode_h32(o, T, Vbf, Xu);
                                orc_decode_h32(o, T, Xu, Vbf, Df);
                                orc_reduce_h32(o, T, V, Df, Phi);
                                if (std::memcmp(Df, Vbf, nvb * sizeof(float))) return fail("h32 decode", K, r, c, m, jobs);
                                for (void *q : {(void *)V, (void *)Vb, (void *)X, (void *)D, (void *)Phi, (void *)Ref, (void *)Vbf,
                                                (void *)Df, (void *)Xu})
                                    std::free(q);
                            }
                            {   // XOR algebra
                                uint32_t *V = exact<uint32_t>(nv), *Vb = exact<uint32_t>(nvb), *X = exact<uint32_t>(nx),
                                         *D = exact<uint32_t>(nvb), *Phi = exact<uint32_t>(nphi), *Ref = exact<uint32_t>(nphi);
                                for (size_t i = 0; i < nv; i++) V[i] = (uint32_t)(i * 2654435761u) ^ (uint32_t)(i >> 3);
                                std::memset(D, 0, nvb * sizeof(uint32_t));
                                orc_combine_u32(o, T, V, Vb);
                                orc_encode_u32(o, T, Vb, X);
                                orc_decode_u32(o, T, X, Vb, D);
                                orc_reduce_u32(o, T, V, D, Phi);
                                orc_direct_u32(o, T, V, Ref);
                                if (std::memcmp(Phi, Ref, nphi * 4) || std::memcmp(D, Vb, nvb * 4)) return fail("u32 recovery", K, r, c, m, jobs);
                                for (void *q : {(void *)V, (void *)Vb, (void *)X, (void *)D, (void *)Phi, (void *)Ref}) std::free(q);
                            }
                            for (int fmt = 0; fmt < 2; fmt++) {   // 16-bit hybrids
                                uint16_t *V = exact<uint16_t>(nv), *Vb = exact<uint16_t>(nvb), *X = exact<uint16_t>(nx),
                                         *D = exact<uint16_t>(nvb);
                                double *Phi = exact<double>(nphi), *Ref = exact<double>(nphi);
                                float *tmp = exact<float>(nv);
                                for (size_t i = 0; i < nv; i++) tmp[i] = (float)((int)(i * 2246822519u % 13) - 6);
                                orc_h16_narrow(tmp, V, (int64_t)nv, fmt);
                                std::memset(D, 0, nvb * 2);
                                orc_combine_h16(o, T, fmt, V, Vb);
                                orc_encode_h16(o, T, Vb, X);
                                orc_decode_h16(o, T, X, Vb, D);
                                orc_reduce_h16(o, T, fmt, V, D, Phi);
                                orc_direct_h16(o, T, fmt, V, Ref);
                                if (std::memcmp(D, Vb, nvb * 2) || std::memcmp(Phi, Ref, nphi * sizeof(double)))
                                    return fail("h16 recovery", K, r, c, m, jobs);
                                for (void *q : {(void *)V, (void *)Vb, (void *)X, (void *)D, (void *)Phi, (void *)Ref, (void *)tmp}) std::free(q);
                            }
                            stage_runs++;
                        }
                        // sampling and repetition helpers of the oracle, repetition of the library
                        const int64_t pick[3] = {o->n_round - 1, 0, o->n_round / 2};
                        orc_plan *sub = orc_plan_select_rounds(o, pick, 3);
                        if (!sub || std::memcmp(sub->round_member + r1, o->round_member, sizeof(int) * r1))
                            return fail("select_rounds", K, r, c, m, jobs);
                        orc_plan_free(sub);
                        if (jobs) {
                            orc_plan *rep = orc_plan_repeat(o, 2);
                            ccdc_plan_t *p2 = nullptr;
                            if (!rep || ccdc::build_plan(K, r, Q, N, true, 2, &p2) != CCDC_OK) return fail("repeat", K, r, c, m, jobs);
                            if (p2->nround != rep->n_round ||
                                std::memcmp(p2->round_batch.data(), rep->round_batch, sizeof(int) * rep->n_round * r1))
                                return fail("repeated tables", K, r, c, m, jobs);
                            orc_plan_free(rep);
                            delete p2;
                        }
                        orc_plan_free(o);
                        delete p;
                    }
    // compression-only comparison scheme
    long cplans = 0;
    for (int K = 2; K <= kmax + 2; K++)
        for (int r = 1; r < K; r++) {
            const int N = 2 * K * (K - 1) * r;               // mu*N whole for every r, even
            ccdc_plan_t *p = nullptr;
            orc_cplan *o = orc_cplan_build(K, r, K, N);
            const int rc = ccdc::build_compression_plan(K, r, K, N, &p);
            if ((rc == CCDC_OK) != (o != nullptr)) return fail("compression plan accepted by one side only", K, r, 1, 0, 0);
            if (!o) continue;
            cplans++;
            if (p->nrows != o->n_packet || std::memcmp(p->pkt_send.data(), o->pkt_send, sizeof(int) * o->n_packet) ||
                std::memcmp(p->pkt_batch.data(), o->pkt_batch, sizeof(int) * o->n_packet))
                return fail("compression tables", K, r, 1, 0, 0);
            for (int64_t T : {1, 5, 8}) {
                if (ccdc::bind_plan(p, T, CCDC_U32_XOR) != CCDC_OK) return fail("compression bind", K, r, 1, 0, 0);
                const size_t nv = (size_t)N * K * T, np = (size_t)o->n_packet * T, nphi = (size_t)K * T;
                uint32_t *V = exact<uint32_t>(nv), *P = exact<uint32_t>(np), *Phi = exact<uint32_t>(nphi);
                for (size_t i = 0; i < nv; i++) V[i] = (uint32_t)(i * 40503u);
                orc_ccombine_u32(o, T, V, P);
                orc_creduce_u32(o, T, V, P, Phi);
                float *Vf = exact<float>(nv);
                double *Pf = exact<double>(np), *Phif = exact<double>(nphi);
                for (size_t i = 0; i < nv; i++) Vf[i] = (float)(i % 17);
                orc_ccombine_f64(o, T, Vf, Pf);
                orc_creduce_f64(o, T, Vf, Pf, Phif);
                for (void *q : {(void *)V, (void *)P, (void *)Phi, (void *)Vf, (void *)Pf, (void *)Phif}) std::free(q);
            }
            orc_cplan_free(o);
            delete p;
        }
    std::printf("clean: %ld plans, %ld stage runs in 5 algebras, %ld compression plans\n", plans, stage_runs, cplans);
    return 0;
}
