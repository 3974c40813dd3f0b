/* The fp64 oracle (oracle/hexi_oracle.c, included as is) under AddressSanitizer and UndefinedBehaviorSanitizer:
 * a few small shards -- ragged lengths, several segments, rows that see nothing, GQA maps, single rows and keys -- go
 * through every entry point with exactly-sized heap buffers, and a few identities are checked on the results.
 * Prints "ok <checksum>"; any sanitizer report aborts the run. */
#include <stdio.h>
#include "../../oracle/hexi_oracle.c"

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static double rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return ((double)(rng_state >> 11) / 9007199254740992.0) * 2.0 - 1.0;
}
static double* rand_vec(size_t n)
{
    double* p = (double*)malloc(n * sizeof(double) + (n == 0));
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
#define REQUIRE(c) do { if (!(c)) { printf("FAILED %s line %d\n", #c, __LINE__); return 1; } } while (0)

static int run_case(int n_qseg, const int64_t* qs, const int64_t* ql, int n_kseg, const int64_t* ks, const int64_t* kl,
                    int nq, int nkv, int d, const int32_t* map, double* checksum)
{
    int64_t Lq = 0, Lk = 0;
    for (int i = 0; i < n_qseg; ++i) Lq += ql[i];
    for (int i = 0; i < n_kseg; ++i) Lk += kl[i];
    int64_t* q_pos = (int64_t*)malloc(Lq * sizeof(int64_t));
    int64_t* kv_pos = (int64_t*)malloc(Lk * sizeof(int64_t));
    oracle_positions(n_qseg, qs, ql, q_pos);
    oracle_positions(n_kseg, ks, kl, kv_pos);
    double *q = rand_vec((size_t)Lq * nq * d), *g = rand_vec((size_t)Lq * nq * d);
    double *k = rand_vec((size_t)Lk * nkv * d), *v = rand_vec((size_t)Lk * nkv * d);
    double *o = rand_vec((size_t)Lq * nq * d), *lse = rand_vec((size_t)Lq * nq);
    double *dq = rand_vec((size_t)Lq * nq * d), *dk = rand_vec((size_t)Lk * nkv * d), *dv = rand_vec((size_t)Lk * nkv * d);
    double *lse2 = rand_vec((size_t)Lq * nq), *delta = rand_vec((size_t)Lq * nq), *delta2 = rand_vec((size_t)Lq * nq);
    const double scale = 1.0 / sqrt((double)d);
    oracle_attn_fwd(Lq, nq, d, q, q_pos, Lk, nkv, k, v, kv_pos, map, scale, o, lse);
    oracle_attn_bwd(Lq, nq, d, q, q_pos, Lk, nkv, k, v, kv_pos, map, scale, g, dq, dk, dv, lse2, delta);
    oracle_delta(Lq, nq, d, o, g, delta2);
    for (int64_t i = 0; i < Lq * nq; ++i) {
        REQUIRE(lse[i] == lse2[i]);
        REQUIRE(fabs(delta[i] - delta2[i]) <= 1e-12 * (1.0 + fabs(delta[i])));
    }
    /* sum_j dV_j = sum over the rows that see at least one key of dO_i, per kv head */
    for (int kh = 0; kh < nkv; ++kh)
        for (int c = 0; c < d; ++c) {
            double a = 0.0, b = 0.0;
            for (int64_t j = 0; j < Lk; ++j) a += dv[(j * nkv + kh) * d + c];
            for (int64_t i = 0; i < Lq; ++i)
                for (int h = 0; h < nq; ++h)
                    if (map[h] == kh && lse[(int64_t)h * Lq + i] != -INFINITY) b += g[(i * nq + h) * d + c];
            REQUIRE(fabs(a - b) <= 1e-9 * (1.0 + fabs(b)));
        }
    /* merge of the partials over the two halves of the key set = the one-shot result */
    if (Lk >= 2) {
        const int64_t h1 = Lk / 2;
        double *oa = rand_vec((size_t)Lq * nq * d), *la = rand_vec((size_t)Lq * nq), *ob = rand_vec((size_t)Lq * nq * d), *lb = rand_vec((size_t)Lq * nq);
        double *om = rand_vec((size_t)Lq * nq * d), *lm = rand_vec((size_t)Lq * nq);
        oracle_attn_fwd(Lq, nq, d, q, q_pos, h1, nkv, k, v, kv_pos, map, scale, oa, la);
        oracle_attn_fwd(Lq, nq, d, q, q_pos, Lk - h1, nkv, k + h1 * nkv * d, v + h1 * nkv * d, kv_pos + h1, map, scale, ob, lb);
        oracle_merge(Lq, nq, d, oa, la, ob, lb, om, lm);
        for (int64_t i = 0; i < Lq * nq * d; ++i) REQUIRE(fabs(om[i] - o[i]) <= 1e-12);
        for (int64_t i = 0; i < Lq * nq; ++i) REQUIRE(lm[i] == lse[i] || fabs(lm[i] - lse[i]) <= 1e-12 * (1.0 + fabs(lse[i])));
        free(oa); free(la); free(ob); free(lb); free(om); free(lm);
    }
    /* tile classes and pair count at awkward tile sizes */
    for (int t = 0; t < 3; ++t) {
        const int tm = t == 0 ? 1 : (t == 1 ? 7 : 128), tn = t == 0 ? 1 : (t == 1 ? 5 : 64);
        const int64_t nm = (Lq + tm - 1) / tm, nn = (Lk + tn - 1) / tn;
        uint8_t* cls = (uint8_t*)malloc((size_t)(nm * nn) + 1);
        int64_t pairs = oracle_mask_bruteforce(Lq, q_pos, Lk, kv_pos, tm, tn, cls);
        int64_t want = 0;
        for (int64_t i = 0; i < Lq; ++i) for (int64_t j = 0; j < Lk; ++j) want += kv_pos[j] <= q_pos[i];
        REQUIRE(pairs == want);
        for (int64_t i = 0; i < nm * nn; ++i) REQUIRE(cls[i] <= 2);
        free(cls);
    }
    for (int64_t i = 0; i < Lq * nq * d; ++i) *checksum += o[i] + dq[i];
    for (int64_t i = 0; i < Lk * nkv * d; ++i) *checksum += dk[i] + dv[i];
    free(q_pos); free(kv_pos); free(q); free(g); free(k); free(v); free(o); free(lse); free(dq); free(dk); free(dv);
    free(lse2); free(delta); free(delta2);
    return 0;
}

int main(void)
{
    double checksum = 0.0;
    {   /* contiguous shard in the middle of the sequence, MHA */
        const int64_t qs[] = {40}, ql[] = {37}, ks[] = {0}, kl[] = {90};
        const int32_t map[] = {0, 1, 2};
        if (run_case(1, qs, ql, 1, ks, kl, 3, 3, 8, map, &checksum)) return 1;
    }
    {   /* zigzag pair against keys with holes; GQA with a non-default map; some rows see nothing */
        const int64_t qs[] = {5, 100}, ql[] = {13, 29}, ks[] = {10, 60, 110}, kl[] = {20, 17, 30};
        const int32_t map[] = {1, 0, 1, 1};
        if (run_case(2, qs, ql, 3, ks, kl, 4, 2, 16, map, &checksum)) return 1;
    }
    {   /* one row, one key; then one row that sees nothing at all */
        const int64_t qs[] = {7}, ql[] = {1}, ks[] = {7}, kl[] = {1}, ks2[] = {8};
        const int32_t map[] = {0};
        if (run_case(1, qs, ql, 1, ks, kl, 1, 1, 4, map, &checksum)) return 1;
        if (run_case(1, qs, ql, 1, ks2, kl, 1, 1, 4, map, &checksum)) return 1;
    }
    {   /* sixteen one-token segments */
        int64_t qs[16], ql[16], ks[16], kl[16];
        for (int i = 0; i < 16; ++i) { qs[i] = 3 * i + 1; ql[i] = 1; ks[i] = 3 * i; kl[i] = 2; }
        const int32_t map[] = {0, 0};
        if (run_case(16, qs, ql, 16, ks, kl, 2, 1, 8, map, &checksum)) return 1;
    }
    printf("ok %.12e threads %d\n", checksum, oracle_num_threads());
    return 0;
}
