/*
 * hexi_oracle.c -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * Plain, slow, fp64 CPU definition of what one device's share of context-parallel causal
 * attention computes (HexiSeq, Sec. 3.2 and App. A.4: a local query block of L_G(d) tokens and
 * n_d heads attends to source KV blocks of L_Gsrc(t) tokens, Eq. 10-11; attention work is
 * forward + backward + recomputation, App. A.1).  The paper states no attention formula: it
 * presupposes ordinary softmax attention and promises that its sharding preserves those semantics
 * (Sec. 1, Sec. 3.2), so the oracle is the textbook definition written out -- no tiling, no online
 * softmax, no chunking, nothing reordered.  Only tests, the smoke check and the bench's cpu_baseline
 * leg may call it.  It shares no code, header, table or helper with the HIP library.
 *
 * Conventions (readings where the paper is silent):
 *   - causal mask on GLOBAL token positions, diagonal inclusive: key j is visible to query i
 *     iff kv_pos[j] <= q_pos[i];
 *   - grouped-query attention: local q head h reads local kv head kv_of_q[h];
 *   - LSE is the natural log of the sum of exp of the scaled scores; a row with no visible key
 *     has LSE = -inf and O = 0.
 *
 * Layouts (all row-major, fp64): q, o, d_o, dq: [Lq][nq][d];  k, v, dk, dv: [Lk][nkv][d];
 * lse, delta: [nq][Lq];  q_pos: [Lq], kv_pos: [Lk] global token positions (int64).
 *
 * Every function here is pinned by tests/test_oracle_pins.py (closed forms, invariants, finite
 * differences, brute force, a library cross-check); none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double dot(const double* a, const double* b, int d)
{
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += a[c] * b[c];
    return s;
}

/* Scaled scores of one (row, head) against every key; invisible keys get -inf.
 * Returns LSE = ln sum_j exp(s_j), evaluated as max + ln sum exp(s - max). */
static double row_scores_and_lse(const double* q_ih, int64_t pos_i, int64_t Lk, int nkv, int d,
                                 const double* k, const int64_t* kv_pos, int g, double scale,
                                 double* s /* [Lk] */)
{
    double m = -INFINITY;
    for (int64_t j = 0; j < Lk; ++j) {
        if (kv_pos[j] <= pos_i) {
            s[j] = scale * dot(q_ih, k + (j * nkv + g) * (int64_t)d, d);
            if (s[j] > m) m = s[j];
        } else {
            s[j] = -INFINITY;
        }
    }
    if (m == -INFINITY) return -INFINITY;
    double l = 0.0;
    for (int64_t j = 0; j < Lk; ++j)
        if (s[j] != -INFINITY) l += exp(s[j] - m);
    return m + log(l);
}

/* Forward: O_i = sum_j P_ij v_j,  P_ij = exp(s_ij - LSE_i),  s_ij = scale <q_i, k_j>, over the keys
 * visible to row i.  Passing one chunk's keys gives that chunk's normalised partial result. */
void oracle_attn_fwd(int64_t Lq, int nq, int d, const double* q, const int64_t* q_pos,
                     int64_t Lk, int nkv, const double* k, const double* v, const int64_t* kv_pos,
                     const int32_t* kv_of_q, double scale, double* o, double* lse)
{
#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)(Lk > 0 ? Lk : 1));
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int64_t i = 0; i < Lq; ++i) {
            for (int h = 0; h < nq; ++h) {
                const int g = kv_of_q[h];
                const double* q_ih = q + (i * nq + h) * (int64_t)d;
                double* o_ih = o + (i * nq + h) * (int64_t)d;
                const double L = row_scores_and_lse(q_ih, q_pos[i], Lk, nkv, d, k, kv_pos, g, scale, s);
                lse[(int64_t)h * Lq + i] = L;
                for (int c = 0; c < d; ++c) o_ih[c] = 0.0;
                if (L == -INFINITY) continue;
                for (int64_t j = 0; j < Lk; ++j) {
                    if (s[j] == -INFINITY) continue;
                    const double p = exp(s[j] - L);
                    const double* v_j = v + (j * nkv + g) * (int64_t)d;
                    for (int c = 0; c < d; ++c) o_ih[c] += p * v_j[c];
                }
            }
        }
        free(s);
    }
}

/* Backward of the scalar loss sum_{i,h} <O_ih, dO_ih> with respect to q, k, v:
 *   Delta_i = <dO_i, O_i>;  dP_ij = <dO_i, v_j>;  dS_ij = P_ij (dP_ij - Delta_i);
 *   dQ_i = scale sum_j dS_ij k_j;  dK_j = scale sum_{h in group} sum_i dS_ij q_i;
 *   dV_j = sum_{h in group} sum_i P_ij dO_i.
 * Everything is recomputed from q, k, v by definition; lse and delta ([nq][Lq]) are also returned.
 * dk, dv hold only the contribution of the Lq query rows given here. */
void oracle_attn_bwd(int64_t Lq, int nq, int d, const double* q, const int64_t* q_pos,
                     int64_t Lk, int nkv, const double* k, const double* v, const int64_t* kv_pos,
                     const int32_t* kv_of_q, double scale, const double* d_o,
                     double* dq, double* dk, double* dv, double* lse, double* delta)
{
    /* pass A, one (row, head) at a time: LSE, O, Delta and the row-local gradient dQ */
#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)(Lk > 0 ? Lk : 1));
        double* o_ih = (double*)malloc(sizeof(double) * (size_t)d);
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int64_t i = 0; i < Lq; ++i) {
            for (int h = 0; h < nq; ++h) {
                const int g = kv_of_q[h];
                const double* q_ih = q + (i * nq + h) * (int64_t)d;
                const double* do_ih = d_o + (i * nq + h) * (int64_t)d;
                double* dq_ih = dq + (i * nq + h) * (int64_t)d;
                const double L = row_scores_and_lse(q_ih, q_pos[i], Lk, nkv, d, k, kv_pos, g, scale, s);
                lse[(int64_t)h * Lq + i] = L;
                for (int c = 0; c < d; ++c) { o_ih[c] = 0.0; dq_ih[c] = 0.0; }
                if (L != -INFINITY)
                    for (int64_t j = 0; j < Lk; ++j) {
                        if (s[j] == -INFINITY) continue;
                        const double p = exp(s[j] - L);
                        const double* v_j = v + (j * nkv + g) * (int64_t)d;
                        for (int c = 0; c < d; ++c) o_ih[c] += p * v_j[c];
                    }
                const double Dl = dot(do_ih, o_ih, d);
                delta[(int64_t)h * Lq + i] = Dl;
                if (L == -INFINITY) continue;
                for (int64_t j = 0; j < Lk; ++j) {
                    if (s[j] == -INFINITY) continue;
                    const double p = exp(s[j] - L);
                    const double dp = dot(do_ih, v + (j * nkv + g) * (int64_t)d, d);
                    const double ds = p * (dp - Dl);
                    const double* k_j = k + (j * nkv + g) * (int64_t)d;
                    for (int c = 0; c < d; ++c) dq_ih[c] += scale * ds * k_j[c];
                }
            }
        }
        free(s);
        free(o_ih);
    }
    /* pass B, one (key, kv head) at a time: dK_j and dV_j, summed over the q heads of the group */
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t j = 0; j < Lk; ++j) {
        for (int g = 0; g < nkv; ++g) {
            const double* k_j = k + (j * nkv + g) * (int64_t)d;
            const double* v_j = v + (j * nkv + g) * (int64_t)d;
            double* dk_j = dk + (j * nkv + g) * (int64_t)d;
            double* dv_j = dv + (j * nkv + g) * (int64_t)d;
            for (int c = 0; c < d; ++c) { dk_j[c] = 0.0; dv_j[c] = 0.0; }
            for (int h = 0; h < nq; ++h) {
                if (kv_of_q[h] != g) continue;
                for (int64_t i = 0; i < Lq; ++i) {
                    if (!(kv_pos[j] <= q_pos[i])) continue;
                    const double* q_ih = q + (i * nq + h) * (int64_t)d;
                    const double* do_ih = d_o + (i * nq + h) * (int64_t)d;
                    const double sij = scale * dot(q_ih, k_j, d);
                    const double p = exp(sij - lse[(int64_t)h * Lq + i]);
                    const double dp = dot(do_ih, v_j, d);
                    const double ds = p * (dp - delta[(int64_t)h * Lq + i]);
                    for (int c = 0; c < d; ++c) {
                        dv_j[c] += p * do_ih[c];
                        dk_j[c] += scale * ds * q_ih[c];
                    }
                }
            }
        }
    }
}

/* Delta_ih = <dO_ih, O_ih>  (the row term of the softmax Jacobian), layout [nq][Lq]. */
void oracle_delta(int64_t Lq, int nq, int d, const double* o, const double* d_o, double* delta)
{
    for (int64_t i = 0; i < Lq; ++i)
        for (int h = 0; h < nq; ++h)
            delta[(int64_t)h * Lq + i] = dot(o + (i * nq + h) * (int64_t)d, d_o + (i * nq + h) * (int64_t)d, d);
}

/* Combine two normalised partial results over disjoint key sets a and b:
 *   LSE = ln(e^LSE_a + e^LSE_b);  O = e^(LSE_a - LSE) O_a + e^(LSE_b - LSE) O_b.
 * -inf (empty key set) is the identity; two empty sets stay (LSE = -inf, O = 0). */
void oracle_merge(int64_t n_rows, int nq, int d, const double* o_a, const double* lse_a,
                  const double* o_b, const double* lse_b, double* o_out, double* lse_out)
{
    for (int64_t i = 0; i < n_rows; ++i)
        for (int h = 0; h < nq; ++h) {
            const double a = lse_a[(int64_t)h * n_rows + i], b = lse_b[(int64_t)h * n_rows + i];
            const double m = a > b ? a : b;
            double* oo = o_out + (i * nq + h) * (int64_t)d;
            if (m == -INFINITY) {
                lse_out[(int64_t)h * n_rows + i] = -INFINITY;
                for (int c = 0; c < d; ++c) oo[c] = 0.0;
                continue;
            }
            const double L = m + log(exp(a - m) + exp(b - m));
            const double wa = exp(a - L), wb = exp(b - L);
            lse_out[(int64_t)h * n_rows + i] = L;
            const double* oa = o_a + (i * nq + h) * (int64_t)d;
            const double* ob = o_b + (i * nq + h) * (int64_t)d;
            for (int c = 0; c < d; ++c) oo[c] = wa * oa[c] + wb * ob[c];
        }
}

/* Global positions of the packed rows of a shard given as segments [start, start+len). */
void oracle_positions(int n_segs, const int64_t* seg_start, const int64_t* seg_len, int64_t* pos)
{
    int64_t r = 0;
    for (int s = 0; s < n_segs; ++s)
        for (int64_t t = 0; t < seg_len[s]; ++t) pos[r++] = seg_start[s] + t;
}

/* Brute-force mask bookkeeping: for every (tile_m x tile_n) tile of the Lq x Lk pair grid, count the
 * visible pairs one by one; class 0 = none visible (EMPTY), 1 = all visible (FULL), 2 = some
 * (PARTIAL).  Tiles are clipped at the ragged edge.  Returns the total number of visible pairs. */
int64_t oracle_mask_bruteforce(int64_t Lq, const int64_t* q_pos, int64_t Lk, const int64_t* kv_pos,
                               int tile_m, int tile_n, uint8_t* tile_class)
{
    const int64_t nm = (Lq + tile_m - 1) / tile_m, nn = (Lk + tile_n - 1) / tile_n;
    int64_t total = 0;
    for (int64_t tm = 0; tm < nm; ++tm)
        for (int64_t tn = 0; tn < nn; ++tn) {
            int64_t vis = 0, all = 0;
            for (int64_t i = tm * tile_m; i < (tm + 1) * tile_m && i < Lq; ++i)
                for (int64_t j = tn * tile_n; j < (tn + 1) * tile_n && j < Lk; ++j) {
                    ++all;
                    if (kv_pos[j] <= q_pos[i]) ++vis;
                }
            total += vis;
            if (tile_class) tile_class[tm * nn + tn] = vis == 0 ? 0 : (vis == all ? 1 : 2);
        }
    return total;
}
