// bf16 backward ring step for gfx950: one workgroup (4 wavefronts) per (128-key tile, kv head).
//
// The workgroup keeps its K and V rows in registers as MFMA operands and its dK / dV tiles in
// accumulators while it sweeps the q tiles (64 rows) of every q head of the GQA group that can see
// the key tile.  Per q tile: S = Q K^T and dP = dO V^T (keys across lanes, query rows in-lane),
// P = exp2(S*scale*log2e - LSE*log2e) from the saved global LSE, dS = P (dP - Delta); the
// accumulator registers holding P and dS are already in operand order for dV += P^T dO and
// dK += dS^T Q (dO and Q fetched with transposed LDS reads).  dS is written to LDS once (bf16,
// transposed) to be re-read as the A operand of dQ = dS K, which goes out through fp32 atomics.
#include "hexi_internal.h"
#include "hexi_mfma.h"

namespace {

constexpr int D = 128;
constexpr int TN = 128;          // keys per workgroup (32 per wavefront)
constexpr int TM = 64;           // q rows per inner tile
constexpr int QSTR = D + 8;      // LDS row stride of Q / dO / K staging (elements)
constexpr int SSTR = TM + 8;     // LDS row stride of dS^T [key][q row]
constexpr float LOG2E = 1.4426950408889634f;

__global__ void __launch_bounds__(256) bwd_bf16_kernel(const BwdArgs a)
{
    const AttnGeom& g = a.g;
    __shared__ __attribute__((aligned(16))) uint16_t Qs[TM * QSTR];
    __shared__ __attribute__((aligned(16))) uint16_t Gs[TM * QSTR];      // dO tile
    __shared__ __attribute__((aligned(16))) uint16_t dSt[TN * SSTR];     // dS^T, bf16
    __shared__ __attribute__((aligned(16))) uint16_t Kst[TN * QSTR];     // K staging (start of kernel only)
    __shared__ __attribute__((aligned(16))) float lse_s[TM];
    __shared__ __attribute__((aligned(16))) float delta_s[TM];
    __shared__ __attribute__((aligned(16))) int qpos_s[TM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int grp2 = (lane >> 4) & 1, j16 = lane & 15;
    const int kvh = blockIdx.y;
    const int col0 = blockIdx.x * TN;
    const int my_col = col0 + 32 * wave + l32;
    const int my_col_c = my_col < g.lc ? my_col : g.lc - 1;
    const int my_kpos = my_col < g.lc ? seg_pos_of_row(g.ks, my_col) : 0x7fffffff;

    const uint16_t* q = static_cast<const uint16_t*>(a.q);
    const uint16_t* go = static_cast<const uint16_t*>(a.d_o);
    const uint16_t* k = static_cast<const uint16_t*>(a.k) + (long long)kvh * g.kv_stride_head;
    const uint16_t* v = static_cast<const uint16_t*>(a.v) + (long long)kvh * g.kv_stride_head;

    // q rows that see at least one key of the tile form a suffix of the shard; rows that see all of
    // its keys form a (shorter) suffix
    const int last_col = (col0 + TN < g.lc ? col0 + TN : g.lc) - 1;
    const int k_min = seg_pos_of_row(g.ks, col0), k_max = seg_pos_of_row(g.ks, last_col);
    const int first_row = seg_rows_le(g.qs, k_min - 1);
    const int first_full_row = seg_rows_le(g.qs, k_max - 1);
    const int qt_begin = first_row / TM;
    const int qt_full = (col0 + TN <= g.lc) ? (first_full_row + TM - 1) / TM : 0x7fffffff;
    const int n_qtiles = (g.lq + TM - 1) / TM;

    // K^T and V^T operand fragments of S = Q K^T and dP = dO V^T: lane (key l32, half hh) holds
    // d = 16*ks + 8*hh .. +7 of its key
    bf16x8 kf[8], vf[8];
    {
        const long long off = (long long)my_col_c * g.kv_stride_tok + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            kf[ks] = *reinterpret_cast<const bf16x8*>(k + off + 16 * ks);
            vf[ks] = *reinterpret_cast<const bf16x8*>(v + off + 16 * ks);
        }
    }
    // K operand fragments of dQ = dS K for this wavefront's 32 output columns d = 32*wave + l32:
    // slot (hh, e) of step u is key 16*u + 8*hh + e, fetched transposed from the staged tile
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
        const int r = (tid >> 4) + 16 * pass, c = tid & 15;
        const int col = col0 + r < g.lc ? col0 + r : g.lc - 1;
        *reinterpret_cast<uint4*>(&Kst[r * QSTR + c * 8]) = *reinterpret_cast<const uint4*>(k + (long long)col * g.kv_stride_tok + c * 8);
    }
    __syncthreads();
    bf16x8 kq[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const uint16_t* p = &Kst[(16 * u + 8 * hh + (j16 >> 2)) * QSTR + 32 * wave + 16 * grp2 + 4 * (j16 & 3)];
        kq[u] = lds_tr_pair(p, p + 4 * QSTR);
    }

    f32x16 dk_acc[4], dv_acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk_acc[db][r] = 0.f; dv_acc[db][r] = 0.f; }
    const float scale_log2 = g.scale * LOG2E;

    for (int h = 0; h < g.nq; ++h) {
        if (g.kv_of_q[h] != kvh) continue;
        for (int qt = qt_begin; qt < n_qtiles; ++qt) {
            const int row0 = qt * TM;
            const bool partial = qt < qt_full;
            __syncthreads();
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int r = (tid >> 4) + 16 * pass, c = tid & 15;
                const int row = row0 + r < g.lq ? row0 + r : g.lq - 1;
                const long long off = (long long)row * g.q_stride_tok + (long long)h * g.q_stride_head + c * 8;
                const uint4 qx = *reinterpret_cast<const uint4*>(q + off);
                const uint4 gx = *reinterpret_cast<const uint4*>(go + off);
                *reinterpret_cast<uint4*>(&Qs[r * QSTR + c * 8]) = qx;
                *reinterpret_cast<uint4*>(&Gs[r * QSTR + c * 8]) = gx;
            }
            if (tid < TM) {
                const bool ok = row0 + tid < g.lq;
                const float l = ok ? a.lse[(long long)h * g.lq + row0 + tid] : INFINITY;
                lse_s[tid] = (l == -INFINITY) ? INFINITY : l * LOG2E;   // rows that see nothing: P = 0
                delta_s[tid] = ok ? a.delta[(long long)h * g.lq + row0 + tid] : 0.f;
                qpos_s[tid] = ok ? seg_pos_of_row(g.qs, row0 + tid) : -1;
            }
            __syncthreads();

            // S[q][key] and dP[q][key]: two 32-row q blocks, this wavefront's 32 keys
            f32x16 s[2], dp[2];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) { s[b][r] = 0.f; dp[b][r] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const bf16x8 qa = *reinterpret_cast<const bf16x8*>(&Qs[(32 * b + l32) * QSTR + 16 * ks + 8 * hh]);
                    const bf16x8 ga = *reinterpret_cast<const bf16x8*>(&Gs[(32 * b + l32) * QSTR + 16 * ks + 8 * hh]);
                    s[b] = mfma32(qa, kf[ks], s[b]);
                    dp[b] = mfma32(ga, vf[ks], dp[b]);
                }
            }
            // P and dS in place (s <- P, dp <- dS); in-lane row index i = 32*b + 8*(r/4) + 4*hh + r%4
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const int i0 = 32 * b + 8 * rb + 4 * hh;
                    const f32x4 l4 = *reinterpret_cast<const f32x4*>(&lse_s[i0]);
                    const f32x4 d4 = *reinterpret_cast<const f32x4*>(&delta_s[i0]);
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        float p = fast_exp2(s[b][4 * rb + t] * scale_log2 - l4[t]);
                        if (partial && my_kpos > qpos_s[i0 + t]) p = 0.f;
                        s[b][4 * rb + t] = p;
                        dp[b][4 * rb + t] = p * (dp[b][4 * rb + t] - d4[t]);
                    }
                }
            // dS^T to LDS for the dQ product: row = key, 4 consecutive q rows per 8-byte store
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    bf16x4 w;
#pragma unroll
                    for (int t = 0; t < 4; ++t) w[t] = (__bf16)dp[b][4 * rb + t];
                    *reinterpret_cast<bf16x4*>(&dSt[(32 * wave + l32) * SSTR + 32 * b + 8 * rb + 4 * hh]) = w;
                }
            // dV += P^T dO, dK += dS^T Q over four 16-row steps
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int b = u >> 1, x = (u & 1) * 8;
                const bf16x8 pf = pack_bf16x8(s[b][x], s[b][x + 1], s[b][x + 2], s[b][x + 3], s[b][x + 4], s[b][x + 5], s[b][x + 6], s[b][x + 7]);
                const bf16x8 df = pack_bf16x8(dp[b][x], dp[b][x + 1], dp[b][x + 2], dp[b][x + 3], dp[b][x + 4], dp[b][x + 5], dp[b][x + 6], dp[b][x + 7]);
                const int roff = (16 * u + 4 * hh + (j16 >> 2)) * QSTR + 16 * grp2 + 4 * (j16 & 3);
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const bf16x8 gf = lds_tr_pair(&Gs[roff + 32 * db], &Gs[roff + 32 * db + 8 * QSTR]);
                    dv_acc[db] = mfma32(pf, gf, dv_acc[db]);
                    const bf16x8 qf = lds_tr_pair(&Qs[roff + 32 * db], &Qs[roff + 32 * db + 8 * QSTR]);
                    dk_acc[db] = mfma32(df, qf, dk_acc[db]);
                }
            }
            __syncthreads();
            // dQ[q][d] for d = 32*wave + l32: contraction over all 128 keys of the tile
            f32x16 dq[2];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) dq[b][r] = 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const uint16_t* p = &dSt[(16 * u + 8 * hh + (j16 >> 2)) * SSTR + 32 * b + 16 * grp2 + 4 * (j16 & 3)];
                    const bf16x8 sf = lds_tr_pair(p, p + 4 * SSTR);
                    dq[b] = mfma32(sf, kq[u], dq[b]);
                }
            }
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = row0 + 32 * b + 8 * (r >> 2) + 4 * hh + (r & 3);
                    if (row < g.lq) unsafeAtomicAdd(a.dq + ((long long)row * g.nq + h) * D + 32 * wave + l32, dq[b][r] * g.scale);
                }
        }
    }

    // dK / dV: lane holds column d = 32*db + l32; register r holds key 32*wave + 8*(r/4) + 4*hh + r%4
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int col = col0 + 32 * wave + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (col < g.lc) {
                const long long idx = ((long long)col * g.nkv + kvh) * D + 32 * db + l32;
                const float kk = dk_acc[db][r] * g.scale, vv = dv_acc[db][r];
                if (a.accumulate) { a.dk[idx] += kk; a.dv[idx] += vv; } else { a.dk[idx] = kk; a.dv[idx] = vv; }
            }
        }
}

}  // namespace

hipError_t hexi_launch_bwd_bf16(const BwdArgs& a, hipStream_t s)
{
    dim3 grid((a.g.lc + TN - 1) / TN, a.g.nkv);
    bwd_bf16_kernel<<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}
