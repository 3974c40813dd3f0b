// fp32 path (no reduced precision anywhere): LDS-tiled plain-FMA kernels for the parity
// configuration with fp32 inputs.  Forward: one workgroup per (64-row q tile, q head), online
// softmax over 64-key tiles.  Backward: one workgroup per (64-key tile, kv head), looping over the
// group's q heads and 32-row q tiles, P recomputed from the saved global LSE; dQ goes out through
// fp32 atomics, dK/dV stay in registers until the end.
#include "hexi_internal.h"

namespace {

constexpr int TQ_F = 64;   // forward q rows per workgroup
constexpr int TK = 64;     // keys per tile (both passes)
constexpr int TQ_B = 32;   // backward q rows per inner tile

template <int D>
__global__ void __launch_bounds__(256) fwd_f32_kernel(const FwdArgs a)
{
    const AttnGeom& g = a.g;
    __shared__ float Qs[TQ_F][D + 1];
    __shared__ float Ks[TK][D + 1];
    __shared__ float Vs[TK][D];
    __shared__ float Ss[TQ_F][TK + 1];
    __shared__ int qpos_s[TQ_F];
    __shared__ int kpos_s[TK];

    const int t = threadIdx.x;
    const int h = blockIdx.y;
    const int kvh = g.kv_of_q[h];
    const int row0 = blockIdx.x * TQ_F;
    const float* q = static_cast<const float*>(a.q);
    const float* k = static_cast<const float*>(a.k);
    const float* v = static_cast<const float*>(a.v);

    if (t < TQ_F) qpos_s[t] = (row0 + t < g.lq) ? seg_pos_of_row(g.qs, row0 + t) : -1;
    for (int idx = t; idx < TQ_F * (D / 4); idx += 256) {
        const int r = idx / (D / 4), c = (idx % (D / 4)) * 4;
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row0 + r < g.lq) x = *reinterpret_cast<const float4*>(q + (long long)(row0 + r) * g.q_stride_tok + (long long)h * g.q_stride_head + c);
        Qs[r][c] = x.x; Qs[r][c + 1] = x.y; Qs[r][c + 2] = x.z; Qs[r][c + 3] = x.w;
    }
    const int last_row = (row0 + TQ_F < g.lq ? row0 + TQ_F : g.lq) - 1;
    const int q_max = seg_pos_of_row(g.qs, last_row);
    const int n_vis = seg_rows_le(g.ks, q_max);           // visible columns form the prefix [0, n_vis)
    const int n_tiles = (n_vis + TK - 1) / TK;

    // softmax / PV mapping: 4 adjacent lanes share a row, each owns D/4 output columns
    const int r = t >> 2, c4 = t & 3;
    constexpr int DS = D / 4;
    float acc[DS];
#pragma unroll
    for (int c = 0; c < DS; ++c) acc[c] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    // score mapping: 4 rows x 4 interleaved columns per thread
    const int ty = t >> 4, tx = t & 15;

    for (int tile = 0; tile < n_tiles; ++tile) {
        const int col0 = tile * TK;
        __syncthreads();
        if (t < TK) kpos_s[t] = (col0 + t < g.lc) ? seg_pos_of_row(g.ks, col0 + t) : 0x7fffffff;
        for (int idx = t; idx < TK * (D / 4); idx += 256) {
            const int j = idx / (D / 4), c = (idx % (D / 4)) * 4;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f), y = x;
            if (col0 + j < g.lc) {
                const long long off = (long long)(col0 + j) * g.kv_stride_tok + (long long)kvh * g.kv_stride_head + c;
                x = *reinterpret_cast<const float4*>(k + off);
                y = *reinterpret_cast<const float4*>(v + off);
            }
            Ks[j][c] = x.x; Ks[j][c + 1] = x.y; Ks[j][c + 2] = x.z; Ks[j][c + 3] = x.w;
            *reinterpret_cast<float4*>(&Vs[j][c]) = y;
        }
        __syncthreads();
        float s[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) s[i][j] = 0.f;
        for (int c = 0; c < D; ++c) {
            float qa[4], kb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) qa[i] = Qs[ty * 4 + i][c];
#pragma unroll
            for (int j = 0; j < 4; ++j) kb[j] = Ks[tx + 16 * j][c];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) s[i][j] = fmaf(qa[i], kb[j], s[i][j]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int rr = ty * 4 + i, cc = tx + 16 * j;
                Ss[rr][cc] = (kpos_s[cc] <= qpos_s[rr]) ? s[i][j] * g.scale : -INFINITY;
            }
        __syncthreads();
        // online softmax for row r: this lane covers columns c4, c4+4, ...
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < TK / 4; ++j) mx = fmaxf(mx, Ss[r][c4 + 4 * j]);
        mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        float ps = 0.f;
#pragma unroll
        for (int j = 0; j < TK / 4; ++j) {
            const float p = expf(Ss[r][c4 + 4 * j] - m_use);
            Ss[r][c4 + 4 * j] = p;
            ps += p;
        }
        ps += __shfl_xor(ps, 1, 64);
        ps += __shfl_xor(ps, 2, 64);
        const float alpha = expf(m_run - m_use);   // m_run = -inf -> 0
        l_run = l_run * alpha + ps;
        m_run = m_new;
        __syncthreads();
#pragma unroll
        for (int c = 0; c < DS; ++c) acc[c] *= alpha;
        for (int j = 0; j < TK; ++j) {
            const float p = Ss[r][j];
#pragma unroll
            for (int c = 0; c < DS; ++c) acc[c] = fmaf(p, Vs[j][c4 * DS + c], acc[c]);
        }
    }

    const int row = row0 + r;
    if (row >= g.lq) return;
    float lse_new;
    if (l_run > 0.f) {
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int c = 0; c < DS; ++c) acc[c] *= inv;
        lse_new = m_run + logf(l_run);
    } else {
        lse_new = -INFINITY;
    }
    float* op = a.o + ((long long)row * g.nq + h) * D + c4 * DS;
    float* lp = a.lse + (long long)h * g.lq + row;
    if (a.accumulate) {
        const float la = *lp;
        const float m = fmaxf(la, lse_new);
        if (m == -INFINITY) {
#pragma unroll
            for (int c = 0; c < DS; ++c) acc[c] = 0.f;
        } else {
            const float ea = expf(la - m), eb = expf(lse_new - m);
            const float inv = 1.0f / (ea + eb);
#pragma unroll
            for (int c = 0; c < DS; ++c) acc[c] = (ea * inv) * op[c] + (eb * inv) * acc[c];
            lse_new = m + logf(ea + eb);
        }
    }
#pragma unroll
    for (int c = 0; c < DS; c += 4) *reinterpret_cast<float4*>(op + c) = make_float4(acc[c], acc[c + 1], acc[c + 2], acc[c + 3]);
    // the 4 lanes of a row all read *lp above (same wavefront instruction) before lane c4==0 writes it
    if (c4 == 0) *lp = lse_new;
}

template <int D>
__global__ void __launch_bounds__(256) bwd_f32_kernel(const BwdArgs a)
{
    const AttnGeom& g = a.g;
    __shared__ float Ks[TK][D + 1];
    __shared__ float Vs[TK][D + 1];
    __shared__ float Qs[TQ_B][D + 1];
    __shared__ float Gs[TQ_B][D + 1];      // dO tile
    __shared__ float Ps[TQ_B][TK + 1];
    __shared__ float dSs[TQ_B][TK + 1];
    __shared__ float lse_s[TQ_B], delta_s[TQ_B];
    __shared__ int qpos_s[TQ_B];
    __shared__ int kpos_s[TK];

    const int t = threadIdx.x;
    const int kvh = blockIdx.y;
    const int col0 = blockIdx.x * TK;
    const float* q = static_cast<const float*>(a.q);
    const float* k = static_cast<const float*>(a.k);
    const float* v = static_cast<const float*>(a.v);
    const float* go = static_cast<const float*>(a.d_o);

    if (t < TK) kpos_s[t] = (col0 + t < g.lc) ? seg_pos_of_row(g.ks, col0 + t) : 0x7fffffff;
    for (int idx = t; idx < TK * (D / 4); idx += 256) {
        const int j = idx / (D / 4), c = (idx % (D / 4)) * 4;
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f), y = x;
        if (col0 + j < g.lc) {
            const long long off = (long long)(col0 + j) * g.kv_stride_tok + (long long)kvh * g.kv_stride_head + c;
            x = *reinterpret_cast<const float4*>(k + off);
            y = *reinterpret_cast<const float4*>(v + off);
        }
        Ks[j][c] = x.x; Ks[j][c + 1] = x.y; Ks[j][c + 2] = x.z; Ks[j][c + 3] = x.w;
        Vs[j][c] = y.x; Vs[j][c + 1] = y.y; Vs[j][c + 2] = y.z; Vs[j][c + 3] = y.w;
    }
    const int k_min = seg_pos_of_row(g.ks, col0);
    const int first_row = seg_rows_le(g.qs, k_min - 1);   // rows before it see nothing of this tile
    const int tile_begin = first_row / TQ_B;
    const int n_qtiles = (g.lq + TQ_B - 1) / TQ_B;

    // dK/dV mapping: 4 adjacent lanes share key j, each owns D/4 columns
    const int j_own = t >> 2, c4 = t & 3;
    constexpr int DS = D / 4;
    float dk_acc[DS], dv_acc[DS];
#pragma unroll
    for (int c = 0; c < DS; ++c) { dk_acc[c] = 0.f; dv_acc[c] = 0.f; }
    // S/dP mapping: 2 rows x 4 interleaved columns per thread
    const int ty = t >> 4, tx = t & 15;
    // dQ mapping: 8 adjacent lanes share row i, each owns D/8 columns
    const int i_own = t >> 3, c8 = t & 7;
    constexpr int DQ = D / 8;

    for (int h = 0; h < g.nq; ++h) {
        if (g.kv_of_q[h] != kvh) continue;
        for (int qt = tile_begin; qt < n_qtiles; ++qt) {
            const int row0 = qt * TQ_B;
            __syncthreads();
            if (t < TQ_B) {
                const bool ok = row0 + t < g.lq;
                qpos_s[t] = ok ? seg_pos_of_row(g.qs, row0 + t) : -1;
                const float l = ok ? a.lse[(long long)h * g.lq + row0 + t] : INFINITY;
                lse_s[t] = (l == -INFINITY) ? INFINITY : l;   // a row with no visible key anywhere: P = 0
                delta_s[t] = ok ? a.delta[(long long)h * g.lq + row0 + t] : 0.f;
            }
            for (int idx = t; idx < TQ_B * (D / 4); idx += 256) {
                const int r = idx / (D / 4), c = (idx % (D / 4)) * 4;
                float4 x = make_float4(0.f, 0.f, 0.f, 0.f), y = x;
                if (row0 + r < g.lq) {
                    const long long off = (long long)(row0 + r) * g.q_stride_tok + (long long)h * g.q_stride_head + c;
                    x = *reinterpret_cast<const float4*>(q + off);
                    y = *reinterpret_cast<const float4*>(go + off);
                }
                Qs[r][c] = x.x; Qs[r][c + 1] = x.y; Qs[r][c + 2] = x.z; Qs[r][c + 3] = x.w;
                Gs[r][c] = y.x; Gs[r][c + 1] = y.y; Gs[r][c + 2] = y.z; Gs[r][c + 3] = y.w;
            }
            __syncthreads();
            float s[2][4], dp[2][4];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) { s[i][j] = 0.f; dp[i][j] = 0.f; }
            for (int c = 0; c < D; ++c) {
                float qa[2], ga[2], kb[4], vb[4];
#pragma unroll
                for (int i = 0; i < 2; ++i) { qa[i] = Qs[ty * 2 + i][c]; ga[i] = Gs[ty * 2 + i][c]; }
#pragma unroll
                for (int j = 0; j < 4; ++j) { kb[j] = Ks[tx + 16 * j][c]; vb[j] = Vs[tx + 16 * j][c]; }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) { s[i][j] = fmaf(qa[i], kb[j], s[i][j]); dp[i][j] = fmaf(ga[i], vb[j], dp[i][j]); }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int rr = ty * 2 + i, cc = tx + 16 * j;
                    const float p = (kpos_s[cc] <= qpos_s[rr]) ? expf(s[i][j] * g.scale - lse_s[rr]) : 0.f;
                    Ps[rr][cc] = p;
                    dSs[rr][cc] = p * (dp[i][j] - delta_s[rr]);
                }
            __syncthreads();
            for (int i = 0; i < TQ_B; ++i) {
                const float p = Ps[i][j_own], ds = dSs[i][j_own];
#pragma unroll
                for (int c = 0; c < DS; ++c) {
                    dv_acc[c] = fmaf(p, Gs[i][c4 * DS + c], dv_acc[c]);
                    dk_acc[c] = fmaf(ds, Qs[i][c4 * DS + c], dk_acc[c]);
                }
            }
            float dq[DQ];
#pragma unroll
            for (int c = 0; c < DQ; ++c) dq[c] = 0.f;
            for (int j = 0; j < TK; ++j) {
                const float ds = dSs[i_own][j];
#pragma unroll
                for (int c = 0; c < DQ; ++c) dq[c] = fmaf(ds, Ks[j][c8 * DQ + c], dq[c]);
            }
            if (a.want_dq && row0 + i_own < g.lq) {
                float* dqp = a.dq + ((long long)(row0 + i_own) * g.nq + h) * D + c8 * DQ;
#pragma unroll
                for (int c = 0; c < DQ; ++c) unsafeAtomicAdd(dqp + c, dq[c] * g.scale);
            }
        }
    }
    if (a.want_dkdv && col0 + j_own < g.lc) {
        float* dkp = a.dk + ((long long)(col0 + j_own) * g.nkv + kvh) * D + c4 * DS;
        float* dvp = a.dv + ((long long)(col0 + j_own) * g.nkv + kvh) * D + c4 * DS;
#pragma unroll
        for (int c = 0; c < DS; ++c) {
            const float kk = dk_acc[c] * g.scale, vv = dv_acc[c];
            if (a.accumulate) { dkp[c] += kk; dvp[c] += vv; } else { dkp[c] = kk; dvp[c] = vv; }
        }
    }
}

}  // namespace

hipError_t hexi_launch_fwd_f32(const FwdArgs& a, hipStream_t s)
{
    dim3 grid((a.g.lq + TQ_F - 1) / TQ_F, a.g.nq);
    if (a.g.d == 64) fwd_f32_kernel<64><<<grid, 256, 0, s>>>(a);
    else fwd_f32_kernel<128><<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}

hipError_t hexi_launch_bwd_f32(const BwdArgs& a, hipStream_t s)
{
    dim3 grid((a.g.lc + TK - 1) / TK, a.g.nkv);
    if (a.g.d == 64) bwd_f32_kernel<64><<<grid, 256, 0, s>>>(a);
    else bwd_f32_kernel<128><<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}
