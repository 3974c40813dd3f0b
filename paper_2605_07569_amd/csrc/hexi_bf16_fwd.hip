// bf16 forward ring step for gfx950: one workgroup (4 wavefronts) per (128-row q tile, q head).
//
// The scores are computed transposed, S^T = K Q^T, so that every lane owns one query row: the
// softmax state (running max, running sum) is a per-lane scalar, the row reductions are in-lane
// plus one exchange between the two half-waves, and the accumulator registers holding P^T are
// already in MFMA operand order for O^T += V^T P^T.  K is read from LDS with 128-bit reads, V^T with
// transposed LDS reads; Q stays in registers for the whole chunk.  KV tiles that lie wholly in the
// visible past of the q tile skip all masking; tiles wholly in the future are never visited.
#include "hexi_internal.h"
#include "hexi_mfma.h"

namespace {

constexpr int D = 128;
constexpr int TM = 128;          // q rows per workgroup (32 per wavefront)
constexpr int TN = 64;           // keys per tile
constexpr int KSTR = D + 8;      // LDS row stride of K (elements): 272 B, conflict-free 128-bit reads
constexpr int VSTR = D + 32;     // LDS row stride of V: 320 B, the 4 rows of a transposed read hit disjoint banks
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

__global__ void __launch_bounds__(256) fwd_bf16_kernel(const FwdArgs a)
{
    const AttnGeom& g = a.g;
    __shared__ __attribute__((aligned(16))) uint16_t Ks[TN * KSTR];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[TN * VSTR];
    __shared__ int kpos_s[TN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int grp2 = (lane >> 4) & 1, j16 = lane & 15;
    const int h = blockIdx.y;
    const int kvh = g.kv_of_q[h];
    const int row0 = blockIdx.x * TM;
    const int my_row = row0 + 32 * wave + l32;
    const int my_row_c = my_row < g.lq ? my_row : g.lq - 1;
    const int my_pos = my_row < g.lq ? seg_pos_of_row(g.qs, my_row) : -1;

    const uint16_t* q = static_cast<const uint16_t*>(a.q);
    const uint16_t* k = static_cast<const uint16_t*>(a.k) + (long long)kvh * g.kv_stride_head;
    const uint16_t* v = static_cast<const uint16_t*>(a.v) + (long long)kvh * g.kv_stride_head;

    // visible columns of this q tile form a prefix of the chunk; columns visible to every row of
    // the tile form a (shorter) prefix
    const int last_row = (row0 + TM < g.lq ? row0 + TM : g.lq) - 1;
    const int n_vis = seg_rows_le(g.ks, seg_pos_of_row(g.qs, last_row));
    const int n_all = seg_rows_le(g.ks, seg_pos_of_row(g.qs, row0));
    const int n_tiles = (n_vis + TN - 1) / TN;
    const int n_full_tiles = n_all / TN;

    // Q^T operand fragments: lane (row l32, half hh) holds d = 16*ks + 8*hh .. +7
    bf16x8 qf[8];
    {
        const uint16_t* qp = q + (long long)my_row_c * g.q_stride_tok + (long long)h * g.q_stride_head + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
    }

    f32x16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f, lr_run = 0.f;
    const float scale_log2 = g.scale * LOG2E;

    for (int tile = 0; tile < n_tiles; ++tile) {
        const int col0 = tile * TN;
        const bool partial = tile >= n_full_tiles;
        __syncthreads();
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int r = (tid >> 4) + 16 * pass, c = tid & 15;
            const int col = col0 + r < g.lc ? col0 + r : g.lc - 1;
            const long long off = (long long)col * g.kv_stride_tok + c * 8;
            const uint4 kx = *reinterpret_cast<const uint4*>(k + off);
            const uint4 vx = *reinterpret_cast<const uint4*>(v + off);
            *reinterpret_cast<uint4*>(&Ks[r * KSTR + c * 8]) = kx;
            *reinterpret_cast<uint4*>(&Vs[r * VSTR + c * 8]) = vx;
        }
        if (partial && tid < TN) kpos_s[tid] = col0 + tid < g.lc ? seg_pos_of_row(g.ks, col0 + tid) : 0x7fffffff;
        __syncthreads();

        // S^T[kv][q] for two 32-key blocks
        f32x16 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Ks[(32 * b + l32) * KSTR + 16 * ks + 8 * hh]);
                s[b] = mfma32(kf, qf[ks], s[b]);
            }
        }
        float mx = -INFINITY;
        if (partial) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kvl = 32 * b + 8 * (r >> 2) + 4 * hh + (r & 3);
                    const float x = kpos_s[kvl] <= my_pos ? s[b][r] * scale_log2 : -INFINITY;
                    s[b][r] = x;
                    mx = fmaxf(mx, x);
                }
        } else {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float x = s[b][r] * scale_log2;
                    s[b][r] = x;
                    mx = fmaxf(mx, x);
                }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = fast_exp2(m_run - m_use);
        // probabilities, rounded to bf16 operand slots.  Two running sums: `l_run` of the exact
        // values (it defines the LSE that the merge and the backward pass use) and `lr_run` of the
        // rounded values (it normalises O, so that O is an exact convex combination with the
        // weights the PV product really used and the rounding of a dominant key cancels).
        float ps = 0.f, psr = 0.f;
        bf16x8 pf[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int b = u >> 1, x = (u & 1) * 8;
            float p[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) { p[e] = fast_exp2(s[b][x + e] - m_use); ps += p[e]; }
            pf[u] = pack_bf16x8_sum(p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7], psr);
        }
        l_run = l_run * alpha + ps;     // per-half partial sums; the two halves are added at the end
        lr_run = lr_run * alpha + psr;
        m_run = m_new;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;

        // O^T[d][q] += V^T P^T over four 16-key steps
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint16_t* vrow = &Vs[(16 * u + 4 * hh + (j16 >> 2)) * VSTR + 16 * grp2 + 4 * (j16 & 3)];
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x8 vf = lds_tr_pair(vrow + 32 * db, vrow + 32 * db + 8 * VSTR);
                oacc[db] = mfma32(vf, pf[u], oacc[db]);
            }
        }
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float lr_tot = lr_run + __shfl_xor(lr_run, 32, 64);
    float inv = 0.f, lse_new = -INFINITY;
    if (l_tot > 0.f) {
        inv = lr_tot > 0.f ? 1.0f / lr_tot : 0.f;
        lse_new = (m_run + __log2f(l_tot)) * LN2;
    }
    if (my_row >= g.lq) return;
    float* op = a.o + ((long long)my_row * g.nq + h) * D + 4 * hh;
    float* lp = a.lse + (long long)h * g.lq + my_row;
    float wa = 0.f, wb = inv;
    if (a.accumulate) {
        const float la = *lp;
        const float m = fmaxf(la, lse_new);
        if (m != -INFINITY) {
            const float ea = __expf(la - m), eb = __expf(lse_new - m);
            const float r = 1.0f / (ea + eb);
            wa = ea * r;
            wb = eb * r * inv;
            lse_new = m + __logf(ea + eb);
        }
    }
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            float4* dst = reinterpret_cast<float4*>(op + 32 * db + 8 * b);
            float4 r = make_float4(oacc[db][4 * b] * wb, oacc[db][4 * b + 1] * wb, oacc[db][4 * b + 2] * wb, oacc[db][4 * b + 3] * wb);
            if (a.accumulate) {
                const float4 old = *dst;
                r.x += wa * old.x; r.y += wa * old.y; r.z += wa * old.z; r.w += wa * old.w;
            }
            *dst = r;
        }
    // both half-wave lanes of a row read *lp in the same instruction above, before this write
    if (hh == 0) *lp = lse_new;
}

}  // namespace

hipError_t hexi_launch_fwd_bf16(const FwdArgs& a, hipStream_t s)
{
    dim3 grid((a.g.lq + TM - 1) / TM, a.g.nq);
    fwd_bf16_kernel<<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}
