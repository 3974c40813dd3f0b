// bf16 backward ring step, dQ part, for gfx950: one workgroup (4 wavefronts) per (128-row q tile,
// q head); the q tile's dQ stays in accumulators while the chunk's keys stream past, so dQ needs no
// atomics and its summation order is fixed.
//
// Everything is computed transposed, as in the forward kernel, so that every lane owns one query
// row and the row constants (saved global LSE, Delta) are per-lane scalars:
//   S^T = K Q^T,  dP^T = V dO^T  (K, V rows read from LDS with 128-bit reads; Q^T, dO^T in registers),
//   P^T = exp2(S^T * scale*log2e - LSE*log2e),  dS^T = P^T (dP^T - Delta),
//   dQ^T += K^T dS^T  (K^T through transposed LDS reads; dS^T straight from the accumulator registers).
// K / V tiles (64 keys) are double-buffered in LDS and fetched one tile ahead with direct global->LDS
// loads, XOR-swizzled, one barrier per tile.  At the end dq_acc += scale * dQ (plain read-modify-write:
// each (row, head) belongs to exactly one workgroup of the launch).
#include "hexi_internal.h"
#include "hexi_mfma.h"

namespace {

constexpr int D = 128;
constexpr int TM = 128;          // q rows per workgroup (32 per wavefront)
constexpr int TN = 64;           // keys per tile
constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ int swz_row(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

struct DqSmem {
    uint16_t k[2][TN * D];   // 2 x 16 KB
    uint16_t v[2][TN * D];   // 2 x 16 KB
    int kpos[2][TN];
};

__global__ void __launch_bounds__(256, 2) bwd_dq_bf16_kernel(const BwdArgs a, const int n_q_tiles)
{
    const AttnGeom& g = a.g;
    __shared__ __attribute__((aligned(1024))) DqSmem sm;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int grp2 = (lane >> 4) & 1, j16 = lane & 15;

    // (head, q tile) units: contiguous ranges per XCD, longest q tiles of a head first
    const int n_units = g.nq * n_q_tiles;
    int unit;
    {
        const int per = n_units / 8, rem = n_units % 8;
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        unit = xcd * per + (xcd < rem ? xcd : rem) + slot;
    }
    const int h = unit / n_q_tiles;
    const int q_tile = n_q_tiles - 1 - (unit - h * n_q_tiles);
    const int kvh = g.kv_of_q[h];
    const int row0 = q_tile * TM;
    const int my_row = row0 + 32 * wave + l32;
    const int my_row_c = my_row < g.lq ? my_row : g.lq - 1;
    const int my_pos = my_row < g.lq ? seg_pos_of_row(g.qs, my_row) : -1;

    const uint16_t* k = static_cast<const uint16_t*>(a.k) + (long long)kvh * g.kv_stride_head;
    const uint16_t* v = static_cast<const uint16_t*>(a.v) + (long long)kvh * g.kv_stride_head;

    const int last_row = (row0 + TM < g.lq ? row0 + TM : g.lq) - 1;
    const int n_vis = seg_rows_le(g.ks, seg_pos_of_row(g.qs, last_row));
    const int n_all = seg_rows_le(g.ks, seg_pos_of_row(g.qs, row0));
    const int n_tiles = (n_vis + TN - 1) / TN;
    const int n_full_tiles = n_all / TN;
    if (n_tiles == 0) return;     // this q tile sees nothing of the chunk: dq_acc unchanged

    // Q^T and dO^T operand fragments: lane (row l32, half hh) holds d = 16*ks + 8*hh .. +7
    bf16x8 qf[8], gf[8];
    float lse2, delta;
    {
        const long long off = (long long)my_row_c * g.q_stride_tok + (long long)h * g.q_stride_head + 8 * hh;
        const uint16_t* qp = static_cast<const uint16_t*>(a.q) + off;
        const uint16_t* gp = static_cast<const uint16_t*>(a.d_o) + off;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            qf[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
            gf[ks] = *reinterpret_cast<const bf16x8*>(gp + 16 * ks);
        }
        const float l = a.lse[(long long)h * g.lq + my_row_c];
        // rows that see nothing anywhere (LSE = -inf) and padding rows: P = 0 through LSE = +inf
        lse2 = (my_row < g.lq && l != -INFINITY) ? l * LOG2E : INFINITY;
        delta = a.delta[(long long)h * g.lq + my_row_c];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) { pin(qf[ks]); pin(gf[ks]); }
        asm volatile("" ::"v"(lse2), "v"(delta));
    }

    int fetch_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = (wave * 4 + i) * 4 + (lane >> 4);
        fetch_off[i] = r * (int)g.kv_stride_tok + (((lane & 15) ^ swz_row(r)) << 3);
    }
    const uint32_t lds_k = (uint32_t)(uintptr_t)(&sm.k[0][0]), lds_v = (uint32_t)(uintptr_t)(&sm.v[0][0]);
    auto fetch_tile = [&](int tile, int buf) {
        const int col0 = tile * TN;
        const uint32_t wk = __builtin_amdgcn_readfirstlane(lds_k + buf * (TN * D * 2) + wave * 4096);
        const uint32_t wv = __builtin_amdgcn_readfirstlane(lds_v + buf * (TN * D * 2) + wave * 4096);
        if (col0 + TN <= g.lc) {
            const uint16_t* kb = k + (long long)col0 * g.kv_stride_tok;
            const uint16_t* vb = v + (long long)col0 * g.kv_stride_tok;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lds_dma16(kb + fetch_off[i], wk + i * 1024);
                lds_dma16(vb + fetch_off[i], wv + i * 1024);
            }
        } else {   // ragged last tile: clamp the key index (the extra keys are masked through their position)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = (wave * 4 + i) * 4 + (lane >> 4);
                const int c = (lane & 15) ^ swz_row(r);
                const int col = col0 + r < g.lc ? col0 + r : g.lc - 1;
                const long long off = (long long)col * g.kv_stride_tok + c * 8;
                lds_dma16(k + off, wk + i * 1024);
                lds_dma16(v + off, wv + i * 1024);
            }
        }
        if (wave == 0 && tile >= n_full_tiles)
            sm.kpos[buf][lane] = col0 + lane < g.lc ? seg_pos_of_row(g.ks, col0 + lane) : 0x7fffffff;
    };

    f32x16 dq[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[db][r] = 0.f;
    const float c_log2 = g.scale * LOG2E;
    const float neg_lse2 = -lse2;
    const int sw_l32 = swz_row(l32);
    const int jj = j16 >> 2, cl = 2 * grp2 + ((j16 & 3) >> 1);

    fetch_tile(0, 0);
    for (int tile = 0; tile < n_tiles; ++tile) {
        const int buf = tile & 1;
        const bool partial = tile >= n_full_tiles;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tile + 1 < n_tiles) fetch_tile(tile + 1, buf ^ 1);

        const uint16_t* Ks = &sm.k[buf][0];
        const uint16_t* Vs = &sm.v[buf][0];
        // S^T[key][q] and dP^T[key][q] for two 32-key blocks
        f32x16 s[2], dp[2];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[b][r] = 0.f; dp[b][r] = 0.f; }
        {
            auto frag_off = [&](int st) { return (32 * (st & 1) + l32) * D + (((2 * (st >> 1) + hh) ^ sw_l32) << 3); };
            constexpr int PF = 3;
            bf16x8 kr[PF], vr[PF];
#pragma unroll
            for (int st = 0; st < PF; ++st) {
                kr[st] = *reinterpret_cast<const bf16x8*>(&Ks[frag_off(st)]);
                vr[st] = *reinterpret_cast<const bf16x8*>(&Vs[frag_off(st)]);
            }
#pragma unroll
            for (int st = 0; st < 16; ++st) {
                const bf16x8 kf = kr[st % PF], vf = vr[st % PF];
                if (st + PF < 16) {
                    kr[st % PF] = *reinterpret_cast<const bf16x8*>(&Ks[frag_off(st + PF)]);
                    vr[st % PF] = *reinterpret_cast<const bf16x8*>(&Vs[frag_off(st + PF)]);
                }
                s[st & 1] = mfma32(kf, qf[st >> 1], s[st & 1]);
                dp[st & 1] = mfma32(vf, gf[st >> 1], dp[st & 1]);
            }
            HEXI_SCHED_DSREAD(2 * PF);
#pragma unroll
            for (int st = 0; st < 16; ++st) {
                HEXI_SCHED_MFMA(2);
                if (st + PF < 16) HEXI_SCHED_DSREAD(2);
            }
        }
        // first K^T fragments on their way while the VALU part runs
        auto kt_off = [&](int st, int second) {
            const int u = st >> 2, db = st & 3;
            const int r = 16 * u + 4 * hh + jj + 8 * second;
            const int pos = (((db ^ jj) << 2) | (cl ^ (hh + 2 * second)));
            return r * D + (pos << 3) + 4 * (j16 & 1);
        };
        constexpr int PFK = 4;
        bf16x8 ktr[PFK];
#pragma unroll
        for (int st = 0; st < PFK; ++st) ktr[st] = lds_tr_pair(&Ks[kt_off(st, 0)], &Ks[kt_off(st, 1)]);

        // P^T into s; keys the row cannot see get P = 0 (one uniform branch per tile); then dS^T into dp
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[b][r] = fast_exp2(fmaf(s[b][r], c_log2, neg_lse2));
        if (partial) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (sm.kpos[buf][32 * b + 8 * (r >> 2) + 4 * hh + (r & 3)] > my_pos) s[b][r] = 0.f;
        }
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) dp[b][r] = s[b][r] * (dp[b][r] - delta);
        bf16x8 dsf[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int b = u >> 1, x = (u & 1) * 8;
            dsf[u] = pack_bf16x8(dp[b][x], dp[b][x + 1], dp[b][x + 2], dp[b][x + 3], dp[b][x + 4], dp[b][x + 5], dp[b][x + 6], dp[b][x + 7]);
        }
        // dQ^T[d][q] += K^T dS^T over four 16-key steps x four 32-column blocks
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            const bf16x8 kt = ktr[st % PFK];
            if (st + PFK < 16) ktr[st % PFK] = lds_tr_pair(&Ks[kt_off(st + PFK, 0)], &Ks[kt_off(st + PFK, 1)]);
            dq[st & 3] = mfma32(kt, dsf[st >> 2], dq[st & 3]);
        }
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            HEXI_SCHED_MFMA(1);
            if (st + PFK < 16) HEXI_SCHED_DSREAD(2);
        }
    }

    if (my_row >= g.lq) return;
    // lane (row l32, half hh): register 4*b + t of block db holds d = 32*db + 8*b + 4*hh + t
    float* dst0 = a.dq + ((long long)my_row * g.nq + h) * D + 4 * hh;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            float4* dst = reinterpret_cast<float4*>(dst0 + 32 * db + 8 * b);
            float4 o = *dst;
            o.x += g.scale * dq[db][4 * b]; o.y += g.scale * dq[db][4 * b + 1];
            o.z += g.scale * dq[db][4 * b + 2]; o.w += g.scale * dq[db][4 * b + 3];
            *dst = o;
        }
}

}  // namespace

hipError_t hexi_launch_bwd_dq_bf16(const BwdArgs& a, hipStream_t s)
{
    const int n_q_tiles = (a.g.lq + TM - 1) / TM;
    bwd_dq_bf16_kernel<<<(unsigned)(a.g.nq * n_q_tiles), 256, 0, s>>>(a, n_q_tiles);
    return hipGetLastError();
}
