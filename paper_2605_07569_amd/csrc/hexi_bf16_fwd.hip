// bf16 forward ring step for gfx950: one workgroup (4 wavefronts) per (128-row q tile, q head),
// two workgroups per CU.
//
// The scores are computed transposed, S^T = K Q^T, so that every lane owns one query row: the
// softmax state (running max, running sums) is a per-lane scalar, the row reductions are in-lane
// plus one exchange between the two half-waves, and the accumulator registers holding P^T are
// already in MFMA operand order for O^T += V^T P^T.  Q stays in registers for the whole chunk.
//
// K / V tiles (64 keys) are double-buffered in LDS and fetched one tile ahead with direct
// global->LDS loads; one barrier per tile.  The tiles are XOR-swizzled (no padding) so that both the
// 128-bit row reads of K and the transposed 64-bit reads of V are bank-conflict free.  KV tiles that
// lie wholly in the visible past of the q tile skip all masking; tiles wholly in the future are
// never visited.
//
// Softmax runs in base 2 with the scale folded into one FMA per score.  The running maximum is only
// raised when a tile exceeds it by more than 2^8 (then O and the sums are rescaled); otherwise the
// probabilities are formed against the stale maximum, which keeps them below 2^8 and leaves the
// result unchanged because the same reference enters the sums.
#include "hexi_internal.h"
#include "hexi_mfma.h"

namespace {

constexpr int D = 128;
constexpr int TM = 128;          // q rows per workgroup (32 per wavefront)
constexpr int TN = 64;           // keys per tile
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float NEG_BIG = -1.0e30f;   // finite stand-in for "no key seen yet"
constexpr float RESCALE_SLACK = 8.0f;

__device__ __forceinline__ int swz_row(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

struct FwdSmem {
    uint16_t k[2][TN * D];   // 2 x 16 KB
    uint16_t v[2][TN * D];   // 2 x 16 KB
    int kpos[2][TN];
#ifdef EXP_BIG_LDS
    int pad[12000];
#endif
};

__global__ void __launch_bounds__(256, 2) fwd_bf16_kernel(const FwdArgs a, const int n_q_tiles)
{
    const AttnGeom& g = a.g;
    __shared__ __attribute__((aligned(1024))) FwdSmem sm;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int grp2 = (lane >> 4) & 1, j16 = lane & 15;

    // Work mapping: workgroup ids are dealt round-robin to the 8 XCDs; each XCD gets a contiguous
    // range of (head, q tile) units, so the workgroups sharing an L2 stream the same kv head.  Within
    // a head the q tiles are taken from the end of the shard backwards: under a causal mask the last
    // tiles see the most keys, and starting the longest units first evens out the tail.
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
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) pin(qf[ks]);
    }

    // Direct global->LDS fetch of one K/V tile: 16 wave-instructions of 1 KB per tensor, 4 per
    // wavefront; lane L of instruction i fills chunk position L%16 of row 4*i + L/16 with the
    // chunk (L%16) ^ swz_row(row).
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

    f32x16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m_run = NEG_BIG, l_run = 0.f, lr_run = 0.f;
    const float c_log2 = g.scale * LOG2E, inv_c_log2 = 1.0f / c_log2;
    float thr_raw = NEG_BIG;   // any finite score exceeds it: the first visible tile always sets the maximum
    const int sw_l32 = swz_row(l32);
    const int jj = j16 >> 2, cl = 2 * grp2 + ((j16 & 3) >> 1);

#ifdef EXP_TIMING
    long long tacc[6] = {0, 0, 0, 0, 0, 0}; long long t0 = __builtin_amdgcn_s_memtime(), t1;
#define TICK(i) { t1 = __builtin_amdgcn_s_memtime(); tacc[i] += t1 - t0; t0 = t1; }
#else
#define TICK(i)
#endif
    if (n_tiles > 0) fetch_tile(0, 0);
    for (int tile = 0; tile < n_tiles; ++tile) {
        const int buf = tile & 1;
        const bool partial = tile >= n_full_tiles;
        // publish tile: wait for this wavefront's outstanding global->LDS loads, then barrier
        TICK(0)
#ifndef EXP_NO_VMWAIT
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
        TICK(1)
#ifndef EXP_NO_BARRIER
        __syncthreads();
#endif
#ifdef EXP_NO_FETCH
        if (tile + 1 < n_tiles && g.scale == 12345.f) fetch_tile(tile + 1, buf ^ 1);
#else
        if (tile + 1 < n_tiles) fetch_tile(tile + 1, buf ^ 1);
#endif

        TICK(2)
        const uint16_t* Ks = &sm.k[buf][0];
        const uint16_t* Vs = &sm.v[buf][0];
        // S^T[key][q] for two 32-key blocks, LDS reads running ahead of the MFMAs
        f32x16 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
        {
            auto frag_off = [&](int st) { return (32 * (st & 1) + l32) * D + (((2 * (st >> 1) + hh) ^ sw_l32) << 3); };
            constexpr int PF = 4;
            bf16x8 kr[PF];
#pragma unroll
            for (int st = 0; st < PF; ++st) kr[st] = *reinterpret_cast<const bf16x8*>(&Ks[frag_off(st)]);
#pragma unroll
            for (int st = 0; st < 16; ++st) {
                const bf16x8 kf = kr[st % PF];
                if (st + PF < 16) kr[st % PF] = *reinterpret_cast<const bf16x8*>(&Ks[frag_off(st + PF)]);
                s[st & 1] = mfma32(kf, qf[st >> 1], s[st & 1]);
            }
            // K fragments run 4 reads ahead of the MFMA that consumes them
            HEXI_SCHED_DSREAD(PF);
#pragma unroll
            for (int st = 0; st < 16; ++st) {
                HEXI_SCHED_MFMA(1);
                if (st + PF < 16) HEXI_SCHED_DSREAD(1);
            }
        }
#ifdef EXP_TIMING
        asm volatile("s_nop 0" :: "v"(s[0][0]), "v"(s[1][15]));
#endif
        TICK(3)
        // first V^T fragments can be on their way while the softmax runs
        auto v_off = [&](int st, int second) {
            const int u = st >> 2, db = st & 3;
            const int r = 16 * u + 4 * hh + jj + 8 * second;
            const int pos = (((db ^ jj) << 2) | (cl ^ (hh + 2 * second)));
            return r * D + (pos << 3) + 4 * (j16 & 1);
        };
        constexpr int PFV = 4;
        bf16x8 vr[PFV];
#pragma unroll
        for (int st = 0; st < PFV; ++st) vr[st] = lds_tr_pair(&Vs[v_off(st, 0)], &Vs[v_off(st, 1)]);

#ifdef EXP_NO_SMAX
        bf16x8 pf[4];
        for (int u = 0; u < 4; ++u) { f32x4 t = {s[u >> 1][(u & 1) * 8], s[u >> 1][(u & 1) * 8 + 1], s[u >> 1][(u & 1) * 8 + 2], s[u >> 1][(u & 1) * 8 + 3]}; pf[u] = __builtin_bit_cast(bf16x8, t); }
#else
        if (partial) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kvl = 32 * b + 8 * (r >> 2) + 4 * hh + (r & 3);
                    if (sm.kpos[buf][kvl] > my_pos) s[b][r] = -INFINITY;
                }
        }
        float mx = max3(s[0][0], s[0][1], s[0][2]);
#pragma unroll
        for (int r = 3; r < 15; r += 2) mx = max3(mx, s[0][r], s[0][r + 1]);
        mx = max3(mx, s[0][15], s[1][0]);
#pragma unroll
        for (int r = 1; r < 15; r += 2) mx = max3(mx, s[1][r], s[1][r + 1]);
        mx = max_across_halves(max2(mx, s[1][15]));
        // raise the running maximum only when this tile exceeds it by more than the slack
        // (mx is the raw score; thr_raw = (m_run + slack) / c)
        if (__any(mx > thr_raw)) {
            const float m_new = fmaxf(m_run, mx * c_log2);
            const float alpha = fast_exp2(m_run - m_new);
            l_run *= alpha;
            lr_run *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
            m_run = m_new;
            thr_raw = (m_run + RESCALE_SLACK) * inv_c_log2;
        }
        // probabilities, rounded to bf16 operand slots.  Two running sums: `l_run` of the exact
        // values (it defines the LSE that the merge and the backward pass use) and `lr_run` of the
        // rounded values (it normalises O, so that O is an exact convex combination with the
        // weights the PV product really used and the rounding of a dominant key cancels).
        float ps = 0.f, psr = 0.f;
        bf16x8 pf[4];
        const float neg_m = -m_run;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int b = u >> 1, x = (u & 1) * 8;
            float p[8];
#pragma unroll
#ifdef EXP_NO_EXP
            for (int e = 0; e < 8; ++e) { p[e] = fmaf(s[b][x + e], c_log2, neg_m); ps += p[e]; }
#else
            for (int e = 0; e < 8; ++e) { p[e] = fast_exp2(fmaf(s[b][x + e], c_log2, neg_m)); ps += p[e]; }
#endif
            pf[u] = pack_bf16x8_sum(p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7], psr);
        }
        l_run += ps;       // per-half partial sums; the two halves are added at the end
        lr_run += psr;

#endif
#ifdef EXP_TIMING
        asm volatile("s_nop 0" :: "v"(pf[3]));
#endif
        TICK(4)
        // O^T[d][q] += V^T P^T over four 16-key steps x four 32-column blocks
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            const bf16x8 vf = vr[st % PFV];
            if (st + PFV < 16) vr[st % PFV] = lds_tr_pair(&Vs[v_off(st + PFV, 0)], &Vs[v_off(st + PFV, 1)]);
#ifndef EXP_NO_PV
            oacc[st & 3] = mfma32(vf, pf[st >> 2], oacc[st & 3]);
#else
            if (st == 0) oacc[0] = mfma32(vf, pf[0], oacc[0]); if (st == 1) oacc[1] = mfma32(vf, pf[1], oacc[1]); if (st == 2) oacc[2] = mfma32(vf, pf[2], oacc[2]); if (st == 3) oacc[3] = mfma32(vf, pf[3], oacc[3]);
#endif
        }
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            HEXI_SCHED_MFMA(1);
            if (st + PFV < 16) HEXI_SCHED_DSREAD(2);
        }
    }

#ifdef EXP_TIMING
    asm volatile("s_nop 0" :: "v"(oacc[0][0]), "v"(oacc[3][15]));
    TICK(0)
    if (tid == 0) { for (int i = 0; i < 6; ++i) a.o[(long long)unit * 8 + i] = (float)tacc[i]; a.o[(long long)unit * 8 + 6] = (float)n_tiles; }
    return;
#endif
    const float l_tot = sum_across_halves(l_run);
    const float lr_tot = sum_across_halves(lr_run);
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
    const int n_q_tiles = (a.g.lq + TM - 1) / TM;
    fwd_bf16_kernel<<<(unsigned)(a.g.nq * n_q_tiles), 256, 0, s>>>(a, n_q_tiles);
    return hipGetLastError();
}
