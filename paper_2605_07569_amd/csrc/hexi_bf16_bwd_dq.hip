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
#include <type_traits>

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

    // Lane parts of the LDS addresses (elements); block, step and buffer are compile-time offsets.
    int nat_lane[8], tr_lane[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) nat_lane[ks] = l32 * D + (((2 * ks + hh) ^ sw_l32) << 3);
#pragma unroll
    for (int x = 0; x < 8; ++x) {   // x = 2*db + second
        const int db = x >> 1, second = x & 1;
        tr_lane[x] = (4 * hh + jj + 8 * second) * D + ((((db ^ jj) << 2) | (cl ^ (hh + 2 * second))) << 3) + 4 * (j16 & 1);
    }

    // One 64-key tile.  The two 32-key blocks are staggered so that the VALU work of one block sits between
    // MFMAs of the other in program order:
    //   A: S^T/dP^T(block 0) | B: S^T/dP^T(block 1) + VALU(block 0) | C: dQ^T(block 0) + VALU(block 1) | D: dQ^T(block 1)
    // Every step ends in a scheduling barrier so that this interleave is what gets issued.
    auto tile_body = [&](auto buf_c, auto masked_c) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_c)::value;
        constexpr int buf = decltype(buf_c)::value;
        const uint16_t* Ks = &sm.k[buf][0];
        const uint16_t* Vs = &sm.v[buf][0];
        f32x16 s[2], dp[2];
        bf16x8 dsf[4];
        constexpr int PF = 2;
        bf16x8 ra[PF], rb_[PF];
        auto load_nat = [&](int b, int ks, int slot) {
            ra[slot] = *reinterpret_cast<const bf16x8*>(&Ks[nat_lane[ks] + 32 * b * D]);
            rb_[slot] = *reinterpret_cast<const bf16x8*>(&Vs[nat_lane[ks] + 32 * b * D]);
        };
        // K^T fragment of 16-key step u (= 2*b + st/4... see callers) and 32-column block db
        auto load_tr = [&](int u, int db, int slot) {
            ra[slot] = lds_tr_pair(&Ks[tr_lane[2 * db] + 16 * u * D], &Ks[tr_lane[2 * db + 1] + 16 * u * D]);
        };
        auto valu2 = [&](int b, int e) {
#pragma unroll
            for (int x = e; x < e + 2; ++x) {
                float p = fast_exp2(fmaf(s[b][x], c_log2, neg_lse2));
                if (MASKED) p = (sm.kpos[buf][32 * b + 8 * (x >> 2) + 4 * hh + (x & 3)] > my_pos) ? 0.f : p;
                dp[b][x] = p * (dp[b][x] - delta);
            }
        };
        auto pack = [&](int b, int half) {
            const int x = 8 * half;
            dsf[2 * b + half] = pack_bf16x8(dp[b][x], dp[b][x + 1], dp[b][x + 2], dp[b][x + 3], dp[b][x + 4], dp[b][x + 5], dp[b][x + 6], dp[b][x + 7]);
        };
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[b][r] = 0.f; dp[b][r] = 0.f; }
        // phase A (global steps 0..7)
#pragma unroll
        for (int ks = 0; ks < PF; ++ks) load_nat(0, ks, ks);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf = ra[ks % PF], vf = rb_[ks % PF];
            if (ks + PF < 8) load_nat(0, ks + PF, ks % PF);
            else load_nat(1, ks + PF - 8, ks % PF);
            s[0] = mfma32(kf, qf[ks], s[0]);
            dp[0] = mfma32(vf, gf[ks], dp[0]);
            __builtin_amdgcn_sched_barrier(0);
        }
        // phase B (global steps 8..15): block 1 products, block 0 VALU
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf = ra[(8 + ks) % PF], vf = rb_[(8 + ks) % PF];
            if (ks + PF < 8) load_nat(1, ks + PF, (8 + ks) % PF);
            else load_tr((ks + PF - 8) >> 2, (ks + PF - 8) & 3, (8 + ks) % PF);
            s[1] = mfma32(kf, qf[ks], s[1]);
            dp[1] = mfma32(vf, gf[ks], dp[1]);
            valu2(0, 2 * ks);
            if (ks == 4) pack(0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        pack(0, 1);
        // phase C (global steps 16..23): dQ^T += K^T dS^T for 16-key steps 0,1 (block 0); block 1 VALU
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            const bf16x8 kt = ra[(16 + st) % PF];
            if (st + PF < 8) load_tr((st + PF) >> 2, (st + PF) & 3, (16 + st) % PF);
            else load_tr(2 + ((st + PF - 8) >> 2), (st + PF - 8) & 3, (16 + st) % PF);
            dq[st & 3] = mfma32(kt, dsf[st >> 2], dq[st & 3]);
            valu2(1, 4 * (st >> 1) + 2 * (st & 1));
            if (st == 4) pack(1, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        pack(1, 1);
        // phase D (global steps 24..31): 16-key steps 2,3 (block 1)
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            const bf16x8 kt = ra[(24 + st) % PF];
            if (st + PF < 8) load_tr(2 + ((st + PF) >> 2), (st + PF) & 3, (24 + st) % PF);
            dq[st & 3] = mfma32(kt, dsf[2 + (st >> 2)], dq[st & 3]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    fetch_tile(0, 0);
    // one tile: publish it (wait for this wavefront's outstanding global->LDS loads, then barrier), start
    // fetching the next one into the other buffer, compute
    auto step = [&](int tile, auto buf_c, auto masked_c) __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tile + 1 < n_tiles) fetch_tile(tile + 1, decltype(buf_c)::value ^ 1);
        tile_body(buf_c, masked_c);
    };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    // unmasked tiles two at a time, then the masked tail (buffer = tile parity throughout)
    int tile = 0;
    for (; tile + 1 < n_full_tiles; tile += 2) {
        step(tile, B0{}, std::false_type{});
        step(tile + 1, B1{}, std::false_type{});
    }
    if (tile < n_full_tiles) { step(tile, B0{}, std::false_type{}); ++tile; }
    if (tile < n_tiles && (tile & 1)) { step(tile, B1{}, std::true_type{}); ++tile; }
    for (; tile + 1 < n_tiles; tile += 2) {
        step(tile, B0{}, std::true_type{});
        step(tile + 1, B1{}, std::true_type{});
    }
    if (tile < n_tiles) step(tile, B0{}, std::true_type{});

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
