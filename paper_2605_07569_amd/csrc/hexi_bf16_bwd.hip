// bf16 backward ring step, dK / dV part, for gfx950: one workgroup (4 wavefronts, one per SIMD) per
// (128-key tile, q head).
//
// The workgroup keeps its K and V rows in registers as MFMA operands and its dK / dV tiles in
// accumulators while it sweeps the 64-row q tiles that can see the key tile.  Per q tile:
// S = Q K^T and dP = dO V^T (keys across lanes, query rows in-lane), P = exp2(S*scale*log2e -
// LSE*log2e) from the saved global LSE, dS = P (dP - Delta); the accumulator registers holding P
// and dS are already in operand order for dV += P^T dO and dK += dS^T Q (dO and Q fetched with
// transposed LDS reads).  dQ is produced by a separate q-stationary kernel: adding it from here
// would need one fp32 atomic per dS K element per key tile, and that atomic traffic (about
// 3 bytes per kFLOP at 128 keys per workgroup) saturates the L2 atomic units long before the MFMA
// pipes; recomputing S and dP in the dQ kernel costs 2 extra matmuls out of 5 but keeps every
// product on the matrix cores.
//
// Pipeline: Q / dO tiles are double-buffered in LDS and fetched one tile ahead with direct
// global->LDS loads, one barrier per tile.  LDS tiles are XOR-swizzled (no padding) so that both the
// 128-bit row reads and the transposed 64-bit reads are bank-conflict free.
//
// The q heads of a GQA group run in different workgroups and add their dK / dV tiles with fp32
// atomics (plain stores when the group has a single head), so dk/dv must be zero-filled (or hold
// the running sum under HEXI_ACCUMULATE) before the launch.
#include "hexi_internal.h"
#include "hexi_mfma.h"
#include <type_traits>

namespace {

constexpr int D = 128;
constexpr int TN = 128;          // keys per workgroup (32 per wavefront)
constexpr int TM = 64;           // q rows per inner tile
constexpr float LOG2E = 1.4426950408889634f;

// [rows][128] bf16 tile, 16-byte chunk c of row r stored at chunk position c ^ swz_row(r)
__device__ __forceinline__ int swz_row(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

struct BwdSmem {
    uint16_t q[2][TM * D];        // 2 x 16 KB
    uint16_t g[2][TM * D];        // dO, 2 x 16 KB
    float lse[2][TM];
    float delta[2][TM];
    int qpos[2][TM];
};

template <bool ATOMIC_DKV>
__global__ void __launch_bounds__(256) bwd_dkdv_bf16_kernel(const BwdArgs a, const int n_kv_tiles)
{
    const AttnGeom& g = a.g;
    __shared__ __attribute__((aligned(1024))) BwdSmem sm;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int grp2 = (lane >> 4) & 1, j16 = lane & 15;

    // Work mapping: consecutive workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a
    // contiguous range of (head, key tile) units so that the workgroups sharing an L2 stream the
    // same head's Q / dO tiles.
    const int n_units = g.nq * n_kv_tiles;
    int unit = blockIdx.x;
    {
        const int per = n_units / 8, rem = n_units % 8;
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        // XCD x owns per + (x < rem) units starting at x*per + min(x, rem)
        unit = xcd * per + (xcd < rem ? xcd : rem) + slot;
    }
    const int h = unit / n_kv_tiles;
    const int kv_tile = unit - h * n_kv_tiles;
    const int kvh = g.kv_of_q[h];
    const int col0 = kv_tile * TN;
    const int my_col = col0 + 32 * wave + l32;
    const int my_col_c = my_col < g.lc ? my_col : g.lc - 1;
    const int my_kpos = my_col < g.lc ? seg_pos_of_row(g.ks, my_col) : 0x7fffffff;

    const uint16_t* q = static_cast<const uint16_t*>(a.q) + (long long)h * g.q_stride_head;
    const uint16_t* go = static_cast<const uint16_t*>(a.d_o) + (long long)h * g.q_stride_head;
    const uint16_t* k = static_cast<const uint16_t*>(a.k) + (long long)kvh * g.kv_stride_head;
    const uint16_t* v = static_cast<const uint16_t*>(a.v) + (long long)kvh * g.kv_stride_head;
    const float* lse_h = a.lse + (long long)h * g.lq;
    const float* delta_h = a.delta + (long long)h * g.lq;

    // q rows that see at least one key of the tile form a suffix of the shard; rows that see all of
    // its keys form a (shorter) suffix
    const int last_col = (col0 + TN < g.lc ? col0 + TN : g.lc) - 1;
    const int k_min = seg_pos_of_row(g.ks, col0), k_max = seg_pos_of_row(g.ks, last_col);
    const int qt_begin = seg_rows_le(g.qs, k_min - 1) / TM;
    const int qt_full = (col0 + TN <= g.lc) ? (seg_rows_le(g.qs, k_max - 1) + TM - 1) / TM : 0x7fffffff;
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
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) { pin(kf[ks]); pin(vf[ks]); }
    }
    f32x16 dk_acc[4], dv_acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk_acc[db][r] = 0.f; dv_acc[db][r] = 0.f; }
    const float scale_log2 = g.scale * LOG2E;

    // Direct global->LDS fetch of one q tile (Q and dO, 16 KB each): 16 wave-instructions of 1 KB per
    // tensor, 4 per wavefront; lane L of instruction i fills chunk position L%16 of row 4*i + L/16.
    // The loads are issued through inline assembly so that the compiler does not serialise later
    // LDS reads of the OTHER buffer behind them; they are waited for explicitly (vmcnt(0)) right
    // before the barrier that publishes the tile.
    int fetch_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = (wave * 4 + i) * 4 + (lane >> 4);
        fetch_off[i] = r * (int)g.q_stride_tok + (((lane & 15) ^ swz_row(r)) << 3);
    }
    const uint32_t lds_q = (uint32_t)(uintptr_t)(&sm.q[0][0]), lds_g = (uint32_t)(uintptr_t)(&sm.g[0][0]);
    const uint32_t lds_lse = (uint32_t)(uintptr_t)(&sm.lse[0][0]), lds_delta = (uint32_t)(uintptr_t)(&sm.delta[0][0]);
    auto fetch_tile = [&](int qt, int buf) {
        const int row0 = qt * TM;
        const uint32_t wq = __builtin_amdgcn_readfirstlane(lds_q + buf * (TM * D * 2) + wave * 4096);
        const uint32_t wg = __builtin_amdgcn_readfirstlane(lds_g + buf * (TM * D * 2) + wave * 4096);
        if (row0 + TM <= g.lq) {
            const uint16_t* qb = q + (long long)row0 * g.q_stride_tok;
            const uint16_t* gb = go + (long long)row0 * g.q_stride_tok;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lds_dma16(qb + fetch_off[i], wq + i * 1024);
                lds_dma16(gb + fetch_off[i], wg + i * 1024);
            }
        } else {   // ragged last tile: clamp the row index (the extra rows are masked out through their position)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = (wave * 4 + i) * 4 + (lane >> 4);
                const int c = (lane & 15) ^ swz_row(r);
                const int row = row0 + r < g.lq ? row0 + r : g.lq - 1;
                const long long off = (long long)row * g.q_stride_tok + c * 8;
                lds_dma16(q + off, wq + i * 1024);
                lds_dma16(go + off, wg + i * 1024);
            }
        }
        // per-row scalars: one 4-byte-per-lane instruction each (LSE by wavefront 0, Delta by wavefront 1)
        if (wave < 2) {
            const int row = row0 + lane < g.lq ? row0 + lane : g.lq - 1;
            const float* src = (wave == 0 ? lse_h : delta_h) + row;
            lds_dma4(src, __builtin_amdgcn_readfirstlane((wave == 0 ? lds_lse : lds_delta) + buf * (TM * 4)));
        }
        // global positions of the tile's rows, only for tiles that need masking
        if (wave == 2 && (qt < qt_full || row0 + TM > g.lq))
            sm.qpos[buf][lane] = row0 + lane < g.lq ? seg_pos_of_row(g.qs, row0 + lane) : -1;
    };

    const int sw_l32 = swz_row(l32);
    const int jj = j16 >> 2, cl = 2 * grp2 + ((j16 & 3) >> 1);

    // One q tile.  The two 32-row q blocks are staggered so that the VALU work of one block sits
    // between MFMAs of the other in program order (the matrix pipe keeps running under the VALU):
    //   A: S/dP(block 0) | B: S/dP(block 1) + VALU(block 0) | C: dV/dK(block 0) + VALU(block 1) | D: dV/dK(block 1)
    // Each step (2 MFMAs, their LDS prefetches, 2 elements of VALU work) ends in a scheduling barrier,
    // so the hand-written interleave is what gets issued.  MASKED is a compile-time flag: masked tiles
    // take a copy of the body with selects, unmasked ones carry no per-element masking at all.
    // Lane parts of the LDS addresses (elements): everything else (q block, step, buffer) is a compile-time
    // offset, so the reads need no address arithmetic inside the loop.
    int nat_lane[8], tr_lane[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) nat_lane[ks] = l32 * D + (((2 * ks + hh) ^ sw_l32) << 3);
#pragma unroll
    for (int x = 0; x < 8; ++x) {   // x = 2*db + second
        const int db = x >> 1, second = x & 1;
        tr_lane[x] = (4 * hh + jj + 8 * second) * D + ((((db ^ jj) << 2) | (cl ^ (hh + 2 * second))) << 3) + 4 * (j16 & 1);
    }
    auto tile_body = [&](auto buf_c, auto masked_c) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_c)::value;
        constexpr int buf = decltype(buf_c)::value;
        const uint16_t* Qs = &sm.q[buf][0];
        const uint16_t* Gs = &sm.g[buf][0];
        f32x16 s[2], dp[2];
        bf16x8 pf[4], df[4];
        f32x4 lse4[2][4], del4[2][4];     // per-row constants of the rows this lane holds: i = 32*b + 8*rb + 4*hh + t
        constexpr int PF = 3;             // LDS fragments requested this many steps ahead of their MFMA
        bf16x8 ra[PF], rb_[PF];

        auto nat_off = [&](int b, int ks) { return nat_lane[ks] + 32 * b * D; };
        auto tr_off = [&](int b, int st, int second) { return tr_lane[2 * (st & 3) + second] + 16 * (2 * b + (st >> 2)) * D; };
        auto load_nat = [&](int b, int ks, int slot) {
            ra[slot] = *reinterpret_cast<const bf16x8*>(&Qs[nat_off(b, ks)]);
            rb_[slot] = *reinterpret_cast<const bf16x8*>(&Gs[nat_off(b, ks)]);
        };
        auto load_tr = [&](int b, int st, int slot) {
            ra[slot] = lds_tr_pair(&Gs[tr_off(b, st, 0)], &Gs[tr_off(b, st, 1)]);
            rb_[slot] = lds_tr_pair(&Qs[tr_off(b, st, 0)], &Qs[tr_off(b, st, 1)]);
        };
        // P and dS of elements e, e+1 of q block b.  Rows whose LSE is -inf see nothing anywhere, so they
        // are masked in every tile they appear in.
        auto valu2 = [&](int b, int e) {
#pragma unroll
            for (int x = e; x < e + 2; ++x) {
                const int rb = x >> 2, t = x & 3;
                float p = fast_exp2(fmaf(s[b][x], scale_log2, lse4[b][rb][t]));
                if (MASKED) p = (my_kpos > sm.qpos[buf][32 * b + 8 * rb + 4 * hh + t]) ? 0.f : p;
                s[b][x] = p;
                dp[b][x] = p * (dp[b][x] - del4[b][rb][t]);
            }
        };
        auto pack = [&](int b, int half) {
            const int x = 8 * half;
            pf[2 * b + half] = pack_bf16x8(s[b][x], s[b][x + 1], s[b][x + 2], s[b][x + 3], s[b][x + 4], s[b][x + 5], s[b][x + 6], s[b][x + 7]);
            df[2 * b + half] = pack_bf16x8(dp[b][x], dp[b][x + 1], dp[b][x + 2], dp[b][x + 3], dp[b][x + 4], dp[b][x + 5], dp[b][x + 6], dp[b][x + 7]);
        };

#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[b][r] = 0.f; dp[b][r] = 0.f; }
        // phase A: S/dP of block 0; the row constants are fetched alongside
#pragma unroll
        for (int ks = 0; ks < PF; ++ks) load_nat(0, ks, ks);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 qa = ra[ks % PF], ga = rb_[ks % PF];      // ring slot = (global step) % PF
            if (ks + PF < 8) load_nat(0, ks + PF, ks % PF);
            else load_nat(1, ks + PF - 8, ks % PF);
            {
                const int b = ks >> 2, rb = ks & 3;
                const f32x4 l = *reinterpret_cast<const f32x4*>(&sm.lse[buf][32 * b + 8 * rb + 4 * hh]);
                lse4[b][rb] = f32x4{-LOG2E * l[0], -LOG2E * l[1], -LOG2E * l[2], -LOG2E * l[3]};
                del4[b][rb] = *reinterpret_cast<const f32x4*>(&sm.delta[buf][32 * b + 8 * rb + 4 * hh]);
            }
            s[0] = mfma32(qa, kf[ks], s[0]);
            dp[0] = mfma32(ga, vf[ks], dp[0]);
            __builtin_amdgcn_sched_barrier(0);
        }
        // phase B: S/dP of block 1, VALU of block 0
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 qa = ra[(8 + ks) % PF], ga = rb_[(8 + ks) % PF];
            if (ks + PF < 8) load_nat(1, ks + PF, (8 + ks) % PF);
            else load_tr(0, ks + PF - 8, (8 + ks) % PF);
            s[1] = mfma32(qa, kf[ks], s[1]);
            dp[1] = mfma32(ga, vf[ks], dp[1]);
            valu2(0, 2 * ks);
            if (ks == 4) pack(0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        pack(0, 1);
        // phase C: dV/dK of block 0, VALU of block 1
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            const bf16x8 gf = ra[(16 + st) % PF], qf = rb_[(16 + st) % PF];
            if (st + PF < 8) load_tr(0, st + PF, (16 + st) % PF);
            else load_tr(1, st + PF - 8, (16 + st) % PF);
            dv_acc[st & 3] = mfma32(pf[st >> 2], gf, dv_acc[st & 3]);
            dk_acc[st & 3] = mfma32(df[st >> 2], qf, dk_acc[st & 3]);
            valu2(1, 2 * st);
            if (st == 4) pack(1, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        pack(1, 1);
        // phase D: dV/dK of block 1
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            const bf16x8 gf = ra[(24 + st) % PF], qf = rb_[(24 + st) % PF];
            if (st + PF < 8) load_tr(1, st + PF, (24 + st) % PF);
            dv_acc[st & 3] = mfma32(pf[2 + (st >> 2)], gf, dv_acc[st & 3]);
            dk_acc[st & 3] = mfma32(df[2 + (st >> 2)], qf, dk_acc[st & 3]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Tile order: first the tiles that need masking (the leading, partly visible q tiles and a ragged last
    // tile), then the fully visible ones -- two plain loops, one instantiation of the body each.
    const int n_all = n_qtiles - qt_begin;
    if (n_all > 0) {
        const bool ragged = n_qtiles * TM > g.lq;
        const int lead = (qt_full < n_qtiles ? qt_full : n_qtiles) - qt_begin;     // partly visible tiles
        const bool extra = ragged && qt_begin + lead < n_qtiles;                    // ragged last tile not among them
        const int n_masked = lead + (extra ? 1 : 0);
        auto tile_of = [&](int i) { return i < lead ? qt_begin + i : (i < n_masked ? n_qtiles - 1 : qt_begin + lead + (i - n_masked)); };
        fetch_tile(tile_of(0), 0);
        // one tile: publish it (wait for this wavefront's outstanding global->LDS loads, then barrier),
        // start fetching the next one into the other buffer, compute
        auto step = [&](int i, auto buf_c, auto masked_c) __attribute__((always_inline)) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (i + 1 < n_all) fetch_tile(tile_of(i + 1), decltype(buf_c)::value ^ 1);
            tile_body(buf_c, masked_c);
        };
        using B0 = std::integral_constant<int, 0>;
        using B1 = std::integral_constant<int, 1>;
        int i = 0;
        // masked tiles (buffer parity follows i), then unmasked tiles two at a time
        for (; i + 1 < n_masked; i += 2) {
            step(i, B0{}, std::true_type{});
            step(i + 1, B1{}, std::true_type{});
        }
        if (i < n_masked) { step(i, B0{}, std::true_type{}); ++i; }
        if (i < n_all && (i & 1)) { step(i, B1{}, std::false_type{}); ++i; }
        for (; i + 1 < n_all; i += 2) {
            step(i, B0{}, std::false_type{});
            step(i + 1, B1{}, std::false_type{});
        }
        if (i < n_all) step(i, B0{}, std::false_type{});
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
                if (ATOMIC_DKV) {
                    global_atomic_add(a.dk + idx, kk);
                    global_atomic_add(a.dv + idx, vv);
                } else if (a.accumulate) {
                    a.dk[idx] += kk; a.dv[idx] += vv;
                } else {
                    a.dk[idx] = kk; a.dv[idx] = vv;
                }
            }
        }
}

}  // namespace

hipError_t hexi_launch_bwd_bf16(const BwdArgs& a, hipStream_t s)
{
    if (a.want_dkdv) {
        const int n_kv_tiles = (a.g.lc + TN - 1) / TN;
        // does any kv head serve more than one q head?  then the heads' dK/dV tiles are summed atomically
        int cnt[HEXI_MAX_HEADS] = {0};
        bool shared = false, unused = false;
        for (int h = 0; h < a.g.nq; ++h) shared |= (++cnt[a.g.kv_of_q[h]] > 1);
        for (int kh = 0; kh < a.g.nkv; ++kh) unused |= (cnt[kh] == 0);   // a kv head no local q head reads: zero gradient
        const unsigned grid = (unsigned)(a.g.nq * n_kv_tiles);
        if ((shared || unused) && !a.accumulate) {
            const long long n = (long long)a.g.lc * a.g.nkv * D;
            hipError_t e = hexi_launch_fill_f32(a.dk, n, 0.f, s);
            if (e == hipSuccess) e = hexi_launch_fill_f32(a.dv, n, 0.f, s);
            if (e != hipSuccess) return e;
        }
        if (shared) bwd_dkdv_bf16_kernel<true><<<grid, 256, 0, s>>>(a, n_kv_tiles);
        else bwd_dkdv_bf16_kernel<false><<<grid, 256, 0, s>>>(a, n_kv_tiles);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return a.want_dq ? hexi_launch_bwd_dq_bf16(a, s) : hipSuccess;
}
