// bf16 backward ring step, dK / dV part, for gfx950 (head_dim D = 128 or 64): one workgroup of 8 wavefronts per
// (128-key tile, run of q heads), one workgroup per CU.
//
// The workgroup keeps its K and V rows in registers as MFMA operands and its dK / dV tiles in accumulators
// while it sweeps the 64-row q tiles that can see the key tile.  Per q tile: S = Q K^T and dP = dO V^T (keys
// across lanes, query rows in-lane), P = exp2(S*scale*log2e - LSE*log2e) from the saved global LSE (each tile's
// LSE values are multiplied by -log2e in LDS once, not once per score),
// dS = P (dP - Delta), dV += P^T dO and dK += dS^T Q (dO and Q fetched with transposed LDS reads).  dQ is
// produced by a separate q-stationary kernel: adding it from here would need one fp32 atomic per dS K element
// per key tile, and that atomic traffic saturates the L2 atomic units long before the MFMA pipes.
//
// Ping-pong schedule (see the forward kernel): two groups of four wavefronts, wavefront w and w + 4 on one
// SIMD, alternate between a matrix phase and a vector phase with one workgroup barrier per phase, group 1 one
// phase behind group 0, so that every SIMD always has one wavefront issuing only MFMAs (and their LDS reads)
// and one issuing only VALU work.  Two wavefronts per SIMD leave 256 registers per wavefront, too few for
// 32 keys x 128 columns of dK and dV (128 registers at D = 128) next to the K / V fragments (64): the wavefronts of a
// group therefore work in pairs on 32 keys.  Each of the two computes S, dP, P, dS for one 32-row half of
// the q tile; then one of them accumulates dV and the other dK over all 64 rows, each taking its partner's
// half of the operand it needs (P^T for dV, dS^T for dK; bf16 fragments, 2 KB per wavefront) from LDS.  No
// product is computed twice, and the accumulators shrink to 64 registers.
//   M(i): dV += P^T dO or dK += dS^T Q of tile i-1 (D / 8 MFMAs), then S and dP of tile i (D / 8 MFMAs);
//   V(i): P and dS of tile i, rounded to bf16 operand slots; the partner's fragments go to the exchange area.
// Q / dO tiles are triple-buffered in LDS (padded, row-permuted layout: conflict-free row and transposed reads
// from single base registers) and fetched two tiles ahead with direct global->LDS loads: Q by group 1 at the
// start of its vector phase, dO (+ LSE, Delta) by group 0 at the start of the matrix phase it runs in the
// same slot.
//
// GQA: the q heads that read one kv head are cut into runs; a workgroup walks the q tiles of all heads of its
// run, one head after the other, into the same dK / dV accumulators (the K / V fragments are loaded once per
// run).  When a kv head has a single run its tiles are written with plain stores; otherwise the runs add theirs
// with fp32 atomics, and dk/dv must be zero-filled (or hold the running sum under HEXI_ACCUMULATE) before the
// launch.  The host picks the run length: as long as possible while the launch still has a few workgroups per CU.
#include "hexi_internal.h"
#include "hexi_mfma.h"

namespace {

constexpr int WG_KEYS = 128;     // keys per workgroup: 2 groups x 2 pairs x 32
constexpr int TM = 64;           // q rows per tile
constexpr int NB = 3;            // LDS buffers per tensor
constexpr float LOG2E = 1.4426950408889634f;

template <int D> struct BwdSmem {
    unsigned char q[NB][p16_tile_bytes(D)];   // 3 x 17 KB (D = 128) or 3 x 9 KB
    unsigned char g[NB][p16_tile_bytes(D)];   // dO, the same
    unsigned char xch[8][2048];            // per wavefront: the two fragments its partner needs (64 lanes x 16 B each)
    float lse[NB][TM];
    float delta[NB][TM];
    int qpos[8][TM];                       // row positions of the tiles that need a mask, written two tiles ahead
};

// LDS reads of matrix-phase step st (ndb = D / 32 column blocks): two transposed reads below 4 ndb (+ a fragment
// of the partner's at steps 2 ndb and 3 ndb), one row read from there on
__host__ __device__ constexpr int reads_of(int st, int ndb)
{
    return st < 4 * ndb ? 2 + ((st == 2 * ndb || st == 3 * ndb) ? 1 : 0) : 1;
}

template <int D, bool ATOMIC_DKV>
__global__ void __launch_bounds__(512) bwd_dkdv_bf16_kernel(const BwdArgs a, const HeadRuns runs, const int n_kv_tiles, const XcdSplit split)
{
    static_assert(D == 64 || D == 128, "head_dim 64 or 128");
    constexpr int NKS = D / 16;     // 16-wide contraction steps across the head dimension
    constexpr int NDB = D / 32;     // 32-column blocks of dK / dV
    constexpr int P16_ROW_BYTES = p16_row_bytes(D), P16_TILE_BYTES = p16_tile_bytes(D);
    constexpr int N_XFER = P16_TILE_BYTES / 1024;          // wave-wide transfers per tile: 17 or 9
    constexpr int DMA_PER_WAVE = (N_XFER + 3) / 4;         // most transfers a wavefront issues per tile: 5 or 3
    const AttnGeom& g = a.g;
    __shared__ __attribute__((aligned(1024))) BwdSmem<D> sm;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2, wg4 = wave & 3, pair = wg4 >> 1, role = wg4 & 1;   // role 0: dV, rows 0..31; 1: dK, rows 32..63
    const int l32 = lane & 31, hh = lane >> 5;
    const int grp2 = (lane >> 4) & 1, j16 = lane & 15;

    // Work mapping: (head run, key tile) units, run-major; each XCD takes a contiguous unit range of about equal
    // work, so that the workgroups sharing an L2 stream the same heads' Q / dO tiles.
    int unit;
    {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        unit = split.start[xcd] + slot;
        if (unit >= split.start[xcd + 1]) return;
    }
    const int run = unit / n_kv_tiles;
    const int kv_tile = unit - run * n_kv_tiles;
    const int n_heads = runs.len[run];
    const int kvh = g.kv_of_q[runs.first[run]];
    const int col0 = kv_tile * WG_KEYS;
    const int wcol0 = col0 + 64 * grp + 32 * pair;     // first key of this wavefront pair
    const int my_col = wcol0 + l32;
    const int my_col_c = my_col < g.lc ? my_col : g.lc - 1;
    const int my_kpos = my_col < g.lc ? seg_pos_of_row(g.ks, my_col) : 0x7fffffff;

    const uint16_t* k = static_cast<const uint16_t*>(a.k) + (long long)kvh * g.kv_stride_head;
    const uint16_t* v = static_cast<const uint16_t*>(a.v) + (long long)kvh * g.kv_stride_head;

    // q rows that see at least one key of the workgroup's tile form a suffix of the shard; rows that see all of
    // its keys form a (shorter) suffix
    const int last_col = (col0 + WG_KEYS < g.lc ? col0 + WG_KEYS : g.lc) - 1;
    const int k_min = seg_pos_of_row(g.ks, col0), k_max = seg_pos_of_row(g.ks, last_col);
    const int qt_begin = seg_rows_le(g.qs, k_min - 1) / TM;
    const int qt_full = (col0 + WG_KEYS <= g.lc) ? (seg_rows_le(g.qs, k_max - 1) + TM - 1) / TM : 0x7fffffff;
    const int n_qtiles = (g.lq + TM - 1) / TM;

    // K^T and V^T operand fragments of S = Q K^T and dP = dO V^T: lane (key l32, half hh) holds
    // d = 16*ks + 8*hh .. +7 of its key
    bf16x8 kf[NKS], vf[NKS];
    {
        const long long off = (long long)my_col_c * g.kv_stride_tok + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            kf[ks] = *reinterpret_cast<const bf16x8*>(k + off + 16 * ks);
            vf[ks] = *reinterpret_cast<const bf16x8*>(v + off + 16 * ks);
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) { pin(kf[ks]); pin(vf[ks]); }
    }
    // dV (role 0) or dK (role 1) of the pair's 32 keys: NDB 32-column blocks
    f32x16 acc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
    const float scale_log2 = g.scale * LOG2E;

    // Tile order within a head: first the tiles that need masking (the leading, partly visible q tiles and a
    // ragged last tile), then the fully visible ones.  The workgroup's tile sequence is that order repeated for
    // every head of the run: n_seq tiles, numbered i = 0 .. n_seq - 1 below.
    const int n_all = n_qtiles - qt_begin;
    const int n_seq = n_all > 0 ? n_all * n_heads : 0;
    const bool ragged = n_qtiles * TM > g.lq;
    const int lead = n_all > 0 ? (qt_full < n_qtiles ? qt_full : n_qtiles) - qt_begin : 0;     // partly visible tiles
    const bool extra = ragged && qt_begin + lead < n_qtiles;                                    // ragged last tile not among them
    const int n_masked = lead + (extra ? 1 : 0);
    auto tile_of = [&](int i) { return i < lead ? qt_begin + i : (i < n_masked ? n_qtiles - 1 : qt_begin + lead + (i - n_masked)); };

    // Direct global->LDS fetch of one 64-row tile by the four wavefronts of a group (group 1: Q, group 0: dO).
    // A transfer is one wave-wide instruction: lane L writes the 16 bytes at (transfer * 1024 + 16 * L) of the
    // tile's LDS image and reads the 16-byte piece of the q row that belongs there (the pad piece re-reads
    // piece 0).  Wavefront wg4 issues the transfers wg4, wg4 + 4, ... below the tile's
    // transfer count (DMA_PER_WAVE of them, or one fewer).
    uint32_t fetch_off[DMA_PER_WAVE];   // byte offsets from the tile's first row
    int fetch_row[DMA_PER_WAVE];
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; ++i) {
        const int pos = (wg4 + 4 * i) * 1024 + 16 * lane;
        int r = pos / P16_ROW_BYTES, c = (pos - r * P16_ROW_BYTES) >> 4;
        r = p16_row(r);     // the permutation is its own inverse: LDS row -> q row
        if (wg4 + 4 * i >= N_XFER) r = 0;
        if (c >= D / 8) c = 0;
        fetch_row[i] = r;
        fetch_off[i] = 2u * (uint32_t)(r * (int)g.q_stride_tok + c * 8);
    }
    const uint32_t lds_q = (uint32_t)(uintptr_t)(&sm.q[0][0]), lds_g = (uint32_t)(uintptr_t)(&sm.g[0][0]);
    const uint32_t lds_lse = (uint32_t)(uintptr_t)(&sm.lse[0][0]), lds_delta = (uint32_t)(uintptr_t)(&sm.delta[0][0]);
    const uint16_t* fetch_src = static_cast<const uint16_t*>(grp ? a.q : a.d_o);
    const uint32_t fetch_lds = grp ? lds_q : lds_g;
    // Tiles are requested in sequence order by every wavefront; (fetch_t, fetch_h) is the next one's tile
    // index within its head and its head.
    int fetch_t = 0, fetch_h = runs.first[run];
    auto fetch_tile = [&](int i) {     // i: index in the sequence; buffer i % NB
        const int qt = tile_of(fetch_t);
        const bool needs_mask = fetch_t < n_masked;
        const int row0 = qt * TM;
        const int buf = i % NB;
        const uint32_t dst = __builtin_amdgcn_readfirstlane(fetch_lds + buf * P16_TILE_BYTES + wg4 * 1024);
        const uint16_t* src = fetch_src + (long long)fetch_h * g.q_stride_head + (long long)row0 * g.q_stride_tok;
        const float* lse_h = a.lse + (long long)fetch_h * g.lq;
        const float* delta_h = a.delta + (long long)fetch_h * g.lq;
        if (++fetch_t == n_all) { fetch_t = 0; fetch_h = runs.next[fetch_h]; }
        if (row0 + TM <= g.lq) {
#pragma unroll
            for (int t = 0; t < DMA_PER_WAVE; ++t) {
                if (wg4 + 4 * t < N_XFER) lds_dma16_base(src, fetch_off[t], __builtin_amdgcn_readfirstlane(dst + t * 4096));
            }
        } else {   // ragged last tile: clamp the row index (the extra rows are masked out through their position)
#pragma unroll
            for (int t = 0; t < DMA_PER_WAVE; ++t) {
                uint32_t off = fetch_off[t];
                if (row0 + fetch_row[t] >= g.lq) off -= 2u * (uint32_t)((row0 + fetch_row[t] - (g.lq - 1)) * (int)g.q_stride_tok);
                if (wg4 + 4 * t < N_XFER) lds_dma16_base(src, off, __builtin_amdgcn_readfirstlane(dst + t * 4096));
            }
        }
        if (grp == 0) {
            // per-row scalars: one 4-byte-per-lane transfer each (LSE by wavefront 0, Delta by wavefront 1)
            if (wg4 < 2) {
                const int row = row0 + lane < g.lq ? row0 + lane : g.lq - 1;
                const float* src4 = (wg4 == 0 ? lse_h : delta_h) + row;
                lds_dma4(src4, __builtin_amdgcn_readfirstlane((wg4 == 0 ? lds_lse : lds_delta) + buf * (TM * 4)));
            }
        } else if (wg4 == 0 && needs_mask) {
            // global positions of the tile's rows, only for tiles that need masking
            sm.qpos[i & 7][lane] = row0 + lane < g.lq ? seg_pos_of_row(g.qs, row0 + lane) : -1;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    };

    // Lane parts of the LDS byte addresses; buffer and step are compile-time offsets of the reads.
    //   row fragment ks of the wavefront's 32-row half, buffer B:   nat_addr[which] + B * TILE + 32 * ks
    //       (which = 0: Q tile for S, 1: dO tile for dP)
    //   transposed fragment (16-row step kq of a 32-row half, 32-column block db, half `second`) of buffer B:
    //   rows 16kq + 8*second + 4*hh + jj of the half sit in LDS rows 16kq + 4*jj + 2*second + hh of it:
    //        tr_addr[half] + B * TILE + (16 * kq + 2 * second) * ROW + 64 * db
    //       (the dO tile for the dV wavefront, the Q tile for the dK wavefront; half 0: its own rows, 1: its partner's)
    //   the partner's fragment f:  xch_partner + f * 1024
    const int jj = j16 >> 2;
    const uint32_t nat_lane = (32 * role + p16_row(l32)) * P16_ROW_BYTES + 16 * hh;
    const uint32_t tr_lane = (role ? lds_q : lds_g) + (4 * jj + hh) * P16_ROW_BYTES + 2 * (16 * grp2 + 4 * (j16 & 3));
    uint32_t nat_addr[2] = {lds_q + nat_lane, lds_g + nat_lane};
    uint32_t tr_addr[2] = {tr_lane + 32 * role * P16_ROW_BYTES, tr_lane + 32 * (1 - role) * P16_ROW_BYTES};   // own rows, partner's rows
    const uint32_t xch_partner = (uint32_t)(uintptr_t)(&sm.xch[wave ^ 1][0]) + lane * 16;
    bf16x8* xch_mine = reinterpret_cast<bf16x8*>(&sm.xch[wave][0]) + lane;

    f32x16 s, dp;
    bf16x8 own[2];     // own operand fragments (P^T for the dV wavefront, dS^T for the dK wavefront)

    // Matrix phase on buffers (B + NB - 1) % NB (previous tile) and B (this tile).  Steps 0..NACC-1: this
    // wavefront's product (dV += P^T dO or dK += dS^T Q) of the previous tile: the first half of them contract
    // over its own 32 rows (fragments in registers), the second half over its partner's (fragments from LDS);
    // 16-row step (st / NDB) % 2, column block st % NDB.  Steps NACC..NST-1: S and dP of this tile's 32-row half,
    // alternating, ks = (st - NACC) / 2.  [FIRST, LAST) selects the steps; operand fragments are requested PF
    // steps ahead.
    constexpr int NACC = 4 * NDB, NST = NACC + 2 * NKS;
    auto m_phase = [&](auto bc, auto first_c, auto last_c) __attribute__((always_inline)) {
        constexpr int B = decltype(bc)::value, FIRST = decltype(first_c)::value, LAST = decltype(last_c)::value;
        constexpr int PF = 3, NS = PF + 1;   // a fragment's registers are busy from its request until its MFMA
        constexpr int BP = (B + NB - 1) % NB;
        s16x4 ta[NS], tb[NS];
        bf16x8 nb[NS];
        bf16x8 pfr[2];                       // the partner's two fragments
        auto issue = [&](auto stc) __attribute__((always_inline)) {
            constexpr int st = decltype(stc)::value, slot = (st - FIRST) % NS;
            if constexpr (st < NACC) {
                constexpr int half = st / (2 * NDB), kq = (st / NDB) & 1, db = st % NDB;
                if constexpr (st == 2 * NDB || st == 3 * NDB) lds_issue_b128<kq * 1024>(pfr[kq], xch_partner);
                constexpr int off = BP * P16_TILE_BYTES + 16 * kq * P16_ROW_BYTES + 64 * db;
                lds_issue_tr16<off>(ta[slot], tr_addr[half]);
                lds_issue_tr16<off + 2 * P16_ROW_BYTES>(tb[slot], tr_addr[half]);
            } else {
                constexpr int which = (st - NACC) & 1, ks = (st - NACC) >> 1;
                lds_issue_b128<B * P16_TILE_BYTES + 32 * ks>(nb[slot], nat_addr[which]);
            }
        };
        auto step = [&](auto stc) __attribute__((always_inline)) {
            constexpr int st = decltype(stc)::value, slot = (st - FIRST) % NS;
            if constexpr (st + PF < LAST) issue(IC<st + PF>{});
            constexpr int hi = st + PF < LAST ? st + PF : LAST - 1;
            constexpr int younger = (hi >= st + 1 ? reads_of(st + 1, NDB) : 0) + (hi >= st + 2 ? reads_of(st + 2, NDB) : 0) +
                                    (hi >= st + 3 ? reads_of(st + 3, NDB) : 0);
            static_assert(PF == 3, "the sum above covers three steps");
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if constexpr (st < NACC) {
                constexpr int half = st / (2 * NDB), kq = (st / NDB) & 1, db = st % NDB;
                if constexpr (half == 0) {
                    lds_wait<younger>(ta[slot], tb[slot]);
                    acc[db] = mfma32(own[kq], join_halves(ta[slot], tb[slot]), acc[db]);
                } else {
                    // the wait ties all three registers: the partner's fragment was requested before the transposed pair
                    asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(ta[slot]), "+v"(tb[slot]), "+v"(pfr[kq]) : "n"(younger));
                    acc[db] = mfma32(pfr[kq], join_halves(ta[slot], tb[slot]), acc[db]);
                }
            } else {
                constexpr int which = (st - NACC) & 1, ks = (st - NACC) >> 1;
                lds_wait<younger>(nb[slot]);
                if constexpr (which == 0) s = mfma32(nb[slot], kf[ks], ks == 0 ? zero : s);
                else dp = mfma32(nb[slot], vf[ks], ks == 0 ? zero : dp);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        __builtin_amdgcn_sched_barrier(0);
        for_range<FIRST, (FIRST + PF < LAST ? FIRST + PF : LAST)>(issue);
        for_range<FIRST, LAST>(step);
    };

    // Vector phase: P and dS of the wavefront's 32 rows x 32 keys.  Register x = 4*rb + t holds row
    // 32*role + 8*rb + 4*hh + t.  Rows whose LSE is -inf see nothing anywhere, so they only occur in masked tiles.
    auto v_phase = [&](int buf, int qpos_slot, auto masked_c) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_c)::value;
        float p[16], ds[16];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            const int r0 = 32 * role + 8 * rb + 4 * hh;
            const f32x4 l4 = *reinterpret_cast<const f32x4*>(&sm.lse[buf][r0]);
            const f32x4 d4 = *reinterpret_cast<const f32x4*>(&sm.delta[buf][r0]);
            int4 qp = make_int4(0, 0, 0, 0);
            if (MASKED) qp = *reinterpret_cast<const int4*>(&sm.qpos[qpos_slot][r0]);
            const int qpv[4] = {qp.x, qp.y, qp.z, qp.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int x = 4 * rb + t;
                float pv = fast_exp2(fmaf(s[x], scale_log2, l4[t]));
                if (MASKED) pv = my_kpos > qpv[t] ? 0.f : pv;
                p[x] = pv;
                ds[x] = pv * (dp[x] - d4[t]);
            }
        }
        const bf16x8 p0 = pack_bf16x8(p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]);
        const bf16x8 p1 = pack_bf16x8(p[8], p[9], p[10], p[11], p[12], p[13], p[14], p[15]);
        const bf16x8 d0 = pack_bf16x8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
        const bf16x8 d1 = pack_bf16x8(ds[8], ds[9], ds[10], ds[11], ds[12], ds[13], ds[14], ds[15]);
        // the dV wavefront keeps P^T and hands dS^T to its partner; the dK wavefront the other way round
        if (role == 0) { own[0] = p0; own[1] = p1; xch_mine[0] = d0; xch_mine[64] = d1; }
        else { own[0] = d0; own[1] = d1; xch_mine[0] = p0; xch_mine[64] = p1; }
        // the fragments must be in LDS before the barrier that ends this phase
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(own[0]), "+v"(own[1]) :: "memory");
    };

    // Phase sequence of a group: M(0) V(0) M(1) V(1) ... M(n_seq), a barrier before every phase; group 1
    // starts one barrier late and group 0 ends with one extra.  Tile i + 2 is requested in the slot in which
    // group 0 runs M(i + 1) and group 1 runs V(i), and must have landed two slots later: both groups wait for
    // their own transfers at the end of the phase in between.
    if (n_seq > 0) {
        int proc_t = 0;     // tile index within its head of the tile in the vector phase
        fetch_tile(0);
        if (n_seq > 1) fetch_tile(1);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        // The vector phase uses the row constant -log2(e) * LSE: each tile's 64 LSE values are converted in
        // place once they have landed (one multiply per tile instead of 16 per wavefront): tile 0 here, by the
        // wavefront that fetched it; tile i + 1 by a wavefront of group 1 at the start of its vector phase of
        // tile i, the slot before the first vector phase that reads it.
        if (grp == 0 && wg4 == 0) {
            sm.lse[0][lane] = sm.lse[0][lane] * -LOG2E;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        if (grp == 1) wg_barrier();
        auto enter_m = [&](int i) __attribute__((always_inline)) {
            if (grp == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            wg_barrier();
            if (grp == 0 && i >= 1 && i + 1 < n_seq) fetch_tile(i + 1);
        };
        auto vector_part = [&](int i) __attribute__((always_inline)) {
            if (grp == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            wg_barrier();
            if (grp == 1 && i + 2 < n_seq) fetch_tile(i + 2);
            if (grp == 1 && wg4 == 3 && i + 1 < n_seq) sm.lse[(i + 1) % NB][lane] = sm.lse[(i + 1) % NB][lane] * -LOG2E;
            if (proc_t < n_masked) v_phase(i % NB, i & 7, std::true_type{});
            else v_phase(i % NB, i & 7, std::false_type{});
            if (++proc_t == n_all) proc_t = 0;
        };
        enter_m(0); m_phase(IC<0>{}, IC<NACC>{}, IC<NST>{}); vector_part(0);
        // tiles 1 .. n_seq-1: three at a time in a straight line (buffer = i % 3 is then a compile-time constant
        // and no accumulator passes through a control-flow merge), then the remaining ones through a switch
        int i = 1;
        for (; i + 2 < n_seq; i += 3) {
            enter_m(i);     m_phase(IC<1>{}, IC<0>{}, IC<NST>{}); vector_part(i);
            enter_m(i + 1); m_phase(IC<2>{}, IC<0>{}, IC<NST>{}); vector_part(i + 1);
            enter_m(i + 2); m_phase(IC<0>{}, IC<0>{}, IC<NST>{}); vector_part(i + 2);
        }
        for (; i < n_seq; ++i) {
            enter_m(i);
            switch (i % NB) {
                case 0: m_phase(IC<0>{}, IC<0>{}, IC<NST>{}); break;
                case 1: m_phase(IC<1>{}, IC<0>{}, IC<NST>{}); break;
                default: m_phase(IC<2>{}, IC<0>{}, IC<NST>{}); break;
            }
            vector_part(i);
        }
        enter_m(n_seq);
        switch (n_seq % NB) {
            case 0: m_phase(IC<0>{}, IC<0>{}, IC<NACC>{}); break;
            case 1: m_phase(IC<1>{}, IC<0>{}, IC<NACC>{}); break;
            default: m_phase(IC<2>{}, IC<0>{}, IC<NACC>{}); break;
        }
        if (grp == 0) wg_barrier();
    }

    // dV (role 0) or dK (role 1): lane holds column d = 32*db + l32; register r holds key wcol0 + 8*(r/4) + 4*hh + r%4
    float* out = role ? a.dk : a.dv;
    const float out_scale = role ? g.scale : 1.0f;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int col = wcol0 + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (col < g.lc) {
                const long long idx = ((long long)col * g.nkv + kvh) * D + 32 * db + l32;
                const float val = acc[db][r] * out_scale;
                if (ATOMIC_DKV) global_atomic_add(out + idx, val);
                else if (a.accumulate) out[idx] += val;
                else out[idx] = val;
            }
        }
}

}  // namespace

hipError_t hexi_launch_bwd_bf16(const BwdArgs& a, hipStream_t s)
{
    if (a.want_dkdv) {
        const int n_kv_tiles = (a.g.lc + WG_KEYS - 1) / WG_KEYS;
        // q heads per kv head, in head order
        int cnt[HEXI_MAX_HEADS] = {0};
        int max_cnt = 0;
        bool unused = false;
        for (int h = 0; h < a.g.nq; ++h) {
            const int c = ++cnt[a.g.kv_of_q[h]];
            max_cnt = c > max_cnt ? c : max_cnt;
        }
        for (int kh = 0; kh < a.g.nkv; ++kh) unused |= (cnt[kh] == 0);   // a kv head no local q head reads: zero gradient
        // Run length: the longest divisor of the largest group's size (so that its runs are equally long) for which
        // the launch still has about three workgroups per CU and a workgroup walks at most 512 q tiles.  A run
        // amortises the workgroup's prologue and epilogue (about 20 tiles' worth) and, when it covers the whole
        // group, needs no atomics; but the workgroups of an XCD stream the same Q / dO tiles only while they stay
        // in step, and long tile sequences let them drift apart (measured: more L2 misses, slower launches).
        auto n_runs_for = [&](int len) {
            int n = 0;
            for (int kh = 0; kh < a.g.nkv; ++kh) n += (cnt[kh] + len - 1) / len;
            return n;
        };
        // q tiles that see the chunk's first key: the longest tile sequence of one head
        const int n_qtiles = (a.g.lq + TM - 1) / TM;
        const int max_tiles = a.g.lc > 0 ? n_qtiles - seg_rows_le(a.g.qs, seg_pos_of_row(a.g.ks, 0) - 1) / TM : 0;
        int run_len = max_cnt;
        while (run_len > 1 && (max_cnt % run_len != 0 || (long long)run_len * max_tiles > 512 ||
                               (long long)n_runs_for(run_len) * n_kv_tiles < 3 * 256))
            --run_len;
        if (const int forced = hexi_dkdv_run_len; forced >= 1)      // tuning / test override of the heuristic
            run_len = forced < max_cnt ? forced : max_cnt;
        HeadRuns runs;
        const bool shared = hexi_build_head_runs(a.g.kv_of_q, a.g.nq, a.g.nkv, run_len, &runs);
        // cost of a unit: the q tiles its key tile sees, once per head of the run, plus the prologue and epilogue
        // (about 20 tiles' worth)
        float seen[4096];
        const int n_known = n_kv_tiles < 4096 ? n_kv_tiles : 4096;     // (longer chunks: the remaining tiles count like the last known one)
        for (int t = 0; t < n_known; ++t) {
            const int k_min = seg_pos_of_row(a.g.ks, t * WG_KEYS);
            const int n_all = n_qtiles - seg_rows_le(a.g.qs, k_min - 1) / TM;
            seen[t] = (float)(n_all > 0 ? n_all : 0);
        }
        unsigned grid = 0;
        const XcdSplit split = hexi_split_units(runs.n * n_kv_tiles, [&](int u) {
            const int run = u / n_kv_tiles, t = u - run * n_kv_tiles;
            return (float)runs.len[run] * seen[t < n_known ? t : n_known - 1] + 20.0f;
        }, &grid);
        if ((shared || unused) && !a.accumulate) {
            const long long n = (long long)a.g.lc * a.g.nkv * a.g.d;
            hipError_t e = hexi_launch_fill_f32(a.dk, n, 0.f, s);
            if (e == hipSuccess) e = hexi_launch_fill_f32(a.dv, n, 0.f, s);
            if (e != hipSuccess) return e;
        }
        if (a.g.d != 128 && a.g.d != 64) return hipErrorInvalidValue;
        if (grid > 0) {
            if (a.g.d == 128) {
                if (shared) bwd_dkdv_bf16_kernel<128, true><<<grid, 512, 0, s>>>(a, runs, n_kv_tiles, split);
                else bwd_dkdv_bf16_kernel<128, false><<<grid, 512, 0, s>>>(a, runs, n_kv_tiles, split);
            } else {
                if (shared) bwd_dkdv_bf16_kernel<64, true><<<grid, 512, 0, s>>>(a, runs, n_kv_tiles, split);
                else bwd_dkdv_bf16_kernel<64, false><<<grid, 512, 0, s>>>(a, runs, n_kv_tiles, split);
            }
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return a.want_dq ? hexi_launch_bwd_dq_bf16(a, s) : hipSuccess;
}
