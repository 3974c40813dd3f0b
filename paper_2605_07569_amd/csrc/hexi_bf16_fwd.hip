// bf16 forward ring step for gfx950 (head_dim D = 128 or 64): one workgroup of 8 wavefronts per (256-row q
// tile, q head), one workgroup per CU.
//
// Ping-pong schedule.  On this hardware a wavefront that has just issued an MFMA cannot issue its own
// VALU work for most of the MFMA's duration, but ANOTHER wavefront of the same SIMD can: a wavefront
// issuing only MFMAs runs the matrix pipe at its full rate while its SIMD partner issues VALU
// instructions at nearly their solo rate.  The workgroup is therefore two groups of four wavefronts
// (wavefront w and w + 4 share a SIMD), each group owning 128 query rows, that alternate between
//   M(t): the matrix phase  -- O^T += V^T P^T of tile t-1, then S^T = K Q^T of tile t (D / 4 MFMAs), and
//   V(t): the vector phase  -- softmax numerators of tile t, P rounded to bf16 operand slots,
// group 1 running one phase behind group 0, so that a SIMD mostly has one wavefront in a matrix phase and one
// in a vector phase.  One workgroup barrier per tile keeps the groups in step and publishes the tiles that
// have landed: group 0 passes it before its matrix phase, group 1 before its vector phase; the second phase
// of each follows without a barrier (a barrier per phase was measured 2 % slower).  The vector-phase group also issues the
// direct global->LDS loads of upcoming tiles (group 1 fetches K four tiles ahead, group 0 fetches V two
// tiles ahead; four LDS buffers per tensor).
//
// As before the scores are computed transposed (S^T = K Q^T) so that every lane owns one query row,
// softmax state is a per-lane scalar, and the accumulator registers holding P^T are already in MFMA
// operand order for O^T += V^T P^T.  K / V tiles (64 keys) sit in LDS with padded rows so that the 128-bit
// row reads of K and the transposed 64-bit reads of V are bank-conflict free.
//
// Softmax reference.  The vector phase must stay short (it is the co-limiter), so the fast path does not
// track a running maximum: the reference m of a row is fixed after its first tile (the row maximum over
// that tile's visible keys) and every later probability is exp2(s - m) against that same m.  This is
// exact as long as nothing over- or underflows, which fp32 / bf16 exponents guarantee unless a later
// score differs from the first tile's maximum by more than about 2^100.  Each row checks its final sum
// against [2^-60, 2^60]; if any row of the workgroup fails, the whole workgroup repeats its tiles with
// the exact online-softmax path (running maximum, lazy rescale).  Rows in the fast path keep two sums:
// the exact one defines the LSE, the one of the bf16-rounded probabilities normalises O.
#include "hexi_internal.h"
#include "hexi_mfma.h"

namespace {

constexpr int TN = 64;             // keys per tile
constexpr int NB = 4;              // LDS buffers per tensor
constexpr int GROUP_ROWS = 128;    // q rows per wavefront group (32 per wavefront)
constexpr int WG_ROWS = 256;       // q rows per workgroup
// LDS rows are padded instead of swizzled, so that every operand fragment sits at (one per-lane base
// register) + (compile-time offset): K rows take 2 D + 16 bytes (272 or 144: 16 consecutive rows then spread
// over all 64 banks for the 128-bit row reads), V rows 2 D + 64 bytes (320 or 192: the 4 rows x 64 bytes of a
// transposed 64-bit read then spread over all 64 banks).  Tiles are whole numbers of wave-wide 1 KB transfers:
// K 17 (D = 128) or 9 (D = 64), V 20 or 12.
template <int D> struct FwdCfg {
    static_assert(D == 64 || D == 128, "head_dim 64 or 128");
    static constexpr int NKS = D / 16;     // 16-wide contraction steps across the head dimension
    static constexpr int NDB = D / 32;     // 32-column blocks of the output
    static constexpr int K_ROW_BYTES = 2 * D + 16, V_ROW_BYTES = 2 * D + 64;
    static constexpr int K_TILE_BYTES = TN * K_ROW_BYTES, V_TILE_BYTES = TN * V_ROW_BYTES;
    static constexpr int DMA_PER_WAVE = (V_TILE_BYTES / 1024 + 3) / 4;   // most transfers a wavefront issues per tile (5 or 3)
    static constexpr int O_STAGE_STRIDE = D + 4;   // floats per staged output row (epilogue)
    static_assert(K_TILE_BYTES % 1024 == 0 && V_TILE_BYTES % 1024 == 0, "tiles are whole transfers");
    static_assert((K_TILE_BYTES / 1024 + 3) / 4 == DMA_PER_WAVE, "K and V wavefronts issue the same maximum");
};
constexpr int K_AHEAD = 4;         // group 1 fetches K(t + 4) during V(t)
constexpr int V_AHEAD = 2;         // group 0 fetches V(t + 2) during V(t)
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float NEG_BIG = -1.0e30f;   // finite stand-in for "no key seen yet"
constexpr float RESCALE_SLACK = 8.0f;
constexpr float SUM_LO = 8.6736174e-19f;   // 2^-60
constexpr float SUM_HI = 1.1529215e18f;    // 2^60

template <int D> struct FwdSmem {
    unsigned char k[NB][FwdCfg<D>::K_TILE_BYTES];   // 4 x 17 KB (D = 128)
    unsigned char v[NB][FwdCfg<D>::V_TILE_BYTES];   // 4 x 20 KB
    int kpos[2 * NB][TN];     // key positions of the tiles that need a mask, written K_AHEAD tiles ahead
    // The epilogue stages 8 x (32 x (D + 4) + 32) floats over the start of this struct: the regions of wavefronts
    // 4..7 lie over v[], so every wavefront must be done with the tiles (a workgroup barrier) before any stages.
};

template <int D>
__global__ void __launch_bounds__(512) fwd_bf16_kernel(const FwdArgs a, const int n_q_tiles, const XcdSplit split)
{
    using C = FwdCfg<D>;
    constexpr int NKS = C::NKS, NDB = C::NDB, K_ROW_BYTES = C::K_ROW_BYTES, V_ROW_BYTES = C::V_ROW_BYTES;
    constexpr int K_TILE_BYTES = C::K_TILE_BYTES, V_TILE_BYTES = C::V_TILE_BYTES, DMA_PER_WAVE = C::DMA_PER_WAVE;
    constexpr int O_STAGE_STRIDE = C::O_STAGE_STRIDE;
    constexpr bool PAIR_BARRIER = D == 128;     // one workgroup barrier per pair of phases instead of one per phase
    static_assert(sizeof(FwdSmem<D>) >= 8 * (32 * O_STAGE_STRIDE + 32) * 4, "epilogue staging does not fit");
    const AttnGeom& g = a.g;
    __shared__ __attribute__((aligned(1024))) FwdSmem<D> sm;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2, wg = wave & 3;
    const int l32 = lane & 31, hh = lane >> 5;
    const int grp2 = (lane >> 4) & 1, j16 = lane & 15;

    // Work mapping: (head, q tile) units, head-major; within a head the q tiles are taken from the end of the shard
    // backwards (under a causal mask the last tiles see the most keys, and starting the longest units first evens
    // out the tail).  Each XCD takes a contiguous unit range of about equal work, so the workgroups sharing an L2
    // stream the same kv head.
    int unit;
    {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        unit = split.start[xcd] + slot;
        if (unit >= split.start[xcd + 1]) return;
    }
    const int h = unit / n_q_tiles;
    const int q_tile = n_q_tiles - 1 - (unit - h * n_q_tiles);
    const int kvh = g.kv_of_q[h];
    const int row0 = q_tile * WG_ROWS;
    const int grow0 = row0 + GROUP_ROWS * grp;
    const int my_row = grow0 + 32 * wg + l32;
    const int my_row_c = my_row < g.lq ? my_row : g.lq - 1;
    const int my_pos = my_row < g.lq ? seg_pos_of_row(g.qs, my_row) : -1;

    const uint16_t* q = static_cast<const uint16_t*>(a.q);
    const uint16_t* k = static_cast<const uint16_t*>(a.k) + (long long)kvh * g.kv_stride_head;
    const uint16_t* v = static_cast<const uint16_t*>(a.v) + (long long)kvh * g.kv_stride_head;

    // Visible keys of a row range form a prefix of the chunk; keys visible to every row of the range a
    // shorter prefix.  n_full_g: tiles this group needs no mask for (the rest are masked by position).
    // NT: tiles the workgroup streams (those of its last rows); n_full_wg: tiles no row needs a mask for.
    int n_full_g = 0;
    if (grow0 < g.lq) n_full_g = seg_rows_le(g.ks, seg_pos_of_row(g.qs, grow0)) / TN;
    const int wg_last_row = (row0 + WG_ROWS < g.lq ? row0 + WG_ROWS : g.lq) - 1;
    const int NT = (seg_rows_le(g.ks, seg_pos_of_row(g.qs, wg_last_row)) + TN - 1) / TN;
    const int n_full_wg = seg_rows_le(g.ks, seg_pos_of_row(g.qs, row0)) / TN;

    // A workgroup whose rows see nothing of the chunk leaves the running (o, lse) as they are: merging an empty
    // partial is the identity.  (Without HEXI_ACCUMULATE it goes on and writes o = 0, lse = -inf.)
    if (NT == 0 && a.accumulate) return;

    // Q^T operand fragments: lane (row l32, half hh) holds d = 16*ks + 8*hh .. +7
    bf16x8 qf[NKS];
    {
        const uint16_t* qp = q + (long long)my_row_c * g.q_stride_tok + (long long)h * g.q_stride_head + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) pin(qf[ks]);
    }

    // Direct global->LDS fetch of one tile by the four wavefronts of a group.  A transfer is one wave-wide
    // instruction: lane L writes the 16 bytes at (transfer * 1024 + 16 * L) of the tile's LDS image and reads
    // them from wherever the kernel points it, here the 16-byte piece of the key row that belongs there (pad
    // pieces re-read piece 0).  Wavefront wg issues the transfers wg, wg + 4, ... below the tile's transfer
    // count (at most DMA_PER_WAVE of them).
    const int row_bytes = grp ? K_ROW_BYTES : V_ROW_BYTES;
    const int n_xfer = grp ? K_TILE_BYTES / 1024 : V_TILE_BYTES / 1024;
    // transfers this wavefront issues per tile: its share wg, wg + 4, ... of the tile's n_xfer (4 or 5)
    const int my_xfers = (n_xfer - wg + 3) / 4;
    uint32_t fetch_off[DMA_PER_WAVE];   // byte offsets from the tile's first key
    int fetch_row[DMA_PER_WAVE];
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; ++i) {
        const int pos = (wg + 4 * i) * 1024 + 16 * lane;
        int r = pos / row_bytes, c = (pos - r * row_bytes) >> 4;
        if (wg + 4 * i >= n_xfer) r = 0;
        if (c >= D / 8) c = 0;
        fetch_row[i] = r;
        fetch_off[i] = 2u * (uint32_t)(r * (int)g.kv_stride_tok + c * 8);
    }
    const uint32_t lds_k = (uint32_t)(uintptr_t)(&sm.k[0][0]), lds_v = (uint32_t)(uintptr_t)(&sm.v[0][0]);
    const uint16_t* fetch_src = grp ? k : v;                 // group 1 streams K, group 0 streams V
    const uint32_t fetch_lds = grp ? lds_k : lds_v;
    const int fetch_tile_bytes = grp ? K_TILE_BYTES : V_TILE_BYTES;
    auto fetch_tile = [&](int tile) {
        const int col0 = tile * TN;
        const uint32_t dst = __builtin_amdgcn_readfirstlane(fetch_lds + (tile & (NB - 1)) * fetch_tile_bytes + wg * 1024);
        const uint16_t* src = fetch_src + (long long)col0 * g.kv_stride_tok;
        if (col0 + TN <= g.lc) {
#pragma unroll
            for (int i = 0; i < DMA_PER_WAVE; ++i) {
                if (wg + 4 * i < n_xfer) lds_dma16_base(src, fetch_off[i], __builtin_amdgcn_readfirstlane(dst + i * 4096));
            }
        } else {   // ragged last tile: clamp the key index (the extra keys are masked through their position)
#pragma unroll
            for (int i = 0; i < DMA_PER_WAVE; ++i) {
                uint32_t off = fetch_off[i];
                if (col0 + fetch_row[i] >= g.lc) off -= 2u * (uint32_t)((col0 + fetch_row[i] - (g.lc - 1)) * (int)g.kv_stride_tok);
                if (wg + 4 * i < n_xfer) lds_dma16_base(src, off, __builtin_amdgcn_readfirstlane(dst + i * 4096));
            }
        }
        // global positions of the tile's keys, for the tiles some row needs a mask for
        if (grp == 1 && wg == 0 && tile >= n_full_wg) {
            sm.kpos[tile & (2 * NB - 1)][lane] = col0 + lane < g.lc ? seg_pos_of_row(g.ks, col0 + lane) : 0x7fffffff;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    };

    // Lane parts of the LDS byte addresses; buffer, key block and step are compile-time offsets of the reads.
    //   K fragment (ks, block b) of buffer B:   k_addr  + B * K_TILE_BYTES + 32 * b * K_ROW_BYTES + 32 * ks
    //   V^T fragment (16-key step u, 32-column block db, half `second`) of buffer BV:
    //        v_addr[BV / 2] + (BV % 2) * V_TILE_BYTES + (16 * u + 8 * second) * V_ROW_BYTES + 64 * db
    // (two base registers for V: the offset field of an LDS read holds 16 bits).  A transposed read hands
    // lane i of a 16-lane group the elements [row0 + e][col0 + i], e = 0..3, where lane j supplies the address
    // of [row0 + j/4][col0 + 4*(j%4)].
    const int jj = j16 >> 2;
    const uint32_t k_addr = lds_k + l32 * K_ROW_BYTES + 16 * hh;
    uint32_t v_addr[2];
    v_addr[0] = lds_v + (4 * hh + jj) * V_ROW_BYTES + 2 * (16 * grp2 + 4 * (j16 & 3));
    v_addr[1] = v_addr[0] + 2 * V_TILE_BYTES;

    f32x16 oacc[NDB];
    f32x16 s[2];
    bf16x8 pf[4];
    float m_run, l_run, lr_run, thr_raw;
    const float c_log2 = g.scale * LOG2E, inv_c_log2 = 1.0f / c_log2;

    // Matrix phase on buffers (B + NB - 1) % NB (V of tile t-1) and B (K of tile t).  Steps 0..NPV-1:
    // O^T[d][q] += V^T P^T, four 16-key steps x NDB 32-column blocks; steps NPV..NST-1: S^T[key][q] for two
    // 32-key blocks.  [FIRST, LAST) selects the steps; operand fragments are requested PF steps ahead.
    constexpr int NPV = 4 * NDB, NST = NPV + 2 * NKS;
    auto m_phase = [&](auto bc, auto first_c, auto last_c) __attribute__((always_inline)) {
        constexpr int B = decltype(bc)::value, FIRST = decltype(first_c)::value, LAST = decltype(last_c)::value;
        constexpr int PF = 4;
        constexpr int BV = (B + NB - 1) % NB;
        constexpr int KOFF = B * K_TILE_BYTES, VOFF = (BV % 2) * V_TILE_BYTES;
        constexpr int NS = PF + 1;   // a fragment's registers are busy from its request until its MFMA
        s16x4 ta[NS], tb[NS];
        bf16x8 kb[NS];
        auto issue = [&](auto stc) __attribute__((always_inline)) {
            constexpr int st = decltype(stc)::value, slot = (st - FIRST) % NS;
            if constexpr (st < NPV) {
                constexpr int u = st / NDB, db = st % NDB;
                lds_issue_tr16<VOFF + 16 * u * V_ROW_BYTES + 64 * db>(ta[slot], v_addr[BV / 2]);
                lds_issue_tr16<VOFF + (16 * u + 8) * V_ROW_BYTES + 64 * db>(tb[slot], v_addr[BV / 2]);
            } else {
                constexpr int b = (st - NPV) & 1, ks = (st - NPV) >> 1;
                lds_issue_b128<KOFF + 32 * b * K_ROW_BYTES + 32 * ks>(kb[slot], k_addr);
            }
        };
        auto step = [&](auto stc) __attribute__((always_inline)) {
            constexpr int st = decltype(stc)::value, slot = (st - FIRST) % NS;
            if constexpr (st + PF < LAST) issue(IC<st + PF>{});
            // LDS reads younger than this step's fragment: those of the next PF steps that exist
            constexpr int hi = st + PF < LAST ? st + PF : LAST - 1;
            constexpr int n_tr = (hi < NPV ? hi : NPV - 1) - (st < NPV ? st : NPV - 1);      // steps in (st, hi] below NPV
            constexpr int younger = 2 * n_tr + ((hi - st) - n_tr);
            if constexpr (st < NPV) {
                lds_wait<younger>(ta[slot], tb[slot]);
                oacc[st % NDB] = mfma32(join_halves(ta[slot], tb[slot]), pf[st / NDB], oacc[st % NDB]);
            } else {
                constexpr int b = (st - NPV) & 1, ks = (st - NPV) >> 1;
                lds_wait<younger>(kb[slot]);
                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                s[b] = mfma32(kb[slot], qf[ks], ks == 0 ? zero : s[b]);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        __builtin_amdgcn_sched_barrier(0);
        for_range<FIRST, (FIRST + PF < LAST ? FIRST + PF : LAST)>(issue);
        for_range<FIRST, LAST>(step);
    };

    // Vector phase: probabilities of the tile whose scores sit in s[], rounded to bf16 operand slots.
    // Two running sums: `l_run` of the exact values (it defines the LSE that the merge and the backward
    // pass use) and `lr_run` of the rounded values (it normalises O, so that O is an exact convex
    // combination with the weights the PV product really used).  Both are per-half partial sums; the two
    // half-waves are added at the end.
    //   MASKED: the tile needs the causal mask (key positions from LDS).
    //   exact:  online softmax -- running maximum raised lazily (only when a tile exceeds it by more than
    //           2^8; then O and the sums are rescaled).  Otherwise the reference is fixed by the first tile.
    auto v_phase = [&](int buf, auto first_c, auto masked_c, const bool exact) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_c)::value, first_tile = decltype(first_c)::value;
        if (MASKED) {
            const int* kp = &sm.kpos[buf][0];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const int4 p4 = *reinterpret_cast<const int4*>(&kp[32 * b + 8 * rb + 4 * hh]);
                    if (p4.x > my_pos) s[b][4 * rb] = -INFINITY;
                    if (p4.y > my_pos) s[b][4 * rb + 1] = -INFINITY;
                    if (p4.z > my_pos) s[b][4 * rb + 2] = -INFINITY;
                    if (p4.w > my_pos) s[b][4 * rb + 3] = -INFINITY;
                }
        }
        if (exact || first_tile) {
            float mx = max3(s[0][0], s[0][1], s[0][2]);
#pragma unroll
            for (int r = 3; r < 15; r += 2) mx = max3(mx, s[0][r], s[0][r + 1]);
            mx = max3(mx, s[0][15], s[1][0]);
#pragma unroll
            for (int r = 1; r < 15; r += 2) mx = max3(mx, s[1][r], s[1][r + 1]);
            mx = max_across_halves(max2(mx, s[1][15]));
            if (exact) {
                // mx is the raw score; thr_raw = (m_run + slack) / c
                if (__any(mx > thr_raw)) {
                    const float m_new = fmaxf(m_run, mx * c_log2);
                    const float alpha = fast_exp2(m_run - m_new);
                    l_run *= alpha;
                    lr_run *= alpha;
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
                    m_run = m_new;
                    thr_raw = (m_run + RESCALE_SLACK) * inv_c_log2;
                }
            } else {
                m_run = mx == -INFINITY ? 0.f : mx * c_log2;   // a row that sees nothing in the first tile sees nothing at all
            }
        }
        // four independent partial sums per kind: a chain of 32 dependent additions would serialise the phase
        float ps[4] = {0.f, 0.f, 0.f, 0.f}, psr[4] = {0.f, 0.f, 0.f, 0.f};
        const float neg_m = -m_run;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int b = u >> 1, x = (u & 1) * 8;
            float p[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) { p[e] = fast_exp2(fmaf(s[b][x + e], c_log2, neg_m)); ps[e & 3] += p[e]; }
            pf[u] = pack_bf16x8_sum4(p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7], psr);
        }
        l_run += (ps[0] + ps[1]) + (ps[2] + ps[3]);
        lr_run += (psr[0] + psr[1]) + (psr[2] + psr[3]);
        // keep the whole vector phase on this side of the next barrier (nothing of it may drift into the
        // matrix phase, where it would hold registers and steal issue slots from the MFMA stream)
        asm volatile("" : "+v"(l_run), "+v"(lr_run), "+v"(pf[0]), "+v"(pf[1]), "+v"(pf[2]), "+v"(pf[3]));
    };

    // One pass over the workgroup's tiles.  Phase sequence of a group: M(0) V(0) M(1) V(1) ... M(NT); group 0
    // passes a workgroup barrier before every matrix phase, group 1 before its first matrix phase and before
    // every vector phase (NT + 1 barriers each), which keeps group 1 one phase behind group 0.  Both
    // groups walk all NT tiles (a group whose rows see fewer tiles masks the rest away), so the control
    // flow is the same everywhere.
    // (The softmax variant is a compile-time parameter: with a run-time flag the compiler keeps both variants'
    // state alive through the tile loop, which cost the fast path 3 %.)
    auto run = [&](auto exact_c) __attribute__((always_inline)) {
        constexpr bool exact = decltype(exact_c)::value;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
        m_run = NEG_BIG; l_run = 0.f; lr_run = 0.f;
        thr_raw = NEG_BIG;   // any finite score exceeds it: the first visible tile always sets the maximum
        if (NT == 0) return;
        // prologue: group 1 requests K(0..3), group 0 requests V(0..1)
        {
            const int n_pre = grp ? K_AHEAD : V_AHEAD;
            for (int j = 0; j < n_pre && j < NT; ++j) fetch_tile(j);
        }
        if (grp == 1) {   // K(0) complete before anyone's M(0)
            wait_tiles_in_flight<DMA_PER_WAVE>((NT < K_AHEAD ? NT : K_AHEAD) - 1, my_xfers);
            wg_barrier();
        }
        // One workgroup barrier B(t) per tile: group 0 passes it before M(t), group 1 before V(t - 1); between two
        // barriers group 0 runs M(t) V(t) and group 1 runs V(t - 1) M(t) back to back, so the groups' matrix and
        // vector phases still pair up but neither waits for the other in the middle.  Everything tile t's matrix
        // phases read -- K(t), V(t - 1) -- has landed by B(t); the buffers refilled after B(t) were last read before it.
        // before B(t): group 0 has requested V up to min(t + 1, NT - 1) and needs V(t - 1) complete
        // (At head_dim 64, where the vector phase is by far the longer one, a barrier before every phase of both
        // groups is faster: PAIR_BARRIER is off and group 0 ends with one extra barrier.)
        auto enter_m = [&](int t) __attribute__((always_inline)) {
            if (grp == 0) wait_tiles_in_flight<DMA_PER_WAVE>(NT - t < 2 ? NT - t : 2, my_xfers);
            if (grp == 0 || !PAIR_BARRIER) wg_barrier();
        };
        // before V(t), i.e. B(t + 1): group 1 has requested K up to min(t + 3, NT - 1) and needs K(t + 1) complete;
        // then the vector phase itself, starting with this group's share of the fetches
        auto vector_part = [&](int t, auto first_c) __attribute__((always_inline)) {
            if (grp == 1 && t + 1 < NT) wait_tiles_in_flight<DMA_PER_WAVE>(NT - 2 - t < 2 ? NT - 2 - t : 2, my_xfers);
            if (grp == 1 || !PAIR_BARRIER) wg_barrier();
            const int j = t + (grp ? K_AHEAD : V_AHEAD);
            if (j < NT) fetch_tile(j);
            if (t >= n_full_g) v_phase(t & (2 * NB - 1), first_c, std::true_type{}, exact);
            else v_phase(t & (2 * NB - 1), first_c, std::false_type{}, exact);
        };
        enter_m(0);
        m_phase(IC<0>{}, IC<NPV>{}, IC<NST>{});
        vector_part(0, std::true_type{});
        // tiles 1 .. NT-1: four at a time in a straight line (buffer = t % 4 is then a compile-time constant and
        // no accumulator passes through a control-flow merge), then the remaining ones through a switch
        int t = 1;
        for (; t + 3 < NT; t += 4) {
            enter_m(t);     m_phase(IC<1>{}, IC<0>{}, IC<NST>{}); vector_part(t, std::false_type{});
            enter_m(t + 1); m_phase(IC<2>{}, IC<0>{}, IC<NST>{}); vector_part(t + 1, std::false_type{});
            enter_m(t + 2); m_phase(IC<3>{}, IC<0>{}, IC<NST>{}); vector_part(t + 2, std::false_type{});
            enter_m(t + 3); m_phase(IC<0>{}, IC<0>{}, IC<NST>{}); vector_part(t + 3, std::false_type{});
        }
        for (; t < NT; ++t) {
            enter_m(t);
            switch (t & 3) {
                case 0: m_phase(IC<0>{}, IC<0>{}, IC<NST>{}); break;
                case 1: m_phase(IC<1>{}, IC<0>{}, IC<NST>{}); break;
                case 2: m_phase(IC<2>{}, IC<0>{}, IC<NST>{}); break;
                default: m_phase(IC<3>{}, IC<0>{}, IC<NST>{}); break;
            }
            vector_part(t, std::false_type{});
        }
        enter_m(NT);
        switch (NT & 3) {
            case 0: m_phase(IC<0>{}, IC<0>{}, IC<NPV>{}); break;
            case 1: m_phase(IC<1>{}, IC<0>{}, IC<NPV>{}); break;
            case 2: m_phase(IC<2>{}, IC<0>{}, IC<NPV>{}); break;
            default: m_phase(IC<3>{}, IC<0>{}, IC<NPV>{}); break;
        }
        if (!PAIR_BARRIER && grp == 0) wg_barrier();
    };

    run(std::false_type{});
    float l_tot = sum_across_halves(l_run), lr_tot = sum_across_halves(lr_run);
    {
        // a row that sees any key of the chunk sees its first key
        const bool sees = my_row < g.lq && my_pos >= g.ks.start[0];
        const int bad = sees && !(l_tot >= SUM_LO && l_tot <= SUM_HI);
        if (__syncthreads_or(bad)) {   // a row left the safe range: repeat the tiles with the exact online softmax
            run(std::true_type{});
            l_tot = sum_across_halves(l_run);
            lr_tot = sum_across_halves(lr_run);
            // the last matrix phase of the other wavefronts may still be reading V tiles that the staging below
            // overwrites (after the fast pass the vote above is that barrier)
            __syncthreads();
        }
    }

    // Epilogue.  Every lane scales its row's O^T registers and merges the LSE; the scaled rows go through
    // LDS (free now; a private 32 x (D + 4)-float region per wavefront, padded against bank conflicts) so that
    // the global accesses are row-contiguous: one instruction covers 1 KB of whole rows of o (two at D = 128).
    float inv = 0.f, lse_new = -INFINITY;
    if (l_tot > 0.f) {
        inv = lr_tot > 0.f ? 1.0f / lr_tot : 0.f;
        lse_new = (m_run + __log2f(l_tot)) * LN2;
    }
    float wa = 0.f, wb = inv;
    float* lp = a.lse + (long long)h * g.lq + my_row_c;
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
    float* stage = reinterpret_cast<float*>(&sm) + wave * (32 * O_STAGE_STRIDE + 32);
    float* stage_wa = stage + 32 * O_STAGE_STRIDE;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int b = 0; b < 4; ++b)
            *reinterpret_cast<float4*>(&stage[l32 * O_STAGE_STRIDE + 32 * db + 8 * b + 4 * hh]) =
                make_float4(oacc[db][4 * b] * wb, oacc[db][4 * b + 1] * wb, oacc[db][4 * b + 2] * wb, oacc[db][4 * b + 3] * wb);
    if (hh == 0) {
        stage_wa[l32] = wa;
        if (my_row < g.lq) *lp = lse_new;   // both half-wave lanes of a row read *lp above, in the same instruction
    }
    // the region is private to the wavefront: its own LDS writes only need to have completed
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // lane -> (row within a group of ROWS_PER_INST rows, 16-byte piece of the row)
    constexpr int LANES_PER_ROW = D / 4, ROWS_PER_INST = 64 / LANES_PER_ROW, N_INST = 32 / ROWS_PER_INST;
    const int sub_row = lane / LANES_PER_ROW, piece = lane % LANES_PER_ROW;
    const int wrow0 = grow0 + 32 * wg;
    float* obase = a.o + ((long long)wrow0 * g.nq + h) * D + 4 * piece;
    const long long row_stride = (long long)g.nq * D;
    float4 val[N_INST];
    float4 old[N_INST];
#pragma unroll
    for (int i = 0; i < N_INST; ++i) {
        const int r = ROWS_PER_INST * i + sub_row;
        val[i] = *reinterpret_cast<const float4*>(&stage[r * O_STAGE_STRIDE + 4 * piece]);
        if (a.accumulate && wrow0 + r < g.lq) old[i] = *reinterpret_cast<const float4*>(obase + r * row_stride);
        else old[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int i = 0; i < N_INST; ++i) {
        const int r = ROWS_PER_INST * i + sub_row;
        const float w = stage_wa[r];
        float4 o4 = val[i];
        o4.x += w * old[i].x; o4.y += w * old[i].y; o4.z += w * old[i].z; o4.w += w * old[i].w;
        if (wrow0 + r < g.lq) *reinterpret_cast<float4*>(obase + r * row_stride) = o4;
    }
}

}  // namespace

hipError_t hexi_launch_fwd_bf16(const FwdArgs& a, hipStream_t s)
{
    const AttnGeom& g = a.g;
    const int n_q_tiles = (g.lq + WG_ROWS - 1) / WG_ROWS;
    // cost of a unit: the key tiles its q tile streams, plus the prologue and epilogue (about six tiles' worth);
    // a unit that sees nothing of the chunk returns at once under HEXI_ACCUMULATE and only writes zeros otherwise
    float cost[4096];
    const int n_known = n_q_tiles < 4096 ? n_q_tiles : 4096;     // (longer shards: the remaining tiles count like the last known one)
    for (int p = 0; p < n_known; ++p) {
        const int q_tile = n_q_tiles - 1 - p;
        const int last_row = (q_tile * WG_ROWS + WG_ROWS < g.lq ? q_tile * WG_ROWS + WG_ROWS : g.lq) - 1;
        const int nt = (seg_rows_le(g.ks, seg_pos_of_row(g.qs, last_row)) + TN - 1) / TN;
        cost[p] = nt > 0 ? (float)nt + 6.0f : (a.accumulate ? 0.25f : 2.0f);
    }
    unsigned grid = 0;
    const XcdSplit split = hexi_split_units(g.nq * n_q_tiles, [&](int u) { const int p = u % n_q_tiles; return cost[p < n_known ? p : n_known - 1]; }, &grid);
    if (grid == 0) return hipSuccess;
    if (g.d == 128) fwd_bf16_kernel<128><<<grid, 512, 0, s>>>(a, n_q_tiles, split);
    else if (g.d == 64) fwd_bf16_kernel<64><<<grid, 512, 0, s>>>(a, n_q_tiles, split);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}
