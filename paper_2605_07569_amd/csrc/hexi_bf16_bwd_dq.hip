// bf16 backward ring step, dQ part, for gfx950 (head_dim D = 128 or 64): one workgroup of 8 wavefronts per
// (256-row q tile, q head), one workgroup per CU; the q tile's dQ stays in accumulators while the chunk's keys stream past, so dQ needs
// no atomics and its summation order is fixed.
//
// Everything is computed transposed, as in the forward kernel, so that every lane owns one query row and the
// row constants (saved global LSE, Delta) are per-lane scalars:
//   S^T = K Q^T,  dP^T = V dO^T  (K, V rows read from LDS with 128-bit reads; Q^T, dO^T in registers),
//   P^T = exp2(S^T * scale*log2e - LSE*log2e),  dS^T = P^T (dP^T - Delta),
//   dQ^T += K^T dS^T  (K^T through transposed LDS reads; dS^T straight from the accumulator registers).
//
// Ping-pong schedule (see the forward kernel): two groups of four wavefronts, wavefront w and w + 4 on one
// SIMD, alternate between a matrix phase and a vector phase, group 1 one phase behind group 0, so that a SIMD
// mostly has one wavefront issuing only MFMAs (and their LDS reads) and one issuing only VALU work.  One
// workgroup barrier per pair of phases keeps the groups in step (group 0 passes it before a matrix phase,
// group 1 before a vector phase).  A phase covers a 32-key block (half a 64-key LDS tile), which keeps the
// scores and dP of one block only in registers:
//   M(b): dQ^T += K^T dS^T of block b-1 (D / 16 MFMAs), then S^T and dP^T of block b (D / 8 MFMAs);
//   V(b): P^T and dS^T of block b, dS^T rounded to bf16 operand slots.
// The vector-phase group also issues the direct global->LDS loads: during the first block of tile j, group 1
// requests K of tile j + 3 and group 0 requests V of tile j + 3 (four LDS buffers per tensor).
#include "hexi_internal.h"
#include "hexi_mfma.h"

namespace {

constexpr int TN = 64;             // keys per LDS tile (two 32-key blocks)
constexpr int NB = 4;              // LDS buffers per tensor
constexpr int GROUP_ROWS = 128;    // q rows per wavefront group (32 per wavefront)
constexpr int WG_ROWS = 256;       // q rows per workgroup
constexpr int AHEAD = 3;           // tile j + 3 is requested during tile j
constexpr float LOG2E = 1.4426950408889634f;

// A 32-key block in which some |bf16(dS)| reaches this value also accumulates the residuals dS - bf16(dS) of the rounding:
// rounding dS to bf16 costs up to 2^-9 |dS| scale |k| per element of dQ, which for the few keys that dominate a
// sharply peaked row (|dS| of several units) is most of the output tolerance.
constexpr float DS_SPLIT = 2.0f;

// dQ^T += K^T (dS^T - bf16(dS^T)) for one 32-key block, executed only when `any_large` (a wave-uniform lane mask) is
// non-zero: a few blocks in a thousand even on sharply peaked rows, so the path is written for simplicity, with fp32
// MFMAs (v_mfma_f32_32x32x2_f32: every operand is one register per lane; accumulator register x of a lane pairs its
// two half-waves' keys).  ds[0..15]: the lane's dS^T values in fp32; hw[0..7]: their bf16 roundings, two per dword;
// ka: the lane's LDS byte address of K[first key of the block + (lane / 32)][2 * (lane % 32)] in the tile's padded,
// row-permuted image (row pitch ROW): accumulator register x = 4b + t holds key 8b + 4 (lane / 32) + t, stored in
// LDS row 16 (b / 2) + 4 t + 2 (b % 2) + (lane / 32) of the block.  The branch lives inside the assembly statement so
// that the compiler sees straight-line code (a visible branch around MFMAs makes it copy the accumulators at the merge).
template <int NDB, int ROW>
__device__ __forceinline__ void dq_add_residuals(f32x16 (&dq)[NDB], const float (&ds)[16], const uint32_t (&hw)[8], uint32_t ka,
                                                 unsigned long long any_large)
{
    static_assert(NDB == 4 || NDB == 2, "two or four 32-column blocks");
    float t_k, t_r;
    if constexpr (NDB == 4) {
        asm volatile(
            "s_cmp_eq_u64 %[f], 0\n\ts_cbranch_scc1 .Lhexi_skip%=\n\ts_nop 15\n\ts_nop 15\n\t"
            "v_lshlrev_b32 %[r], 16, %[h0]\n\t"
            "v_sub_f32 %[r], %[d0], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o0_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o0_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o0_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o0_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h0]\n\t"
            "v_sub_f32 %[r], %[d1], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o1_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o1_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o1_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o1_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h1]\n\t"
            "v_sub_f32 %[r], %[d2], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o2_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o2_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o2_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o2_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h1]\n\t"
            "v_sub_f32 %[r], %[d3], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o3_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o3_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o3_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o3_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h2]\n\t"
            "v_sub_f32 %[r], %[d4], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o4_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o4_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o4_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o4_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h2]\n\t"
            "v_sub_f32 %[r], %[d5], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o5_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o5_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o5_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o5_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h3]\n\t"
            "v_sub_f32 %[r], %[d6], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o6_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o6_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o6_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o6_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h3]\n\t"
            "v_sub_f32 %[r], %[d7], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o7_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o7_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o7_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o7_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h4]\n\t"
            "v_sub_f32 %[r], %[d8], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o8_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o8_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o8_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o8_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h4]\n\t"
            "v_sub_f32 %[r], %[d9], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o9_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o9_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o9_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o9_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h5]\n\t"
            "v_sub_f32 %[r], %[d10], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o10_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o10_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o10_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o10_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h5]\n\t"
            "v_sub_f32 %[r], %[d11], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o11_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o11_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o11_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o11_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h6]\n\t"
            "v_sub_f32 %[r], %[d12], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o12_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o12_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o12_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o12_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h6]\n\t"
            "v_sub_f32 %[r], %[d13], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o13_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o13_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o13_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o13_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h7]\n\t"
            "v_sub_f32 %[r], %[d14], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o14_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o14_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o14_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o14_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h7]\n\t"
            "v_sub_f32 %[r], %[d15], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o15_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o15_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o15_2]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a2], %[t], %[r], %[a2]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o15_3]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a3], %[t], %[r], %[a3]\n\t"
            "s_nop 15\n\ts_nop 15\n\t"
            ".Lhexi_skip%=:"
            : [a0] "+v"(dq[0]), [a1] "+v"(dq[1]), [a2] "+v"(dq[2]), [a3] "+v"(dq[3]), [t] "=&v"(t_k), [r] "=&v"(t_r)
            : [f] "s"(any_large), [ka] "v"(ka), [h0] "v"(hw[0]), [h1] "v"(hw[1]), [h2] "v"(hw[2]), [h3] "v"(hw[3]), [h4] "v"(hw[4]), [h5] "v"(hw[5]), [h6] "v"(hw[6]), [h7] "v"(hw[7]),
              [d0] "v"(ds[0]), [d1] "v"(ds[1]), [d2] "v"(ds[2]), [d3] "v"(ds[3]), [d4] "v"(ds[4]), [d5] "v"(ds[5]), [d6] "v"(ds[6]), [d7] "v"(ds[7]), [d8] "v"(ds[8]), [d9] "v"(ds[9]), [d10] "v"(ds[10]), [d11] "v"(ds[11]), [d12] "v"(ds[12]), [d13] "v"(ds[13]), [d14] "v"(ds[14]), [d15] "v"(ds[15]),
              [o0_0] "n"((16 * (0 >> 1) + 4 * 0 + 2 * (0 & 1)) * ROW + 64 * 0), [o0_1] "n"((16 * (0 >> 1) + 4 * 0 + 2 * (0 & 1)) * ROW + 64 * 1), [o0_2] "n"((16 * (0 >> 1) + 4 * 0 + 2 * (0 & 1)) * ROW + 64 * 2), [o0_3] "n"((16 * (0 >> 1) + 4 * 0 + 2 * (0 & 1)) * ROW + 64 * 3), [o1_0] "n"((16 * (0 >> 1) + 4 * 1 + 2 * (0 & 1)) * ROW + 64 * 0), [o1_1] "n"((16 * (0 >> 1) + 4 * 1 + 2 * (0 & 1)) * ROW + 64 * 1), [o1_2] "n"((16 * (0 >> 1) + 4 * 1 + 2 * (0 & 1)) * ROW + 64 * 2), [o1_3] "n"((16 * (0 >> 1) + 4 * 1 + 2 * (0 & 1)) * ROW + 64 * 3), [o2_0] "n"((16 * (0 >> 1) + 4 * 2 + 2 * (0 & 1)) * ROW + 64 * 0), [o2_1] "n"((16 * (0 >> 1) + 4 * 2 + 2 * (0 & 1)) * ROW + 64 * 1), [o2_2] "n"((16 * (0 >> 1) + 4 * 2 + 2 * (0 & 1)) * ROW + 64 * 2), [o2_3] "n"((16 * (0 >> 1) + 4 * 2 + 2 * (0 & 1)) * ROW + 64 * 3), [o3_0] "n"((16 * (0 >> 1) + 4 * 3 + 2 * (0 & 1)) * ROW + 64 * 0), [o3_1] "n"((16 * (0 >> 1) + 4 * 3 + 2 * (0 & 1)) * ROW + 64 * 1), [o3_2] "n"((16 * (0 >> 1) + 4 * 3 + 2 * (0 & 1)) * ROW + 64 * 2), [o3_3] "n"((16 * (0 >> 1) + 4 * 3 + 2 * (0 & 1)) * ROW + 64 * 3), [o4_0] "n"((16 * (1 >> 1) + 4 * 0 + 2 * (1 & 1)) * ROW + 64 * 0), [o4_1] "n"((16 * (1 >> 1) + 4 * 0 + 2 * (1 & 1)) * ROW + 64 * 1), [o4_2] "n"((16 * (1 >> 1) + 4 * 0 + 2 * (1 & 1)) * ROW + 64 * 2), [o4_3] "n"((16 * (1 >> 1) + 4 * 0 + 2 * (1 & 1)) * ROW + 64 * 3), [o5_0] "n"((16 * (1 >> 1) + 4 * 1 + 2 * (1 & 1)) * ROW + 64 * 0), [o5_1] "n"((16 * (1 >> 1) + 4 * 1 + 2 * (1 & 1)) * ROW + 64 * 1), [o5_2] "n"((16 * (1 >> 1) + 4 * 1 + 2 * (1 & 1)) * ROW + 64 * 2), [o5_3] "n"((16 * (1 >> 1) + 4 * 1 + 2 * (1 & 1)) * ROW + 64 * 3), [o6_0] "n"((16 * (1 >> 1) + 4 * 2 + 2 * (1 & 1)) * ROW + 64 * 0), [o6_1] "n"((16 * (1 >> 1) + 4 * 2 + 2 * (1 & 1)) * ROW + 64 * 1), [o6_2] "n"((16 * (1 >> 1) + 4 * 2 + 2 * (1 & 1)) * ROW + 64 * 2), [o6_3] "n"((16 * (1 >> 1) + 4 * 2 + 2 * (1 & 1)) * ROW + 64 * 3), [o7_0] "n"((16 * (1 >> 1) + 4 * 3 + 2 * (1 & 1)) * ROW + 64 * 0), [o7_1] "n"((16 * (1 >> 1) + 4 * 3 + 2 * (1 & 1)) * ROW + 64 * 1), [o7_2] "n"((16 * (1 >> 1) + 4 * 3 + 2 * (1 & 1)) * ROW + 64 * 2), [o7_3] "n"((16 * (1 >> 1) + 4 * 3 + 2 * (1 & 1)) * ROW + 64 * 3), [o8_0] "n"((16 * (2 >> 1) + 4 * 0 + 2 * (2 & 1)) * ROW + 64 * 0), [o8_1] "n"((16 * (2 >> 1) + 4 * 0 + 2 * (2 & 1)) * ROW + 64 * 1), [o8_2] "n"((16 * (2 >> 1) + 4 * 0 + 2 * (2 & 1)) * ROW + 64 * 2), [o8_3] "n"((16 * (2 >> 1) + 4 * 0 + 2 * (2 & 1)) * ROW + 64 * 3), [o9_0] "n"((16 * (2 >> 1) + 4 * 1 + 2 * (2 & 1)) * ROW + 64 * 0), [o9_1] "n"((16 * (2 >> 1) + 4 * 1 + 2 * (2 & 1)) * ROW + 64 * 1), [o9_2] "n"((16 * (2 >> 1) + 4 * 1 + 2 * (2 & 1)) * ROW + 64 * 2), [o9_3] "n"((16 * (2 >> 1) + 4 * 1 + 2 * (2 & 1)) * ROW + 64 * 3), [o10_0] "n"((16 * (2 >> 1) + 4 * 2 + 2 * (2 & 1)) * ROW + 64 * 0), [o10_1] "n"((16 * (2 >> 1) + 4 * 2 + 2 * (2 & 1)) * ROW + 64 * 1), [o10_2] "n"((16 * (2 >> 1) + 4 * 2 + 2 * (2 & 1)) * ROW + 64 * 2), [o10_3] "n"((16 * (2 >> 1) + 4 * 2 + 2 * (2 & 1)) * ROW + 64 * 3), [o11_0] "n"((16 * (2 >> 1) + 4 * 3 + 2 * (2 & 1)) * ROW + 64 * 0), [o11_1] "n"((16 * (2 >> 1) + 4 * 3 + 2 * (2 & 1)) * ROW + 64 * 1), [o11_2] "n"((16 * (2 >> 1) + 4 * 3 + 2 * (2 & 1)) * ROW + 64 * 2), [o11_3] "n"((16 * (2 >> 1) + 4 * 3 + 2 * (2 & 1)) * ROW + 64 * 3), [o12_0] "n"((16 * (3 >> 1) + 4 * 0 + 2 * (3 & 1)) * ROW + 64 * 0), [o12_1] "n"((16 * (3 >> 1) + 4 * 0 + 2 * (3 & 1)) * ROW + 64 * 1), [o12_2] "n"((16 * (3 >> 1) + 4 * 0 + 2 * (3 & 1)) * ROW + 64 * 2), [o12_3] "n"((16 * (3 >> 1) + 4 * 0 + 2 * (3 & 1)) * ROW + 64 * 3), [o13_0] "n"((16 * (3 >> 1) + 4 * 1 + 2 * (3 & 1)) * ROW + 64 * 0), [o13_1] "n"((16 * (3 >> 1) + 4 * 1 + 2 * (3 & 1)) * ROW + 64 * 1), [o13_2] "n"((16 * (3 >> 1) + 4 * 1 + 2 * (3 & 1)) * ROW + 64 * 2), [o13_3] "n"((16 * (3 >> 1) + 4 * 1 + 2 * (3 & 1)) * ROW + 64 * 3), [o14_0] "n"((16 * (3 >> 1) + 4 * 2 + 2 * (3 & 1)) * ROW + 64 * 0), [o14_1] "n"((16 * (3 >> 1) + 4 * 2 + 2 * (3 & 1)) * ROW + 64 * 1), [o14_2] "n"((16 * (3 >> 1) + 4 * 2 + 2 * (3 & 1)) * ROW + 64 * 2), [o14_3] "n"((16 * (3 >> 1) + 4 * 2 + 2 * (3 & 1)) * ROW + 64 * 3), [o15_0] "n"((16 * (3 >> 1) + 4 * 3 + 2 * (3 & 1)) * ROW + 64 * 0), [o15_1] "n"((16 * (3 >> 1) + 4 * 3 + 2 * (3 & 1)) * ROW + 64 * 1), [o15_2] "n"((16 * (3 >> 1) + 4 * 3 + 2 * (3 & 1)) * ROW + 64 * 2), [o15_3] "n"((16 * (3 >> 1) + 4 * 3 + 2 * (3 & 1)) * ROW + 64 * 3)
            : "scc", "memory");
    } else {
        asm volatile(
            "s_cmp_eq_u64 %[f], 0\n\ts_cbranch_scc1 .Lhexi_skip%=\n\ts_nop 15\n\ts_nop 15\n\t"
            "v_lshlrev_b32 %[r], 16, %[h0]\n\t"
            "v_sub_f32 %[r], %[d0], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o0_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o0_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h0]\n\t"
            "v_sub_f32 %[r], %[d1], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o1_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o1_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h1]\n\t"
            "v_sub_f32 %[r], %[d2], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o2_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o2_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h1]\n\t"
            "v_sub_f32 %[r], %[d3], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o3_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o3_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h2]\n\t"
            "v_sub_f32 %[r], %[d4], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o4_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o4_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h2]\n\t"
            "v_sub_f32 %[r], %[d5], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o5_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o5_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h3]\n\t"
            "v_sub_f32 %[r], %[d6], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o6_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o6_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h3]\n\t"
            "v_sub_f32 %[r], %[d7], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o7_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o7_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h4]\n\t"
            "v_sub_f32 %[r], %[d8], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o8_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o8_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h4]\n\t"
            "v_sub_f32 %[r], %[d9], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o9_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o9_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h5]\n\t"
            "v_sub_f32 %[r], %[d10], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o10_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o10_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h5]\n\t"
            "v_sub_f32 %[r], %[d11], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o11_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o11_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h6]\n\t"
            "v_sub_f32 %[r], %[d12], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o12_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o12_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h6]\n\t"
            "v_sub_f32 %[r], %[d13], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o13_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o13_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_lshlrev_b32 %[r], 16, %[h7]\n\t"
            "v_sub_f32 %[r], %[d14], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o14_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o14_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "v_and_b32 %[r], 0xffff0000, %[h7]\n\t"
            "v_sub_f32 %[r], %[d15], %[r]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o15_0]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a0], %[t], %[r], %[a0]\n\t"
            "ds_read_u16 %[t], %[ka] offset:%c[o15_1]\n\ts_waitcnt lgkmcnt(0)\n\tv_lshlrev_b32 %[t], 16, %[t]\n\ts_nop 1\n\t"
            "v_mfma_f32_32x32x2_f32 %[a1], %[t], %[r], %[a1]\n\t"
            "s_nop 15\n\ts_nop 15\n\t"
            ".Lhexi_skip%=:"
            : [a0] "+v"(dq[0]), [a1] "+v"(dq[1]), [t] "=&v"(t_k), [r] "=&v"(t_r)
            : [f] "s"(any_large), [ka] "v"(ka), [h0] "v"(hw[0]), [h1] "v"(hw[1]), [h2] "v"(hw[2]), [h3] "v"(hw[3]), [h4] "v"(hw[4]), [h5] "v"(hw[5]), [h6] "v"(hw[6]), [h7] "v"(hw[7]),
              [d0] "v"(ds[0]), [d1] "v"(ds[1]), [d2] "v"(ds[2]), [d3] "v"(ds[3]), [d4] "v"(ds[4]), [d5] "v"(ds[5]), [d6] "v"(ds[6]), [d7] "v"(ds[7]), [d8] "v"(ds[8]), [d9] "v"(ds[9]), [d10] "v"(ds[10]), [d11] "v"(ds[11]), [d12] "v"(ds[12]), [d13] "v"(ds[13]), [d14] "v"(ds[14]), [d15] "v"(ds[15]),
              [o0_0] "n"((16 * (0 >> 1) + 4 * 0 + 2 * (0 & 1)) * ROW + 64 * 0), [o0_1] "n"((16 * (0 >> 1) + 4 * 0 + 2 * (0 & 1)) * ROW + 64 * 1), [o1_0] "n"((16 * (0 >> 1) + 4 * 1 + 2 * (0 & 1)) * ROW + 64 * 0), [o1_1] "n"((16 * (0 >> 1) + 4 * 1 + 2 * (0 & 1)) * ROW + 64 * 1), [o2_0] "n"((16 * (0 >> 1) + 4 * 2 + 2 * (0 & 1)) * ROW + 64 * 0), [o2_1] "n"((16 * (0 >> 1) + 4 * 2 + 2 * (0 & 1)) * ROW + 64 * 1), [o3_0] "n"((16 * (0 >> 1) + 4 * 3 + 2 * (0 & 1)) * ROW + 64 * 0), [o3_1] "n"((16 * (0 >> 1) + 4 * 3 + 2 * (0 & 1)) * ROW + 64 * 1), [o4_0] "n"((16 * (1 >> 1) + 4 * 0 + 2 * (1 & 1)) * ROW + 64 * 0), [o4_1] "n"((16 * (1 >> 1) + 4 * 0 + 2 * (1 & 1)) * ROW + 64 * 1), [o5_0] "n"((16 * (1 >> 1) + 4 * 1 + 2 * (1 & 1)) * ROW + 64 * 0), [o5_1] "n"((16 * (1 >> 1) + 4 * 1 + 2 * (1 & 1)) * ROW + 64 * 1), [o6_0] "n"((16 * (1 >> 1) + 4 * 2 + 2 * (1 & 1)) * ROW + 64 * 0), [o6_1] "n"((16 * (1 >> 1) + 4 * 2 + 2 * (1 & 1)) * ROW + 64 * 1), [o7_0] "n"((16 * (1 >> 1) + 4 * 3 + 2 * (1 & 1)) * ROW + 64 * 0), [o7_1] "n"((16 * (1 >> 1) + 4 * 3 + 2 * (1 & 1)) * ROW + 64 * 1), [o8_0] "n"((16 * (2 >> 1) + 4 * 0 + 2 * (2 & 1)) * ROW + 64 * 0), [o8_1] "n"((16 * (2 >> 1) + 4 * 0 + 2 * (2 & 1)) * ROW + 64 * 1), [o9_0] "n"((16 * (2 >> 1) + 4 * 1 + 2 * (2 & 1)) * ROW + 64 * 0), [o9_1] "n"((16 * (2 >> 1) + 4 * 1 + 2 * (2 & 1)) * ROW + 64 * 1), [o10_0] "n"((16 * (2 >> 1) + 4 * 2 + 2 * (2 & 1)) * ROW + 64 * 0), [o10_1] "n"((16 * (2 >> 1) + 4 * 2 + 2 * (2 & 1)) * ROW + 64 * 1), [o11_0] "n"((16 * (2 >> 1) + 4 * 3 + 2 * (2 & 1)) * ROW + 64 * 0), [o11_1] "n"((16 * (2 >> 1) + 4 * 3 + 2 * (2 & 1)) * ROW + 64 * 1), [o12_0] "n"((16 * (3 >> 1) + 4 * 0 + 2 * (3 & 1)) * ROW + 64 * 0), [o12_1] "n"((16 * (3 >> 1) + 4 * 0 + 2 * (3 & 1)) * ROW + 64 * 1), [o13_0] "n"((16 * (3 >> 1) + 4 * 1 + 2 * (3 & 1)) * ROW + 64 * 0), [o13_1] "n"((16 * (3 >> 1) + 4 * 1 + 2 * (3 & 1)) * ROW + 64 * 1), [o14_0] "n"((16 * (3 >> 1) + 4 * 2 + 2 * (3 & 1)) * ROW + 64 * 0), [o14_1] "n"((16 * (3 >> 1) + 4 * 2 + 2 * (3 & 1)) * ROW + 64 * 1), [o15_0] "n"((16 * (3 >> 1) + 4 * 3 + 2 * (3 & 1)) * ROW + 64 * 0), [o15_1] "n"((16 * (3 >> 1) + 4 * 3 + 2 * (3 & 1)) * ROW + 64 * 1)
            : "scc", "memory");
    }
}

template <int D> struct DqSmem {
    unsigned char k[NB][p16_tile_bytes(D)];   // 4 x 17 KB (D = 128) or 4 x 9 KB
    unsigned char v[NB][p16_tile_bytes(D)];
    int kpos[2 * NB][TN];     // key positions of the tiles that need a mask, written AHEAD tiles ahead
    // the epilogue stages 8 x (32 x (D + 4)) floats over the start of this struct
};

template <int D>
__global__ void __launch_bounds__(512) bwd_dq_bf16_kernel(const BwdArgs a, const int n_q_tiles, const XcdSplit split)
{
    static_assert(D == 64 || D == 128, "head_dim 64 or 128");
    constexpr int NKS = D / 16;     // 16-wide contraction steps across the head dimension
    constexpr int NDB = D / 32;     // 32-column blocks of dQ
    constexpr int P16_ROW_BYTES = p16_row_bytes(D), P16_TILE_BYTES = p16_tile_bytes(D);
    constexpr int N_XFER = P16_TILE_BYTES / 1024;          // wave-wide transfers per tile: 17 or 9
    constexpr int DMA_PER_WAVE = (N_XFER + 3) / 4;         // most transfers a wavefront issues per tile: 5 or 3
    constexpr int STAGE_STRIDE = D + 4;                    // floats per staged output row (epilogue)
    // one workgroup barrier per pair of phases instead of one per phase (at head_dim 64, where the vector phase is by
    // far the longer one, a barrier before every phase of both groups is faster; group 0 then ends with one extra)
    constexpr bool PAIR_BARRIER = D == 128;
    static_assert(sizeof(DqSmem<D>) >= 8 * 32 * STAGE_STRIDE * 4, "epilogue staging does not fit");
    const AttnGeom& g = a.g;
    __shared__ __attribute__((aligned(1024))) DqSmem<D> sm;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2, wg = wave & 3;
    const int l32 = lane & 31, hh = lane >> 5;
    const int grp2 = (lane >> 4) & 1, j16 = lane & 15;

    // (head, q tile) units, head-major, longest q tiles of a head first; each XCD takes a contiguous unit range of
    // about equal work
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

    const uint16_t* k = static_cast<const uint16_t*>(a.k) + (long long)kvh * g.kv_stride_head;
    const uint16_t* v = static_cast<const uint16_t*>(a.v) + (long long)kvh * g.kv_stride_head;

    // n_full_g: tiles this group needs no mask for; NT: tiles the workgroup streams (those visible to its last
    // rows; a group whose rows see fewer masks the rest away); n_full_wg: tiles no row needs a mask for.
    int n_full_g = 0;
    if (grow0 < g.lq) n_full_g = seg_rows_le(g.ks, seg_pos_of_row(g.qs, grow0)) / TN;
    const int wg_last_row = (row0 + WG_ROWS < g.lq ? row0 + WG_ROWS : g.lq) - 1;
    const int NT = (seg_rows_le(g.ks, seg_pos_of_row(g.qs, wg_last_row)) + TN - 1) / TN;
    const int n_full_wg = seg_rows_le(g.ks, seg_pos_of_row(g.qs, row0)) / TN;
    if (NT == 0) return;     // this q tile sees nothing of the chunk: dq_acc unchanged

    // Q^T and dO^T operand fragments: lane (row l32, half hh) holds d = 16*ks + 8*hh .. +7
    bf16x8 qf[NKS], gf[NKS];
    float neg_lse2, delta;
    {
        const long long off = (long long)my_row_c * g.q_stride_tok + (long long)h * g.q_stride_head + 8 * hh;
        const uint16_t* qp = static_cast<const uint16_t*>(a.q) + off;
        const uint16_t* gp = static_cast<const uint16_t*>(a.d_o) + off;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            qf[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
            gf[ks] = *reinterpret_cast<const bf16x8*>(gp + 16 * ks);
        }
        const float l = a.lse[(long long)h * g.lq + my_row_c];
        // rows that see nothing anywhere (LSE = -inf) and padding rows: P = 0 through LSE = +inf
        neg_lse2 = (my_row < g.lq && l != -INFINITY) ? -l * LOG2E : -INFINITY;
        delta = a.delta[(long long)h * g.lq + my_row_c];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) { pin(qf[ks]); pin(gf[ks]); }
        asm volatile("" ::"v"(neg_lse2), "v"(delta));
    }

    // Direct global->LDS fetch of one tile by the four wavefronts of a group (group 1: K, group 0: V).  A
    // transfer is one wave-wide instruction: lane L writes the 16 bytes at (transfer * 1024 + 16 * L) of the
    // tile's LDS image and reads the 16-byte piece of the key row that belongs there (the pad piece re-reads
    // piece 0).  Wavefront wg issues the transfers wg, wg + 4, ... below the tile's transfer count
    // (DMA_PER_WAVE of them, or one fewer).
    const int my_xfers = (N_XFER - wg + 3) / 4;     // transfers this wavefront issues per tile: wg, wg + 4, ...
    uint32_t fetch_off[DMA_PER_WAVE];   // byte offsets from the tile's first key
    int fetch_row[DMA_PER_WAVE];
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; ++i) {
        const int pos = (wg + 4 * i) * 1024 + 16 * lane;
        int r = pos / P16_ROW_BYTES, c = (pos - r * P16_ROW_BYTES) >> 4;
        r = p16_row(r);     // the permutation is its own inverse: LDS row -> key
        if (wg + 4 * i >= N_XFER) r = 0;
        if (c >= D / 8) c = 0;
        fetch_row[i] = r;
        fetch_off[i] = 2u * (uint32_t)(r * (int)g.kv_stride_tok + c * 8);
    }
    const uint32_t lds_k = (uint32_t)(uintptr_t)(&sm.k[0][0]), lds_v = (uint32_t)(uintptr_t)(&sm.v[0][0]);
    const uint16_t* fetch_src = grp ? k : v;
    const uint32_t fetch_lds = grp ? lds_k : lds_v;
    auto fetch_tile = [&](int tile) {
        const int col0 = tile * TN;
        const uint32_t dst = __builtin_amdgcn_readfirstlane(fetch_lds + (tile & (NB - 1)) * P16_TILE_BYTES + wg * 1024);
        const uint16_t* src = fetch_src + (long long)col0 * g.kv_stride_tok;
        if (col0 + TN <= g.lc) {
#pragma unroll
            for (int i = 0; i < DMA_PER_WAVE; ++i) {
                if (wg + 4 * i < N_XFER) lds_dma16_base(src, fetch_off[i], __builtin_amdgcn_readfirstlane(dst + i * 4096));
            }
        } else {   // ragged last tile: clamp the key index (the extra keys are masked through their position)
#pragma unroll
            for (int i = 0; i < DMA_PER_WAVE; ++i) {
                uint32_t off = fetch_off[i];
                if (col0 + fetch_row[i] >= g.lc) off -= 2u * (uint32_t)((col0 + fetch_row[i] - (g.lc - 1)) * (int)g.kv_stride_tok);
                if (wg + 4 * i < N_XFER) lds_dma16_base(src, off, __builtin_amdgcn_readfirstlane(dst + i * 4096));
            }
        }
        // global positions of the tile's keys, for the tiles some row needs a mask for
        if (grp == 1 && wg == 0 && tile >= n_full_wg) {
            sm.kpos[tile & (2 * NB - 1)][lane] = col0 + lane < g.lc ? seg_pos_of_row(g.ks, col0 + lane) : 0x7fffffff;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    };

    // Lane parts of the LDS byte addresses; buffer, block and step are compile-time offsets of the reads.
    //   row fragment (block b, ks) of buffer B:  nat_addr + B * TILE + 32 * b * ROW + 32 * ks     (K and V alike)
    //   K^T fragment (16-key step u of the tile, 32-column block db, half `second`) of buffer B: keys
    //   16u + 8*second + 4*hh + jj sit in LDS rows 16u + 4*jj + 2*second + hh:
    //        ktr_addr[B / 2] + (B % 2) * TILE + (16 * u + 2 * second) * ROW + 64 * db
    // (two base registers: the offset field of an LDS read holds 16 bits).
    const int jj = j16 >> 2;
    const uint32_t nat_lane = p16_row(l32) * P16_ROW_BYTES + 16 * hh;
    const uint32_t knat_addr = lds_k + nat_lane, vnat_addr = lds_v + nat_lane;
    uint32_t ktr_addr[2];
    ktr_addr[0] = lds_k + (4 * jj + hh) * P16_ROW_BYTES + 2 * (16 * grp2 + 4 * (j16 & 3));
    ktr_addr[1] = ktr_addr[0] + 2 * P16_TILE_BYTES;
    const uint32_t kres_addr = lds_k + hh * P16_ROW_BYTES + 2 * l32;     // single K elements, for the residual path

    f32x16 dq[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[db][r] = 0.f;
    f32x16 s, dp;
    bf16x8 dsf[2];
    const float c_log2 = g.scale * LOG2E;

    // Matrix phase of block (tile buffer B, half HALF).  Steps 0..NDQ-1: dQ^T += K^T dS^T of the previous block
    // (two 16-key steps x NDB 32-column blocks; the previous block is the other half of the same tile, or
    // the second half of the tile before).  Steps NDQ..NST-1: S^T and dP^T of this block, alternating.
    // [FIRST, LAST) selects the steps; operand fragments are requested PF steps ahead.
    constexpr int NDQ = 2 * NDB, NST = NDQ + 2 * NKS;
    auto m_phase = [&](auto bc, auto half_c, auto first_c, auto last_c) __attribute__((always_inline)) {
        constexpr int B = decltype(bc)::value, HALF = decltype(half_c)::value;
        constexpr int FIRST = decltype(first_c)::value, LAST = decltype(last_c)::value;
        constexpr int PF = 4, NS = PF + 1;   // a fragment's registers are busy from its request until its MFMA
        constexpr int BP = HALF ? B : (B + NB - 1) % NB;     // buffer of the previous block
        constexpr int UP = HALF ? 0 : 2;                      // its first 16-key step within that tile
        s16x4 ta[NS], tb[NS];
        bf16x8 nb[NS];
        auto issue = [&](auto stc) __attribute__((always_inline)) {
            constexpr int st = decltype(stc)::value, slot = (st - FIRST) % NS;
            if constexpr (st < NDQ) {
                constexpr int u = UP + st / NDB, db = st % NDB;
                constexpr int off = (BP % 2) * P16_TILE_BYTES + 16 * u * P16_ROW_BYTES + 64 * db;
                lds_issue_tr16<off>(ta[slot], ktr_addr[BP / 2]);
                lds_issue_tr16<off + 2 * P16_ROW_BYTES>(tb[slot], ktr_addr[BP / 2]);
            } else {
                constexpr int ks = (st - NDQ) >> 1;
                constexpr int off = B * P16_TILE_BYTES + 32 * HALF * P16_ROW_BYTES + 32 * ks;
                if constexpr (((st - NDQ) & 1) == 0) lds_issue_b128<off>(nb[slot], knat_addr);
                else lds_issue_b128<off>(nb[slot], vnat_addr);
            }
        };
        auto step = [&](auto stc) __attribute__((always_inline)) {
            constexpr int st = decltype(stc)::value, slot = (st - FIRST) % NS;
            if constexpr (st + PF < LAST) issue(IC<st + PF>{});
            // LDS reads younger than this step's fragment: those of the next PF steps that exist
            constexpr int hi = st + PF < LAST ? st + PF : LAST - 1;
            constexpr int n_tr = (hi < NDQ ? hi : NDQ - 1) - (st < NDQ ? st : NDQ - 1);      // steps in (st, hi] below NDQ
            constexpr int younger = 2 * n_tr + ((hi - st) - n_tr);
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if constexpr (st < NDQ) {
                lds_wait<younger>(ta[slot], tb[slot]);
                dq[st % NDB] = mfma32(join_halves(ta[slot], tb[slot]), dsf[st / NDB], dq[st % NDB]);
            } else {
                constexpr int ks = (st - NDQ) >> 1;
                lds_wait<younger>(nb[slot]);
                if constexpr (((st - NDQ) & 1) == 0) s = mfma32(nb[slot], qf[ks], ks == 0 ? zero : s);
                else dp = mfma32(nb[slot], gf[ks], ks == 0 ? zero : dp);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        __builtin_amdgcn_sched_barrier(0);
        for_range<FIRST, (FIRST + PF < LAST ? FIRST + PF : LAST)>(issue);
        for_range<FIRST, LAST>(step);
    };

    // Vector phase of a block: P^T = exp2(S^T c - LSE log2e), dS^T = P^T (dP^T - Delta), rounded to bf16
    // operand slots.  MASKED: the tile needs the causal mask (key positions from LDS).
    // The lane's dS^T values of the block in fp32, kept for the residual path.
    float ds[16];
    auto v_phase = [&](int kpos_slot, int half, auto masked_c) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_c)::value;
#pragma unroll
        for (int x = 0; x < 16; ++x) {
            const float p = fast_exp2(fmaf(s[x], c_log2, neg_lse2));
            ds[x] = p * (dp[x] - delta);
        }
        if (MASKED) {
            const int* kp = &sm.kpos[kpos_slot][32 * half];
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const int4 p4 = *reinterpret_cast<const int4*>(&kp[8 * rb + 4 * hh]);
                if (p4.x > my_pos) ds[4 * rb] = 0.f;
                if (p4.y > my_pos) ds[4 * rb + 1] = 0.f;
                if (p4.z > my_pos) ds[4 * rb + 2] = 0.f;
                if (p4.w > my_pos) ds[4 * rb + 3] = 0.f;
            }
        }
        dsf[0] = pack_bf16x8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
        dsf[1] = pack_bf16x8(ds[8], ds[9], ds[10], ds[11], ds[12], ds[13], ds[14], ds[15]);
    };
    // Blocks with a large |dS| add the residuals of the rounding (rare; the block's tile stays in LDS until both groups
    // have passed the next matrix phase).  Called after the masked / unmasked variants of the vector phase have joined,
    // so that the accumulators are not modified inside either branch.
    auto v_phase_end = [&](int buf, int half) __attribute__((always_inline)) {
        const f32x4 h0 = __builtin_bit_cast(f32x4, dsf[0]), h1 = __builtin_bit_cast(f32x4, dsf[1]);
        const uint32_t hw[8] = {__float_as_uint(h0[0]), __float_as_uint(h0[1]), __float_as_uint(h0[2]), __float_as_uint(h0[3]),
                                __float_as_uint(h1[0]), __float_as_uint(h1[1]), __float_as_uint(h1[2]), __float_as_uint(h1[3])};
        // |x| >= 2 for a bf16 x is bit 14 of its pattern (the exponent's top bit): one test over the OR of the packed pairs
        static_assert(DS_SPLIT == 2.0f, "the test below is bit 14 of the bf16 pattern");
        const uint32_t any_bits = hw[0] | hw[1] | hw[2] | hw[3] | hw[4] | hw[5] | hw[6] | hw[7];
        dq_add_residuals<NDB, P16_ROW_BYTES>(dq, ds, hw, kres_addr + buf * P16_TILE_BYTES + 32 * half * P16_ROW_BYTES,
                                            __builtin_amdgcn_ballot_w64((any_bits & 0x40004000u) != 0u));
        // keep the whole vector phase on this side of the next barrier
        asm volatile("" : "+v"(dsf[0]), "+v"(dsf[1]));
    };

    // Phase sequence of a group: M(0) V(0) M(1) V(1) ... M(2 NT) over the 2 NT blocks; group 0 passes a workgroup
    // barrier before every matrix phase, group 1 before its first matrix phase and before every vector phase
    // (2 NT + 1 barriers each), which keeps group 1 one phase behind group 0.  Tile j must have landed before
    // group 0 enters M of its first block: group 0 (V) waits there, group 1 (K) waits before the vector phase
    // it runs in that same slot, V(2j - 1).  At that point tiles up to min(j + 2, NT - 1) have been requested.
    auto need_tile = [&](int j) __attribute__((always_inline)) {
        if (j < NT) wait_tiles_in_flight<DMA_PER_WAVE>((j + 2 < NT - 1 ? j + 2 : NT - 1) - j, my_xfers);
    };
    auto enter_m = [&](int blk) __attribute__((always_inline)) {
        if (grp == 0 && (blk & 1) == 0) need_tile(blk >> 1);
        if (grp == 0 || !PAIR_BARRIER) wg_barrier();
    };
    auto vector_part = [&](int blk) __attribute__((always_inline)) {
        if (grp == 1 && (blk & 1) == 1) need_tile((blk + 1) >> 1);
        if (grp == 1 || !PAIR_BARRIER) wg_barrier();
        const int t = blk >> 1;
        if ((blk & 1) == 0 && t + AHEAD < NT) fetch_tile(t + AHEAD);
        if (t >= n_full_g) v_phase(t & (2 * NB - 1), blk & 1, std::true_type{});
        else v_phase(t & (2 * NB - 1), blk & 1, std::false_type{});
        v_phase_end(t & (NB - 1), blk & 1);
    };

    for (int j = 0; j < AHEAD && j < NT; ++j) fetch_tile(j);
    if (grp == 1) {   // K(0) complete before anyone's M(0)
        need_tile(0);
        wg_barrier();
    }
    enter_m(0); m_phase(IC<0>{}, IC<0>{}, IC<NDQ>{}, IC<NST>{}); vector_part(0);
    enter_m(1); m_phase(IC<0>{}, IC<1>{}, IC<0>{}, IC<NST>{}); vector_part(1);
    // tiles 1 .. NT-1: four at a time in a straight line (buffer = t % 4 is then a compile-time constant and no
    // accumulator passes through a control-flow merge), then the remaining ones through a switch
    auto tile_steps = [&](int t, auto bc) __attribute__((always_inline)) {
        enter_m(2 * t);     m_phase(bc, IC<0>{}, IC<0>{}, IC<NST>{}); vector_part(2 * t);
        enter_m(2 * t + 1); m_phase(bc, IC<1>{}, IC<0>{}, IC<NST>{}); vector_part(2 * t + 1);
    };
    int t = 1;
    for (; t + 3 < NT; t += 4) {
        tile_steps(t, IC<1>{});
        tile_steps(t + 1, IC<2>{});
        tile_steps(t + 2, IC<3>{});
        tile_steps(t + 3, IC<0>{});
    }
    for (; t < NT; ++t) {
        switch (t & 3) {
            case 0: tile_steps(t, IC<0>{}); break;
            case 1: tile_steps(t, IC<1>{}); break;
            case 2: tile_steps(t, IC<2>{}); break;
            default: tile_steps(t, IC<3>{}); break;
        }
    }
    enter_m(2 * NT);
    switch (NT & 3) {
        case 0: m_phase(IC<0>{}, IC<0>{}, IC<0>{}, IC<NDQ>{}); break;
        case 1: m_phase(IC<1>{}, IC<0>{}, IC<0>{}, IC<NDQ>{}); break;
        case 2: m_phase(IC<2>{}, IC<0>{}, IC<0>{}, IC<NDQ>{}); break;
        default: m_phase(IC<3>{}, IC<0>{}, IC<0>{}, IC<NDQ>{}); break;
    }
    if (!PAIR_BARRIER && grp == 0) wg_barrier();
    __syncthreads();   // every wavefront is done with the tiles: LDS is free for the epilogue

    // Epilogue: dq_acc += scale * dQ.  The scaled rows go through LDS (a private 32 x (D + 4)-float region per
    // wavefront, padded against bank conflicts) so that the global read-modify-write is row-contiguous: one
    // instruction covers 1 KB of whole rows (two at D = 128).  Each (row, head) belongs to exactly one workgroup.
    float* stage = reinterpret_cast<float*>(&sm) + wave * (32 * STAGE_STRIDE);
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int b = 0; b < 4; ++b)
            *reinterpret_cast<float4*>(&stage[l32 * STAGE_STRIDE + 32 * db + 8 * b + 4 * hh]) =
                make_float4(dq[db][4 * b] * g.scale, dq[db][4 * b + 1] * g.scale, dq[db][4 * b + 2] * g.scale, dq[db][4 * b + 3] * g.scale);
    // the region is private to the wavefront: its own LDS writes only need to have completed
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // lane -> (row within a group of ROWS_PER_INST rows, 16-byte piece of the row)
    constexpr int LANES_PER_ROW = D / 4, ROWS_PER_INST = 64 / LANES_PER_ROW, N_INST = 32 / ROWS_PER_INST;
    const int sub_row = lane / LANES_PER_ROW, piece = lane % LANES_PER_ROW;
    const int wrow0 = grow0 + 32 * wg;
    float* obase = a.dq + ((long long)wrow0 * g.nq + h) * D + 4 * piece;
    const long long row_stride = (long long)g.nq * D;
    float4 old[N_INST];
#pragma unroll
    for (int i = 0; i < N_INST; ++i) {
        const int r = ROWS_PER_INST * i + sub_row;
        old[i] = wrow0 + r < g.lq ? *reinterpret_cast<const float4*>(obase + r * row_stride) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int i = 0; i < N_INST; ++i) {
        const int r = ROWS_PER_INST * i + sub_row;
        const float4 val = *reinterpret_cast<const float4*>(&stage[r * STAGE_STRIDE + 4 * piece]);
        float4 o4 = old[i];
        o4.x += val.x; o4.y += val.y; o4.z += val.z; o4.w += val.w;
        if (wrow0 + r < g.lq) *reinterpret_cast<float4*>(obase + r * row_stride) = o4;
    }
}

}  // namespace

hipError_t hexi_launch_bwd_dq_bf16(const BwdArgs& a, hipStream_t s)
{
    const AttnGeom& g = a.g;
    const int n_q_tiles = (g.lq + WG_ROWS - 1) / WG_ROWS;
    // cost of a unit: the key tiles its q tile streams, plus the prologue and epilogue (about six tiles' worth); a
    // unit that sees nothing of the chunk returns at once
    float cost[4096];
    const int n_known = n_q_tiles < 4096 ? n_q_tiles : 4096;     // (longer shards: the remaining tiles count like the last known one)
    for (int p = 0; p < n_known; ++p) {
        const int q_tile = n_q_tiles - 1 - p;
        const int last_row = (q_tile * WG_ROWS + WG_ROWS < g.lq ? q_tile * WG_ROWS + WG_ROWS : g.lq) - 1;
        const int nt = (seg_rows_le(g.ks, seg_pos_of_row(g.qs, last_row)) + TN - 1) / TN;
        cost[p] = nt > 0 ? (float)nt + 6.0f : 0.25f;
    }
    unsigned grid = 0;
    const XcdSplit split = hexi_split_units(g.nq * n_q_tiles, [&](int u) { const int p = u % n_q_tiles; return cost[p < n_known ? p : n_known - 1]; }, &grid);
    if (grid == 0) return hipSuccess;
    if (g.d == 128) bwd_dq_bf16_kernel<128><<<grid, 512, 0, s>>>(a, n_q_tiles, split);
    else if (g.d == 64) bwd_dq_bf16_kernel<64><<<grid, 512, 0, s>>>(a, n_q_tiles, split);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}
