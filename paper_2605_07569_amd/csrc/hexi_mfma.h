// gfx950 MFMA / LDS helpers shared by the bf16 forward and backward kernels.
//
// v_mfma_f32_32x32x16_bf16 operand layout (wave64; l32 = lane % 32, hh = lane / 32):
//   A (32 x 16): lane holds row l32, contraction slots k = 8*hh + e, e = 0..7
//   B (16 x 32): lane holds column l32, contraction slots k = 8*hh + e
//   C (32 x 32): lane holds column l32; register r = 4*b + t holds row 8*b + 4*hh + t
// The contraction index may be permuted freely as long as A and B agree.  Feeding accumulator
// registers [8*x .. 8*x+7] of one lane straight back in as an operand therefore assigns slot
// (hh, e) to accumulator row 16*x + 8*(e/4) + 4*hh + (e%4); the other operand is then fetched with
// that same assignment.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

#define HEXI_LDS __attribute__((address_space(3)))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives, for e = 0..3, the (i % 4)-th
// 16-bit element of the 8-byte word addressed by lane 4*e + i/4 of its group.  With lane j
// addressing element [row0 + j/4][col0 + 4*(j%4)] of a row-major tile, lane i ends up with the four
// elements [row0 + e][col0 + i]: a 4 x 16 block read transposed.
__device__ __forceinline__ s16x4 lds_read_tr16(const uint16_t* p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 HEXI_LDS*)(p));
}

// Eight contraction slots for a lane from two transposed 4-row reads (rows row_a.. and row_b..).
__device__ __forceinline__ bf16x8 lds_tr_pair(const uint16_t* pa, const uint16_t* pb)
{
    const s16x4 x = lds_read_tr16(pa), y = lds_read_tr16(pb);
    s16x8 r = {x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
    return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ bf16x8 pack_bf16x8(float a0, float a1, float a2, float a3, float a4, float a5, float a6, float a7)
{
    bf16x8 r;
    r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
    r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
    return r;
}

// Rounds 8 probabilities to bf16 operand slots and adds the ROUNDED values to `sum` (v_dot2c_f32_bf16
// against a vector of ones), so that a normaliser built from `sum` matches the weights the MFMA
// actually uses.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x8 pack_bf16x8_sum(float a0, float a1, float a2, float a3, float a4, float a5, float a6, float a7, float& sum)
{
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    const bf16x2 t0 = {(__bf16)a0, (__bf16)a1}, t1 = {(__bf16)a2, (__bf16)a3}, t2 = {(__bf16)a4, (__bf16)a5}, t3 = {(__bf16)a6, (__bf16)a7};
    sum = __builtin_amdgcn_fdot2_f32_bf16(t0, ones, sum, false);
    sum = __builtin_amdgcn_fdot2_f32_bf16(t1, ones, sum, false);
    sum = __builtin_amdgcn_fdot2_f32_bf16(t2, ones, sum, false);
    sum = __builtin_amdgcn_fdot2_f32_bf16(t3, ones, sum, false);
    bf16x8 r = {t0[0], t0[1], t1[0], t1[1], t2[0], t2[1], t3[0], t3[1]};
    return r;
}

// Same with four independent running sums (one per pair), so that the additions do not form one chain.
__device__ __forceinline__ bf16x8 pack_bf16x8_sum4(float a0, float a1, float a2, float a3, float a4, float a5, float a6, float a7, float (&sum)[4])
{
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    const bf16x2 t0 = {(__bf16)a0, (__bf16)a1}, t1 = {(__bf16)a2, (__bf16)a3}, t2 = {(__bf16)a4, (__bf16)a5}, t3 = {(__bf16)a6, (__bf16)a7};
    sum[0] = __builtin_amdgcn_fdot2_f32_bf16(t0, ones, sum[0], false);
    sum[1] = __builtin_amdgcn_fdot2_f32_bf16(t1, ones, sum[1], false);
    sum[2] = __builtin_amdgcn_fdot2_f32_bf16(t2, ones, sum[2], false);
    sum[3] = __builtin_amdgcn_fdot2_f32_bf16(t3, ones, sum[3], false);
    bf16x8 r = {t0[0], t0[1], t1[0], t1[1], t2[0], t2[1], t3[0], t3[1]};
    return r;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Direct global->LDS load (LDS DMA): every lane supplies its own global address; the 64 lanes' 16-byte
// (or 4-byte) pieces land back to back in LDS starting at the wave-uniform byte address `lds_addr`
// (passed through M0).  Completion is tracked by vmcnt; the caller waits with s_waitcnt vmcnt(0)
// before the barrier that publishes the data.  Issued through inline assembly so the compiler does
// not order unrelated LDS reads behind it.
__device__ __forceinline__ void lds_dma16(const void* gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory");
}
// Same with a wave-uniform 64-bit base in SGPRs and a 32-bit per-lane byte offset.
__device__ __forceinline__ void lds_dma16_base(const void* base, uint32_t byte_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(byte_off), "s"(base) : "memory");
}
__device__ __forceinline__ void lds_dma4(const void* gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(gptr) : "memory");
}

// LDS reads issued through inline assembly with a compile-time offset field, for software pipelines whose
// address registers must stay exactly the ones the kernel computed (the compiler otherwise materialises
// one address register per buffer).  The compiler does not see these reads: the destination is valid
// only after the matching lds_wait<N>(), which waits until at most N younger LDS operations of the
// wavefront are outstanding and ties the destination registers to the wait, so that no consumer (and no
// register copy) can be scheduled before it.
template <int OFF> __device__ __forceinline__ void lds_issue_b128(bf16x8& r, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
}
template <int OFF> __device__ __forceinline__ void lds_issue_tr16(s16x4& r, uint32_t addr)
{
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
}
template <int N> __device__ __forceinline__ void lds_wait(bf16x8& r)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(r) : "n"(N));
}
template <int N> __device__ __forceinline__ void lds_wait(s16x4& a, s16x4& b)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}
__device__ __forceinline__ bf16x8 join_halves(s16x4 x, s16x4 y)
{
    s16x8 r = {x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
    return __builtin_bit_cast(bf16x8, r);
}

// fp32 atomic add to global memory without a return value (global_atomic_add_f32)
__device__ __forceinline__ void global_atomic_add(float* p, float v)
{
    __builtin_amdgcn_global_atomic_fadd_f32((float __attribute__((address_space(1)))*)p, v);
}

// max of three without NaN canonicalisation overhead (scores are finite or -inf)
__device__ __forceinline__ float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float max2(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
// max over the two half-waves: lanes l and l^32 end up with max(x[l], x[l^32]) (v_permlane32_swap, no LDS)
__device__ __forceinline__ float max_across_halves(float x)
{
    const unsigned xi = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    return max2(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float x)
{
    const unsigned xi = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Forces a value that came from an ordinary global load to be complete here.  The direct global->LDS
// loads above are invisible to the compiler's wait-count bookkeeping; if an ordinary load were
// still pending when they are issued, the compiler's later "wait until that load is done" would
// also wait for every LDS DMA issued since.  Pinning the operand fragments before the main loop
// keeps all such waits out of the loop.
__device__ __forceinline__ void pin(const bf16x8& x) { asm volatile("" ::"v"(x)); }

// Scheduling hints (one scheduling group each): the next `n` instructions of a class, in order.
#define HEXI_SCHED_MFMA(n) __builtin_amdgcn_sched_group_barrier(0x008, n, 0)
#define HEXI_SCHED_DSREAD(n) __builtin_amdgcn_sched_group_barrier(0x100, n, 0)
#define HEXI_SCHED_DSWRITE(n) __builtin_amdgcn_sched_group_barrier(0x200, n, 0)
#define HEXI_SCHED_VALU(n) __builtin_amdgcn_sched_group_barrier(0x002, n, 0)

// ---- helpers of the ping-pong kernels (8 wavefronts, two groups alternating matrix and vector phases) ----

template <int N> using IC = std::integral_constant<int, N>;

// f(IC<FIRST>{}), ..., f(IC<LAST - 1>{})
template <int FIRST, int... I, class F> __device__ __forceinline__ void for_range_impl(std::integer_sequence<int, I...>, F& f)
{
    (f(IC<FIRST + I>{}), ...);
}
template <int FIRST, int LAST, class F> __device__ __forceinline__ void for_range(F& f)
{
    for_range_impl<FIRST>(std::make_integer_sequence<int, LAST - FIRST>{}, f);
}

// Tiles are fetched with wave-wide global->LDS transfers, PER_TILE of them per wavefront per tile; transfers
// complete in order, so "at most `allowed_tiles` younger tiles still in flight" is a vmcnt of PER_TILE per tile.
template <int PER_TILE> __device__ __forceinline__ void wait_tiles_in_flight_n(int allowed_tiles)
{
    static_assert(3 * PER_TILE < 64, "vmcnt holds 6 bits");
    if (allowed_tiles >= 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * PER_TILE) : "memory");
    else if (allowed_tiles == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * PER_TILE) : "memory");
    else if (allowed_tiles == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER_TILE) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Same for a wavefront that issues `per_tile` transfers per tile, where per_tile (wave-uniform) is MOST or
// MOST - 1: the four wavefronts of a group share a tile's transfers round-robin.
template <int MOST> __device__ __forceinline__ void wait_tiles_in_flight(int allowed_tiles, int per_tile)
{
    if (per_tile == MOST) wait_tiles_in_flight_n<MOST>(allowed_tiles);
    else wait_tiles_in_flight_n<MOST - 1>(allowed_tiles);
}

// Workgroup barrier that the compiler's scheduler does not move code across.
__device__ __forceinline__ void wg_barrier()
{
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

// LDS tile layout of the kernels that read a [64 rows][D bf16] tile (D = 64 or 128) both row-wise (128-bit
// reads, 32 consecutive rows across the lanes) and transposed (ds_read_b64_tr_b16, 4 consecutive rows per
// 16-lane group): rows are 2 D + 16 bytes apart (16 of padding: 68 or 36 dwords, so that 16 consecutive LDS
// rows start 4 banks apart and every fourth one 16 banks apart) and stored in the order p16_row(), which
// swaps the two 2-bit digits of the row index inside every block of 16 rows.  Consecutive rows r..r+3 then
// sit 4 LDS rows (= 16 banks) apart, so both access patterns touch all 64 banks exactly once, and every
// operand fragment is at (one per-lane base register) + (a compile-time offset).  A tile is a whole number of
// wave-wide 1 KB transfers: 17 (D = 128) or 9 (D = 64).
__host__ __device__ constexpr int p16_row_bytes(int d) { return 2 * d + 16; }
__host__ __device__ constexpr int p16_tile_bytes(int d) { return 64 * p16_row_bytes(d); }
__host__ __device__ constexpr int p16_row(int r) { return (r & ~15) | ((r & 3) << 2) | ((r >> 2) & 3); }
