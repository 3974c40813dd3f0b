// HBM-bound elementwise kernels: two-term log-sum-exp merge, Delta = rowsum(dO * O), fill.
#include "hexi_internal.h"
#include <hip/hip_bf16.h>

namespace {

// One thread per 4 consecutive head_dim elements of one (row, head); this pass only reads the lse
// arrays (merge_lse_kernel rewrites lse_acc afterwards, so no thread ever sees a replaced value).
// o_*: [n_rows][nq][d] fp32, lse_*: [nq][n_rows].  Weights are formed as e_a/(e_a+e_b) with
// e_x = exp(lse_x - max), which keeps them exact convex weights; -inf on one side is the identity.
template <int OUT_MODE>  // 0: no o_final, 1: fp32 o_final, 2: bf16 o_final
__global__ void __launch_bounds__(256) merge_kernel(long long n_vec, int nq, int d4, long long n_rows,
                                                    float* __restrict__ o_acc, float* __restrict__ lse_acc,
                                                    const float* __restrict__ o_part, const float* __restrict__ lse_part,
                                                    void* __restrict__ o_final)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n_vec) return;
    const long long rh = idx / d4;
    const int c4 = (int)(idx - rh * d4);
    const long long row = rh / nq;
    const int h = (int)(rh - row * nq);
    const long long li = (long long)h * n_rows + row;
    const float a = lse_acc[li], b = lse_part[li];
    const float m = fmaxf(a, b);
    typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
    const nt_f32x4 oa_v = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4*>(o_acc) + idx);
    float4 oa = make_float4(oa_v[0], oa_v[1], oa_v[2], oa_v[3]);
    float4 r;
    if (m == -INFINITY) {
        r = make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
        const nt_f32x4 ob_v = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4*>(o_part) + idx);
        const float4 ob = make_float4(ob_v[0], ob_v[1], ob_v[2], ob_v[3]);
        const float ea = expf(a - m), eb = expf(b - m);
        const float inv = 1.0f / (ea + eb);
        const float wa = ea * inv, wb = eb * inv;
        r = make_float4(wa * oa.x + wb * ob.x, wa * oa.y + wb * ob.y, wa * oa.z + wb * ob.z, wa * oa.w + wb * ob.w);
    }
    { const nt_f32x4 r_v = {r.x, r.y, r.z, r.w}; __builtin_nontemporal_store(r_v, reinterpret_cast<nt_f32x4*>(o_acc) + idx); }
    if (OUT_MODE == 1) reinterpret_cast<float4*>(o_final)[idx] = r;
    if (OUT_MODE == 2) {
        __hip_bfloat16 t[4] = {__float2bfloat16(r.x), __float2bfloat16(r.y), __float2bfloat16(r.z), __float2bfloat16(r.w)};
        reinterpret_cast<uint2*>(o_final)[idx] = *reinterpret_cast<const uint2*>(t);
    }
}

// Second pass: one thread per (row, head) rewrites lse_acc.
__global__ void __launch_bounds__(256) merge_lse_kernel(long long n, float* __restrict__ lse_acc, const float* __restrict__ lse_part)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float a = lse_acc[i], b = lse_part[i];
    const float m = fmaxf(a, b);
    lse_acc[i] = (m == -INFINITY) ? -INFINITY : m + logf(expf(a - m) + expf(b - m));
}

}  // namespace

hipError_t hexi_launch_merge(long long n_rows, int nq, int d, float* o_acc, float* lse_acc, const float* o_part,
                             const float* lse_part, void* o_final, int o_final_dtype, hipStream_t s)
{
    const int d4 = d / 4;
    const long long n_vec = n_rows * nq * d4;
    const unsigned grid = (unsigned)((n_vec + 255) / 256);
    if (!o_final)
        merge_kernel<0><<<grid, 256, 0, s>>>(n_vec, nq, d4, n_rows, o_acc, lse_acc, o_part, lse_part, nullptr);
    else if (o_final_dtype == HEXI_F32)
        merge_kernel<1><<<grid, 256, 0, s>>>(n_vec, nq, d4, n_rows, o_acc, lse_acc, o_part, lse_part, o_final);
    else
        merge_kernel<2><<<grid, 256, 0, s>>>(n_vec, nq, d4, n_rows, o_acc, lse_acc, o_part, lse_part, o_final);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long n = n_rows * nq;
    merge_lse_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(n, lse_acc, lse_part);
    return hipGetLastError();
}

namespace {

// Delta[h][i] = sum_c dO[i][h][c] * O[i][h][c]; O fp32 dense, dO in the input dtype with strides.
// D/4 consecutive lanes share one (row, head).
template <typename T, int D>
__global__ void __launch_bounds__(256) delta_kernel(long long lq, int nq, const float* __restrict__ o, const T* __restrict__ d_o,
                                                    long long stride_tok, long long stride_head, float* __restrict__ delta)
{
    constexpr int LANES = D / 4;
    const long long rh = ((long long)blockIdx.x * 256 + threadIdx.x) / LANES;
    const int c4 = threadIdx.x % LANES;
    float acc = 0.f;
    const bool valid = rh < lq * nq;
    long long row = 0; int h = 0;
    if (valid) {
        row = rh / nq; h = (int)(rh - row * nq);
        typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
        const nt_f32x4 ov_v = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4*>(o + rh * D) + c4);
        const float4 ov = make_float4(ov_v[0], ov_v[1], ov_v[2], ov_v[3]);
        const T* p = d_o + row * stride_tok + h * stride_head + c4 * 4;
        float g0, g1, g2, g3;
        if constexpr (sizeof(T) == 4) {
            const float4 gv = *reinterpret_cast<const float4*>(p);
            g0 = gv.x; g1 = gv.y; g2 = gv.z; g3 = gv.w;
        } else {
            const uint2 raw = *reinterpret_cast<const uint2*>(p);
            g0 = __uint_as_float(raw.x << 16); g1 = __uint_as_float(raw.x & 0xffff0000u);
            g2 = __uint_as_float(raw.y << 16); g3 = __uint_as_float(raw.y & 0xffff0000u);
        }
        acc = ov.x * g0 + ov.y * g1 + ov.z * g2 + ov.w * g3;
    }
#pragma unroll
    for (int off = LANES / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (valid && c4 == 0) delta[(long long)h * lq + row] = acc;
}

}  // namespace

hipError_t hexi_launch_delta(long long lq, int nq, int d, const float* o, const void* d_o, int dtype,
                             long long stride_tok, long long stride_head, float* delta, hipStream_t s)
{
    const long long n_threads = lq * nq * (d / 4);
    const unsigned grid = (unsigned)((n_threads + 255) / 256);
    if (dtype == HEXI_F32) {
        if (d == 64) delta_kernel<float, 64><<<grid, 256, 0, s>>>(lq, nq, o, (const float*)d_o, stride_tok, stride_head, delta);
        else delta_kernel<float, 128><<<grid, 256, 0, s>>>(lq, nq, o, (const float*)d_o, stride_tok, stride_head, delta);
    } else {
        if (d == 64) delta_kernel<uint16_t, 64><<<grid, 256, 0, s>>>(lq, nq, o, (const uint16_t*)d_o, stride_tok, stride_head, delta);
        else delta_kernel<uint16_t, 128><<<grid, 256, 0, s>>>(lq, nq, o, (const uint16_t*)d_o, stride_tok, stride_head, delta);
    }
    return hipGetLastError();
}

namespace {

__global__ void __launch_bounds__(256) fill_kernel(float* __restrict__ p, long long n, float value)
{
    long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long stride = (long long)gridDim.x * 256;
    for (; i < n; i += stride) p[i] = value;
}

}  // namespace

hipError_t hexi_launch_fill_f32(float* p, long long n, float value, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    long long blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    fill_kernel<<<(unsigned)blocks, 256, 0, s>>>(p, n, value);
    return hipGetLastError();
}
