// Measurement aid, built into its own library (libhexi_probe.so): a register-only MFMA loop that shows what the
// matrix cores sustain on given operand bits with nothing else going on.  Not part of the attention library.
// 256 workgroups x 8 wavefronts (two per SIMD), four independent accumulators per wavefront.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "hexi_probe.h"

namespace {

typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));

__global__ void __launch_bounds__(512) mfma_probe_kernel(const probe_bf16x8* __restrict__ in, float* __restrict__ sink, int iters)
{
    probe_bf16x8 a[4], b[4];
    for (int i = 0; i < 4; ++i) { a[i] = in[(threadIdx.x * 8 + i) % 4096]; b[i] = in[(threadIdx.x * 8 + 4 + i) % 4096]; }
    probe_f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2], b[2], c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[3], b[3], c3, 0, 0, 0);
    }
    float s = 0.f;
    for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
    sink[blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace

extern "C" __attribute__((visibility("default")))
int hexi_mfma_probe(const void* operands, float* sink, int32_t iters, void* hip_stream)
{
    if (!operands || !sink || iters < 1) return -1;
    if (reinterpret_cast<uintptr_t>(operands) & 15u) return -3;
    mfma_probe_kernel<<<256, 512, 0, (hipStream_t)hip_stream>>>(static_cast<const probe_bf16x8*>(operands), sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}
