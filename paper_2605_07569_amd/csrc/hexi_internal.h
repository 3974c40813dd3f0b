// Internal declarations shared by the host entry points and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "hexi_attn.h"

#define HEXI_MAX_HEADS 128

// Segment table of a shard / chunk, passed by value in kernel arguments.
// Rows are packed in ascending global position (segments ascending, non-overlapping).
struct SegTable {
    int n;                          // number of segments
    int total;                      // total packed rows
    int start[HEXI_MAX_SEGS];       // global position of each segment's first token
    int row0[HEXI_MAX_SEGS + 1];    // packed row of each segment's first token; row0[n] = total
};

// Global position of a packed row (row must be < total).
__host__ __device__ inline int seg_pos_of_row(const SegTable& t, int row)
{
    int p = 0;
    for (int s = 0; s < t.n; ++s)
        if (row >= t.row0[s]) p = t.start[s] + (row - t.row0[s]);
    return p;
}

// Number of packed rows whose position is <= p.  Because positions ascend with the packed row
// index, these rows are exactly rows [0, count).
__host__ __device__ inline int seg_rows_le(const SegTable& t, int p)
{
    int c = 0;
    for (int s = 0; s < t.n; ++s) {
        const int len = t.row0[s + 1] - t.row0[s];
        int k = p - t.start[s] + 1;
        k = k < 0 ? 0 : (k > len ? len : k);
        c += k;
    }
    return c;
}

struct AttnGeom {
    int lq, lc, nq, nkv, d;
    long long q_stride_tok, q_stride_head, kv_stride_tok, kv_stride_head;  // elements
    float scale;
    SegTable qs, ks;
    signed char kv_of_q[HEXI_MAX_HEADS];
};

struct FwdArgs {
    AttnGeom g;
    const void *q, *k, *v;
    float *o, *lse;
    int accumulate;
};

struct BwdArgs {
    AttnGeom g;
    const void *q, *k, *v, *d_o;
    const float *lse, *delta;
    float *dq, *dk, *dv;
    int accumulate;
    int want_dq, want_dkdv;   // which halves of the backward step to run
};

// Launchers (each returns a hipError_t from the launch).
hipError_t hexi_launch_fwd_f32(const FwdArgs& a, hipStream_t s);
hipError_t hexi_launch_bwd_f32(const BwdArgs& a, hipStream_t s);
hipError_t hexi_launch_fwd_bf16(const FwdArgs& a, hipStream_t s);
hipError_t hexi_launch_bwd_bf16(const BwdArgs& a, hipStream_t s);      // dK/dV kernel, then the dQ kernel
hipError_t hexi_launch_bwd_dq_bf16(const BwdArgs& a, hipStream_t s);
hipError_t hexi_launch_merge(long long n_rows, int nq, int d, float* o_acc, float* lse_acc, const float* o_part,
                             const float* lse_part, void* o_final, int o_final_dtype, hipStream_t s);
hipError_t hexi_launch_delta(long long lq, int nq, int d, const float* o, const void* d_o, int dtype,
                             long long stride_tok, long long stride_head, float* delta, hipStream_t s);
hipError_t hexi_launch_fill_f32(float* p, long long n, float value, hipStream_t s);
hipError_t hexi_launch_mfma_probe(const void* operands, float* sink, int iters, hipStream_t s);
// pack (x -> packed) or unpack (packed -> y, which has x's layout); host tables, validated by the caller
hipError_t hexi_launch_a2a(bool pack, const void* x, void* packed, void* y, long long s, int n_heads_total, int row_bytes,
                           long long x_stride_bytes, int n_ranks, const int* heads_per_rank, const int* head_list, hipStream_t st);
