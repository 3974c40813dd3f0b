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

// Work split over the 8 XCDs of the chip.  Workgroup ids are dealt round-robin to the XCDs (id % 8) and every XCD
// starts its workgroups in id order, so workgroup `id` takes unit start[id % 8] + id / 8 of a launch whose units are
// numbered so that neighbours share their streamed operands (same head, adjacent tiles): every XCD works on a
// contiguous unit range, its L2 sees one head's stream at a time, and the ranges carry (nearly) equal WORK rather
// than equal counts -- under a causal mask the units of a head differ in length by large factors, and equal counts
// leave some XCDs idle for a sixth of a diagonal chunk's launch when a head's units straddle two XCDs.
struct XcdSplit {
    int start[9];     // XCD x takes units [start[x], start[x + 1])
};

// weight(u) > 0: estimated cost of unit u.  Returns the split and the grid size (8 x the longest range; workgroups
// past the end of their XCD's range exit at once).
template <class W> inline XcdSplit hexi_split_units(int n_units, W weight, unsigned* grid)
{
    double total = 0.0;
    for (int u = 0; u < n_units; ++u) total += weight(u);
    XcdSplit s;
    s.start[0] = 0;
    double acc = 0.0;
    int x = 1;
    for (int u = 0; u < n_units && x < 8; ++u) {
        acc += weight(u);
        while (x < 8 && acc * 8.0 >= total * x) s.start[x++] = u + 1;
    }
    while (x <= 8) s.start[x++] = n_units;
    int longest = 0;
    for (int i = 0; i < 8; ++i) longest = s.start[i + 1] - s.start[i] > longest ? s.start[i + 1] - s.start[i] : longest;
    *grid = 8u * (unsigned)longest;
    return s;
}

// Runs of q heads for the dK/dV kernel: run r covers len[r] heads starting at first[r], linked through next[] (all
// read kv head kv_of_q[first[r]]).
struct HeadRuns {
    int n;
    signed char first[HEXI_MAX_HEADS], next[HEXI_MAX_HEADS];
    unsigned char len[HEXI_MAX_HEADS];     // up to HEXI_MAX_HEADS = 128 heads in one run
};

// Cuts the q heads of every kv head, in head order, into runs of at most run_len heads.  Returns true when some kv
// head has more than one run (its runs then add their dK / dV tiles with atomics).
inline bool hexi_build_head_runs(const signed char* kv_of_q, int nq, int nkv, int run_len, HeadRuns* runs)
{
    int last[HEXI_MAX_HEADS], open_run[HEXI_MAX_HEADS];   // per kv head: its last q head so far, its run being filled
    bool shared = false;
    runs->n = 0;
    for (int kh = 0; kh < nkv; ++kh) { last[kh] = -1; open_run[kh] = -1; }
    for (int h = 0; h < nq; ++h) {
        const int kh = kv_of_q[h];
        runs->next[h] = -1;
        if (open_run[kh] >= 0 && runs->len[open_run[kh]] < run_len) {
            runs->next[last[kh]] = (signed char)h;
            ++runs->len[open_run[kh]];
        } else {
            shared |= open_run[kh] >= 0;     // a second run on this kv head
            open_run[kh] = runs->n;
            runs->first[runs->n] = (signed char)h;
            runs->len[runs->n] = 1;
            ++runs->n;
        }
        last[kh] = h;
    }
    return shared;
}

// Forced number of q heads per dK/dV workgroup run (0: the launcher chooses); see hexi_set_dkdv_run_len().
extern int hexi_dkdv_run_len;

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
// pack (x -> packed) or unpack (packed -> y, which has x's layout); host tables, validated by the caller
hipError_t hexi_launch_a2a(bool pack, const void* x, void* packed, void* y, long long s, int n_heads_total, int row_bytes,
                           long long x_stride_bytes, int n_ranks, const int* heads_per_rank, const int* head_list, hipStream_t st);
