/*
 * hexi_attn.h -- C ABI of the MI355X (gfx950) chunked-ring causal attention library.
 *
 * One device's share of HexiSeq's asymmetric CP-HP attention (Sec. 3.2): a query shard of
 * arbitrary length and global offset (uneven group lengths L_k, Sec. 4.1), an arbitrary packed
 * subset of attention heads (per-rank head counts n_d, possibly non-contiguous ranges packed into
 * contiguous buffers, Sec. 3.2 "Sub-ring KV exchange"), run forward and backward against a stream
 * of source KV blocks, one per ring step (App. A.4, Eq. 10-12), with forward, backward and
 * recomputation all counted as attention work (App. A.1).  The paper presupposes ordinary softmax
 * attention and states no formula for it; the mask, scale, GQA map and log-sum-exp merge below are
 * the textbook ones.
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers owned by the caller; descriptors, segment lists and
 *     kv_of_q are HOST pointers read during the call only.  The library allocates no device memory
 *     and keeps no state between calls except a thread-local error string.
 *   - Every device call is enqueued on `hip_stream` (a hipStream_t; NULL = the default stream) and
 *     returns without synchronising.  On error nothing is enqueued.
 *   - Return value: HEXI_OK (0) or a negative error code; hexi_last_error() describes it.
 *   - Causal mask on GLOBAL positions, diagonal inclusive: key j is visible to query row i iff
 *     pos(j) <= pos(i).  Rows with no visible key in a chunk get lse = -INFINITY and o = 0.
 *   - LSE values are natural logarithms of the sum of exp(softmax_scale * <q, k>).
 *   - Layouts: q, d_o: [Lq][n_q_heads][head_dim] with the strides of the descriptor (elements);
 *     k, v: [Lc][n_kv_heads][head_dim] likewise; the head_dim stride is 1.  fp32 outputs are dense:
 *     o, dq_acc: [Lq][n_q_heads][head_dim]; dk, dv: [Lc][n_kv_heads][head_dim]; lse, delta:
 *     [n_q_heads][Lq].  Lq / Lc are the total lengths of q_range / kv_range.
 */
#ifndef HEXI_ATTN_H
#define HEXI_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HEXI_OK            0
#define HEXI_EINVAL       (-1)  /* null pointer, bad size, unsorted/overlapping/empty segments, bad head map */
#define HEXI_EUNSUPPORTED (-2)  /* head_dim / dtype combination without a kernel, position >= 2^31-1 */
#define HEXI_EALIGN       (-3)  /* a tensor base pointer or token/head stride is not 16-byte aligned */
#define HEXI_EWORKSPACE   (-4)  /* workspace smaller than hexi_workspace_bytes() */
#define HEXI_EHIP         (-5)  /* the HIP runtime refused a launch */
#define HEXI_EINFEASIBLE   (-6)  /* hexi_sched_solve: no candidate schedule fits the devices' memory */

#define HEXI_MAX_TOKEN_STRIDE (1 << 22)  /* elements; larger token strides are HEXI_EUNSUPPORTED */

#define HEXI_BF16 0
#define HEXI_F32  1

#define HEXI_MAX_SEGS 16

/* flags */
#define HEXI_ACCUMULATE     1u  /* fwd: merge the chunk's result into o/lse in place (fused LSE merge);
                                   bwd: dk/dv += instead of = */
#define HEXI_COMPUTE_DELTA  2u  /* bwd: first fill delta = rowsum(d_o * o) from the merged o */
#define HEXI_SKIP_DQ        4u  /* bwd: produce only dk/dv (dq_acc is not touched and may be NULL) */
#define HEXI_SKIP_DKDV      8u  /* bwd: produce only dq (dk/dv are not touched and may be NULL) */

#define HEXI_TILE_EMPTY   0
#define HEXI_TILE_FULL    1
#define HEXI_TILE_PARTIAL 2

/* Global token range [start, start+len). */
typedef struct { int64_t start, len; } hexi_seg;

/* A shard or a KV chunk: 1..HEXI_MAX_SEGS segments, ascending, non-overlapping, len > 0.  The rows
 * (columns) of the device tensors are the segments' tokens packed back to back in this order.  One
 * segment = a contiguous shard; two = a zigzag pair. */
typedef struct { int32_t n_segs; const hexi_seg* segs; } hexi_range;

typedef struct {
    int32_t dtype;              /* HEXI_BF16 | HEXI_F32: element type of q, k, v, d_o */
    int32_t head_dim;           /* 64 or 128 */
    int32_t n_q_heads;          /* local (assigned) q heads, packed */
    int32_t n_kv_heads;         /* local kv heads, packed */
    const int32_t* kv_of_q;     /* HOST [n_q_heads]: local kv head read by each local q head;
                                   NULL => h / (n_q_heads / n_kv_heads) */
    float   softmax_scale;      /* e.g. 1/sqrt(head_dim) */
    int64_t q_stride_tok, q_stride_head;    /* strides of q and d_o, in elements; token strides <= HEXI_MAX_TOKEN_STRIDE */
    int64_t kv_stride_tok, kv_stride_head;  /* strides of k and v, in elements */
} hexi_attn_desc;

/*
 * Offset / mask bookkeeping for one (query shard, KV chunk) pair -- the integer side of the uneven
 * shard lengths of Sec. 3.2 / Sec. 4.1 and of the per-step source block of App. A.4.  Pure host
 * function, exact integer arithmetic, no GPU needed.  Any output pointer may be NULL.
 *   q_pos [Lq], kv_pos [Lc]: global position of every packed row / column (HOST, int32).
 *   tile_class: HOST uint8, row-major [ceil(Lq/tile_m)][ceil(Lc/tile_n)], HEXI_TILE_* per tile
 *               (tiles clipped at the ragged edge): EMPTY = no visible pair, FULL = all visible.
 *   n_pairs: number of visible (row, column) pairs of the whole grid.
 * Errors: HEXI_EINVAL for malformed ranges or tile sizes <= 0; HEXI_EUNSUPPORTED if a position
 * does not fit int32.
 */
int hexi_shard_mask(const hexi_range* q_range, const hexi_range* kv_range, int32_t tile_m, int32_t tile_n,
                    int32_t* q_pos, int32_t* kv_pos, uint8_t* tile_class, int64_t* n_pairs);

/*
 * One ring step forward (App. A.4, Eq. 11: the local query block against one source KV block):
 * for every local q head h and shard row i, over the chunk's visible columns j,
 *   s_ij = softmax_scale * <q_ih, k_j,kv(h)>,  lse_ih = ln sum_j exp(s_ij),
 *   o_ih = sum_j exp(s_ij - lse_ih) * v_j,kv(h)      (normalised partial result).
 * Without HEXI_ACCUMULATE o/lse are overwritten with this chunk's partial; with it they are the
 * running accumulators and the partial is merged in place by the rule of hexi_attn_merge_lse (start
 * from o = 0, lse = -INFINITY).  A chunk wholly in the shard's future costs one fill (or nothing
 * under HEXI_ACCUMULATE).  o: fp32 [Lq][nq][d]; lse: fp32 [nq][Lq].  workspace may be NULL when
 * hexi_workspace_bytes() is 0.
 */
int hexi_attn_fwd_chunk(const hexi_attn_desc* desc, const hexi_range* q_range, const hexi_range* kv_range,
                        const void* q, const void* k, const void* v,
                        float* o, float* lse, uint32_t flags,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Combine two normalised partial results over disjoint key sets (the rule that makes the ring's
 * per-step results equal un-sharded attention, Sec. 3.2 "preserving attention semantics"):
 *   lse = ln(e^lse_acc + e^lse_part);  o = e^(lse_acc - lse) o_acc + e^(lse_part - lse) o_part,
 * written back into o_acc / lse_acc.  -INFINITY is the identity.  If o_final is not NULL the merged
 * o is also written there in o_final_dtype (HEXI_BF16 or HEXI_F32), dense [n_rows][nq][d].
 * o_*: fp32 [n_rows][n_q_heads][head_dim]; lse_*: fp32 [n_q_heads][n_rows].  head_dim % 4 == 0.
 */
int hexi_attn_merge_lse(int64_t n_rows, int32_t n_q_heads, int32_t head_dim,
                        float* o_acc, float* lse_acc, const float* o_part, const float* lse_part,
                        void* o_final, int32_t o_final_dtype, void* hip_stream);

/*
 * One ring step backward with recomputation (App. A.1: attention work = forward + backward +
 * recomputation; App. A.4 step shape).  P is recomputed from the saved GLOBAL lse of the merged
 * forward:  P_ij = exp(s_ij - lse_i);  dV_j = sum_{h in group} sum_i P_ij dO_i;
 *   dP_ij = <dO_i, v_j>;  dS_ij = P_ij (dP_ij - delta_i);  dQ_i += scale sum_j dS_ij k_j;
 *   dK_j = scale sum_{h in group} sum_i dS_ij q_i.
 * o is the merged fp32 forward output and is read only under HEXI_COMPUTE_DELTA (which fills
 * delta for the whole shard before the chunk is processed); otherwise delta is an input.
 * dq_acc (fp32) accumulates over calls: the caller zeroes it before the first chunk.  Each dq row is
 * updated by one workgroup per call in a fixed order (bf16 path), so dq is reproducible run to run.
 * dk, dv (fp32, this chunk's rows) are overwritten, or added to under HEXI_ACCUMULATE.  The local q
 * heads that share a kv head are summed inside one workgroup when the launch is large enough
 * without splitting them (dk/dv are then reproducible run to run); otherwise groups are cut into
 * runs of heads whose contributions are summed with floating-point atomics, whose order (and so
 * the last bits of dk/dv) can vary between runs.  hexi_set_dkdv_run_len() overrides the run length
 * chosen by the library.  HEXI_SKIP_DQ / HEXI_SKIP_DKDV
 * restrict the call to one of the two halves (they are separate kernels and may be issued on
 * different streams); both set is HEXI_EINVAL.  A chunk
 * wholly in the shard's future writes zeros to dk/dv (nothing under HEXI_ACCUMULATE) and leaves
 * dq_acc untouched.  d_o has the dtype and strides of q.
 */
int hexi_attn_bwd_chunk(const hexi_attn_desc* desc, const hexi_range* q_range, const hexi_range* kv_range,
                        const void* q, const void* k, const void* v, const float* o, const void* d_o,
                        const float* lse, float* delta,
                        float* dq_acc, float* dk, float* dv, uint32_t flags,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Head redistribution either side of the ring (Sec. 3.2: heterogeneous all-to-all with per-rank split
 * tables; sub-ring KV exchange, where non-contiguous head slices are packed into contiguous buffers
 * before transfer; App. A.4: the part for rank j is s * n_j * d_h elements per tensor).
 *
 * x, y: DEVICE [s][n_heads_total][head_dim], elements of elem_bytes (2 or 4) bytes, d contiguous,
 * heads packed, token stride x_stride_tok ELEMENTS (>= n_heads_total * head_dim).  This is a
 * device's pre-A2A sequence shard with all heads, or any tensor a head subset is cut from (Q, K,
 * V, or all three fused along the head axis).
 * heads_per_rank: HOST int32[n_ranks], n_j >= 0.  head_list: HOST int32[sum n_j]: rank 0's heads,
 * then rank 1's, ..., each in [0, n_heads_total), in the order the rank wants them; at most
 * HEXI_A2A_MAX_SLOTS entries, n_ranks <= HEXI_A2A_MAX_RANKS.  Both are copied during the call.
 * packed: DEVICE, contiguous: for j = 0 .. n_ranks-1 the part [s][n_j][head_dim] (sum n_j * s *
 * head_dim elements in all).  hexi_a2a_pack gathers x into packed (a head may be listed for several
 * ranks: replicated kv heads); hexi_a2a_unpack scatters packed into y, leaves heads that no rank
 * lists untouched, and refuses a head listed twice (HEXI_EINVAL).  Results are exact copies.
 * head_dim * elem_bytes and x_stride_tok * elem_bytes must be multiples of 16 and all base pointers
 * 16-byte aligned (HEXI_EALIGN).  Enqueued on hip_stream, no synchronisation, nothing enqueued on
 * error; s == 0 or an empty head_list is a no-op.
 */
#define HEXI_A2A_MAX_SLOTS 256
#define HEXI_A2A_MAX_RANKS 64
int hexi_a2a_pack(const void* x, void* packed, int64_t s, int32_t n_heads_total, int32_t head_dim, int32_t elem_bytes,
                  int64_t x_stride_tok, int32_t n_ranks, const int32_t* heads_per_rank, const int32_t* head_list,
                  void* hip_stream);
int hexi_a2a_unpack(const void* packed, void* y, int64_t s, int32_t n_heads_total, int32_t head_dim, int32_t elem_bytes,
                    int64_t y_stride_tok, int32_t n_ranks, const int32_t* heads_per_rank, const int32_t* head_list,
                    void* hip_stream);

/*
 * Host-side performance model and hierarchical scheduler (Sec. 4: formalization, performance model,
 * scheduler; App. A: cost and memory model; App. B: the scheduler's algorithm).  No GPU is touched.
 * All pointers are HOST pointers; inputs are read during the call only.
 *
 * hexi_cluster: n_devices <= HEXI_SCHED_MAX_DEVICES; c[d] compute throughput (FLOP/s), b[d] memory
 * bandwidth (bytes/s), m[d] HBM capacity and m_static[d] schedule-independent residency (bytes);
 * alpha[i*n + j] startup latency (s) and bw[i*n + j] bandwidth (bytes/s) of the link i -> j (the
 * diagonal is ignored).  hexi_model: L_tot, microbatch B, hidden size H, head dimension d_h, number of
 * attention heads, bytes per element, activation-retention coefficient gamma_act (the paper uses 2).
 * hexi_schedule: n_groups A2A groups forming a ring in index order; group_of[d] in [0, n_groups);
 * l_group[k] = L_k (array of n_devices entries, the first n_groups used); s_pre[d], n_heads[d] per
 * device, with sum_{d in G_k} s_pre = L_k, sum_{d in G_k} n_heads = number of heads for every group
 * (every group attends with all heads over its block), sum_k L_k = L_tot.  Heads lie over a group's
 * devices in device order.
 *
 * hexi_sched_cost: terms[0] = T_blk = terms[1] (max_d T_nonattn) + terms[2] (max_k T_A2A) + terms[3]
 * (sum over the ring steps of T_step) in seconds (terms may be NULL); *is_feasible = 1 iff
 * m_static + Mem_act <= m on every device.  A schedule that violates the constraints above is
 * HEXI_EINVAL.
 * hexi_sched_solve: the three-stage search (topology partitions incl. the Ring / Ulysses / USP
 * layouts, group sequence splits, rank-level coordinate descent); writes the lowest-cost feasible
 * schedule into *out (caller-allocated arrays of n_devices entries each; groups are numbered in
 * order of their smallest device) and its T_blk into *cost.  opts may be NULL; zero fields take the
 * defaults M1 = 64, M2 = 16, I_max = 100 (Sec. 4.3), gap_ratio = 4, token_quantum = 64, perturb =
 * 1/32, move_tokens = max(1, L_tot / (quantum * n_devices * 16)) * quantum.  L_tot must be a multiple
 * of the token quantum.  HEXI_EINFEASIBLE if nothing passes the memory filter.  Deterministic.
 */
#define HEXI_SCHED_MAX_DEVICES 4096
typedef struct {
    int32_t n_devices;
    const double* c;
    const double* b;
    const double* m;
    const double* m_static;
    const double* alpha;
    const double* bw;
} hexi_cluster;
typedef struct {
    int64_t l_tot;
    int32_t batch, hidden, head_dim, n_heads, dtype_bytes;
    double gamma_act;
} hexi_model;
typedef struct {
    int32_t m1, m2, i_max, token_quantum;
    double gap_ratio, perturb;
    int64_t move_tokens;
} hexi_sched_opts;
typedef struct {
    int32_t n_groups;
    int32_t* group_of;
    int64_t* l_group;
    int64_t* s_pre;
    int32_t* n_heads;
} hexi_schedule;
int hexi_sched_cost(const hexi_cluster* cluster, const hexi_model* model, const hexi_schedule* schedule,
                    double* terms, int32_t* is_feasible);
int hexi_sched_solve(const hexi_cluster* cluster, const hexi_model* model, const hexi_sched_opts* opts,
                     hexi_schedule* out, double* cost);

/*
 * Tuning / test knob of hexi_attn_bwd_chunk's dK/dV part (the GQA sum over the n_d local heads of a
 * group, Sec. 3.2): the number of q heads of one kv head that a workgroup walks into the same
 * accumulators.  0 = chosen by the library per call (the default); n >= 1 = at most n (clamped to
 * the largest group).  The initial value is read once, when the library is loaded, from the
 * environment variable HEXI_DKDV_RUN_LEN.  Process-wide; not synchronised with calls in flight on
 * other threads.  Returns the previous value.
 */
int32_t hexi_set_dkdv_run_len(int32_t run_len);

/* Bytes of device workspace the chunk calls need for this descriptor and these lengths
 * (currently 0: no kernel uses scratch memory). */
size_t hexi_workspace_bytes(const hexi_attn_desc* desc, int64_t lq, int64_t lc);

/* Description of the last error on the calling thread ("" if none). */
const char* hexi_last_error(void);

/* Library version string, e.g. "hexi-attn 0.1 (gfx950)". */
const char* hexi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HEXI_ATTN_H */
