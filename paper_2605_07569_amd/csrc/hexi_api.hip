// Host side of the C ABI: argument validation, segment tables, integer mask bookkeeping, dispatch.
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <cmath>
#include <vector>
#include "hexi_internal.h"

#define HEXI_EXPORT extern "C" __attribute__((visibility("default")))

static thread_local char g_err[320] = "";

// forced run length of the dK/dV launcher (0: automatic); initial value from the environment, read once
static int env_run_len()
{
    const char* v = getenv("HEXI_DKDV_RUN_LEN");
    const int n = v ? atoi(v) : 0;
    return n > 0 ? n : 0;
}
int hexi_dkdv_run_len = env_run_len();

static int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// the same for the host-only translation units
int hexi_set_error(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

HEXI_EXPORT const char* hexi_last_error(void) { return g_err; }
HEXI_EXPORT const char* hexi_version(void) { return "hexi-attn 0.1 (gfx950)"; }

// Validates a range and builds its segment table.  Positions must fit int32.
static int build_segtable(const hexi_range* r, const char* what, SegTable* t)
{
    if (!r || !r->segs) return fail(HEXI_EINVAL, "%s: null range", what);
    if (r->n_segs < 1 || r->n_segs > HEXI_MAX_SEGS)
        return fail(HEXI_EINVAL, "%s: n_segs=%d outside 1..%d", what, r->n_segs, HEXI_MAX_SEGS);
    memset(t, 0, sizeof(*t));
    int64_t rows = 0, prev_end = 0;
    for (int s = 0; s < r->n_segs; ++s) {
        const int64_t st = r->segs[s].start, ln = r->segs[s].len;
        if (st < 0 || ln <= 0) return fail(HEXI_EINVAL, "%s: segment %d has start=%lld len=%lld", what, s, (long long)st, (long long)ln);
        if (s > 0 && st < prev_end) return fail(HEXI_EINVAL, "%s: segment %d overlaps or precedes segment %d", what, s, s - 1);
        if (st + ln > 2147483647LL || rows + ln > 2147483647LL)
            return fail(HEXI_EUNSUPPORTED, "%s: positions beyond 2^31-1 are not supported", what);
        t->start[s] = (int)st;
        t->row0[s] = (int)rows;
        rows += ln;
        prev_end = st + ln;
    }
    t->n = r->n_segs;
    t->total = (int)rows;
    for (int s = r->n_segs; s <= HEXI_MAX_SEGS; ++s) t->row0[s] = (int)rows;
    return HEXI_OK;
}

HEXI_EXPORT int hexi_shard_mask(const hexi_range* q_range, const hexi_range* kv_range, int32_t tile_m, int32_t tile_n,
                               int32_t* q_pos, int32_t* kv_pos, uint8_t* tile_class, int64_t* n_pairs)
{
    SegTable qs, ks;
    int rc;
    if ((rc = build_segtable(q_range, "q_range", &qs)) != HEXI_OK) return rc;
    if ((rc = build_segtable(kv_range, "kv_range", &ks)) != HEXI_OK) return rc;
    if (tile_class && (tile_m <= 0 || tile_n <= 0)) return fail(HEXI_EINVAL, "tile sizes must be positive");
    if (q_pos)
        for (int s = 0; s < qs.n; ++s)
            for (int r = qs.row0[s]; r < qs.row0[s + 1]; ++r) q_pos[r] = qs.start[s] + (r - qs.row0[s]);
    if (kv_pos)
        for (int s = 0; s < ks.n; ++s)
            for (int r = ks.row0[s]; r < ks.row0[s + 1]; ++r) kv_pos[r] = ks.start[s] + (r - ks.row0[s]);
    if (n_pairs) {
        // Row at position p sees the columns with position <= p.  Within a q segment p runs over
        // consecutive integers, so each (q segment, kv segment) pair contributes a clipped ramp.
        int64_t total = 0;
        for (int a = 0; a < qs.n; ++a) {
            const int64_t lo = qs.start[a], hi = lo + (qs.row0[a + 1] - qs.row0[a]) - 1;
            for (int b = 0; b < ks.n; ++b) {
                const int64_t s = ks.start[b], n = ks.row0[b + 1] - ks.row0[b];
                const int64_t ra = lo > s ? lo : s;                    // first p on the ramp
                const int64_t rb = hi < s + n - 1 ? hi : s + n - 1;    // last p on the ramp
                if (ra <= rb) total += ((ra - s + 1) + (rb - s + 1)) * (rb - ra + 1) / 2;
                if (hi >= s + n) total += n * (hi - (lo > s + n ? lo : s + n) + 1);
            }
        }
        *n_pairs = total;
    }
    if (tile_class) {
        const int nm = (qs.total + tile_m - 1) / tile_m, nn = (ks.total + tile_n - 1) / tile_n;
        for (int tm = 0; tm < nm; ++tm) {
            const int r0 = tm * tile_m, r1 = (r0 + tile_m < qs.total ? r0 + tile_m : qs.total) - 1;
            const int q_min = seg_pos_of_row(qs, r0), q_max = seg_pos_of_row(qs, r1);
            for (int tn = 0; tn < nn; ++tn) {
                const int c0 = tn * tile_n, c1 = (c0 + tile_n < ks.total ? c0 + tile_n : ks.total) - 1;
                const int k_min = seg_pos_of_row(ks, c0), k_max = seg_pos_of_row(ks, c1);
                tile_class[(size_t)tm * nn + tn] =
                    k_min > q_max ? HEXI_TILE_EMPTY : (k_max <= q_min ? HEXI_TILE_FULL : HEXI_TILE_PARTIAL);
            }
        }
    }
    return HEXI_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int build_geom(const hexi_attn_desc* d, const hexi_range* q_range, const hexi_range* kv_range, AttnGeom* g)
{
    if (!d) return fail(HEXI_EINVAL, "null descriptor");
    if (d->dtype != HEXI_BF16 && d->dtype != HEXI_F32) return fail(HEXI_EUNSUPPORTED, "dtype %d not supported", d->dtype);
    if (d->head_dim != 64 && d->head_dim != 128) return fail(HEXI_EUNSUPPORTED, "head_dim %d not supported (64 or 128)", d->head_dim);
    if (d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads > HEXI_MAX_HEADS || d->n_kv_heads > d->n_q_heads)
        return fail(HEXI_EINVAL, "head counts nq=%d nkv=%d invalid (1 <= nkv <= nq <= %d)", d->n_q_heads, d->n_kv_heads, HEXI_MAX_HEADS);
    if (!(d->softmax_scale > 0.f) || !std::isfinite(d->softmax_scale)) return fail(HEXI_EINVAL, "softmax_scale must be positive and finite");
    int rc;
    if ((rc = build_segtable(q_range, "q_range", &g->qs)) != HEXI_OK) return rc;
    if ((rc = build_segtable(kv_range, "kv_range", &g->ks)) != HEXI_OK) return rc;
    g->lq = g->qs.total; g->lc = g->ks.total;
    g->nq = d->n_q_heads; g->nkv = d->n_kv_heads; g->d = d->head_dim;
    g->scale = d->softmax_scale;
    g->q_stride_tok = d->q_stride_tok; g->q_stride_head = d->q_stride_head;
    g->kv_stride_tok = d->kv_stride_tok; g->kv_stride_head = d->kv_stride_head;
    if (d->q_stride_head < d->head_dim || d->kv_stride_head < d->head_dim ||
        d->q_stride_tok < (int64_t)d->head_dim || d->kv_stride_tok < (int64_t)d->head_dim)
        return fail(HEXI_EINVAL, "strides must be at least head_dim");
    // the bf16 kernels address the 64 rows of a tile through 32-bit byte offsets from the tile's first row
    if (d->q_stride_tok > HEXI_MAX_TOKEN_STRIDE || d->kv_stride_tok > HEXI_MAX_TOKEN_STRIDE)
        return fail(HEXI_EUNSUPPORTED, "token stride above %d elements", HEXI_MAX_TOKEN_STRIDE);
    const int esz = d->dtype == HEXI_BF16 ? 2 : 4;
    if ((d->q_stride_tok * esz) % 16 || (d->q_stride_head * esz) % 16 || (d->kv_stride_tok * esz) % 16 || (d->kv_stride_head * esz) % 16)
        return fail(HEXI_EALIGN, "token and head strides must be multiples of 16 bytes");
    if (d->kv_of_q) {
        for (int h = 0; h < d->n_q_heads; ++h) {
            if (d->kv_of_q[h] < 0 || d->kv_of_q[h] >= d->n_kv_heads) return fail(HEXI_EINVAL, "kv_of_q[%d]=%d out of range", h, d->kv_of_q[h]);
            g->kv_of_q[h] = (signed char)d->kv_of_q[h];
        }
    } else {
        if (d->n_q_heads % d->n_kv_heads) return fail(HEXI_EINVAL, "kv_of_q is NULL but n_q_heads %% n_kv_heads != 0");
        const int grp = d->n_q_heads / d->n_kv_heads;
        for (int h = 0; h < d->n_q_heads; ++h) g->kv_of_q[h] = (signed char)(h / grp);
    }
    return HEXI_OK;
}

// True when no key of the chunk is visible to any row of the shard.
static bool chunk_in_future(const AttnGeom& g)
{
    const int q_max = seg_pos_of_row(g.qs, g.lq - 1);
    return g.ks.start[0] > q_max;
}

HEXI_EXPORT int32_t hexi_set_dkdv_run_len(int32_t run_len)
{
    const int32_t old = hexi_dkdv_run_len;
    hexi_dkdv_run_len = run_len > 0 ? run_len : 0;
    return old;
}

HEXI_EXPORT size_t hexi_workspace_bytes(const hexi_attn_desc*, int64_t, int64_t) { return 0; }

HEXI_EXPORT int hexi_attn_fwd_chunk(const hexi_attn_desc* desc, const hexi_range* q_range, const hexi_range* kv_range,
                                   const void* q, const void* k, const void* v, float* o, float* lse, uint32_t flags,
                                   void* workspace, size_t workspace_bytes, void* hip_stream)
{
    (void)workspace; (void)workspace_bytes;
    FwdArgs a;
    int rc = build_geom(desc, q_range, kv_range, &a.g);
    if (rc != HEXI_OK) return rc;
    if (!q || !k || !v || !o || !lse) return fail(HEXI_EINVAL, "null tensor pointer");
    if (flags & ~(HEXI_ACCUMULATE)) return fail(HEXI_EINVAL, "unknown flag bits 0x%x", flags);
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse))
        return fail(HEXI_EALIGN, "tensor base pointers must be 16-byte aligned");
    hipStream_t s = (hipStream_t)hip_stream;
    a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
    a.accumulate = (flags & HEXI_ACCUMULATE) ? 1 : 0;
    hipError_t e = hipSuccess;
    if (chunk_in_future(a.g)) {
        if (!a.accumulate) {
            e = hexi_launch_fill_f32(o, (long long)a.g.lq * a.g.nq * a.g.d, 0.f, s);
            if (e == hipSuccess) e = hexi_launch_fill_f32(lse, (long long)a.g.lq * a.g.nq, -INFINITY, s);
        }
    } else {
        e = desc->dtype == HEXI_F32 ? hexi_launch_fwd_f32(a, s) : hexi_launch_fwd_bf16(a, s);
    }
    if (e != hipSuccess) return fail(HEXI_EHIP, "forward launch failed: %s", hipGetErrorString(e));
    return HEXI_OK;
}

HEXI_EXPORT int hexi_attn_merge_lse(int64_t n_rows, int32_t n_q_heads, int32_t head_dim,
                                   float* o_acc, float* lse_acc, const float* o_part, const float* lse_part,
                                   void* o_final, int32_t o_final_dtype, void* hip_stream)
{
    if (n_rows < 0 || n_q_heads < 1 || head_dim < 4 || head_dim % 4) return fail(HEXI_EINVAL, "bad sizes n_rows=%lld nq=%d d=%d", (long long)n_rows, n_q_heads, head_dim);
    if (n_rows * (int64_t)n_q_heads > 2147483647LL) return fail(HEXI_EUNSUPPORTED, "n_rows * n_q_heads exceeds 2^31-1");
    if (!o_acc || !lse_acc || !o_part || !lse_part) return fail(HEXI_EINVAL, "null tensor pointer");
    if (o_final && o_final_dtype != HEXI_BF16 && o_final_dtype != HEXI_F32) return fail(HEXI_EUNSUPPORTED, "o_final_dtype %d", o_final_dtype);
    if (!aligned16(o_acc) || !aligned16(o_part) || (o_final && !aligned16(o_final))) return fail(HEXI_EALIGN, "o pointers must be 16-byte aligned");
    if (n_rows == 0) return HEXI_OK;
    hipError_t e = hexi_launch_merge(n_rows, n_q_heads, head_dim, o_acc, lse_acc, o_part, lse_part, o_final, o_final_dtype, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(HEXI_EHIP, "merge launch failed: %s", hipGetErrorString(e));
    return HEXI_OK;
}

HEXI_EXPORT int hexi_attn_bwd_chunk(const hexi_attn_desc* desc, const hexi_range* q_range, const hexi_range* kv_range,
                                   const void* q, const void* k, const void* v, const float* o, const void* d_o,
                                   const float* lse, float* delta, float* dq_acc, float* dk, float* dv, uint32_t flags,
                                   void* workspace, size_t workspace_bytes, void* hip_stream)
{
    (void)workspace; (void)workspace_bytes;
    BwdArgs a;
    int rc = build_geom(desc, q_range, kv_range, &a.g);
    if (rc != HEXI_OK) return rc;
    if (flags & ~(HEXI_ACCUMULATE | HEXI_COMPUTE_DELTA | HEXI_SKIP_DQ | HEXI_SKIP_DKDV)) return fail(HEXI_EINVAL, "unknown flag bits 0x%x", flags);
    const bool want_dq = !(flags & HEXI_SKIP_DQ), want_dkdv = !(flags & HEXI_SKIP_DKDV);
    if (!want_dq && !want_dkdv) return fail(HEXI_EINVAL, "HEXI_SKIP_DQ and HEXI_SKIP_DKDV are both set");
    if (!q || !k || !v || !d_o || !lse || !delta || (want_dq && !dq_acc) || (want_dkdv && (!dk || !dv)))
        return fail(HEXI_EINVAL, "null tensor pointer");
    if ((flags & HEXI_COMPUTE_DELTA) && !o) return fail(HEXI_EINVAL, "HEXI_COMPUTE_DELTA needs o");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || (want_dq && !aligned16(dq_acc)) ||
        (want_dkdv && (!aligned16(dk) || !aligned16(dv))) || !aligned16(lse) || !aligned16(delta) ||
        ((flags & HEXI_COMPUTE_DELTA) && !aligned16(o)))
        return fail(HEXI_EALIGN, "tensor base pointers must be 16-byte aligned");
    hipStream_t s = (hipStream_t)hip_stream;
    a.q = q; a.k = k; a.v = v; a.d_o = d_o; a.lse = lse; a.delta = delta; a.dq = dq_acc; a.dk = dk; a.dv = dv;
    a.accumulate = (flags & HEXI_ACCUMULATE) ? 1 : 0;
    a.want_dq = want_dq ? 1 : 0;
    a.want_dkdv = want_dkdv ? 1 : 0;
    hipError_t e = hipSuccess;
    if (flags & HEXI_COMPUTE_DELTA)
        e = hexi_launch_delta(a.g.lq, a.g.nq, a.g.d, o, d_o, desc->dtype, a.g.q_stride_tok, a.g.q_stride_head, delta, s);
    if (e == hipSuccess) {
        if (chunk_in_future(a.g)) {
            if (!a.accumulate && want_dkdv) {
                const long long n = (long long)a.g.lc * a.g.nkv * a.g.d;
                e = hexi_launch_fill_f32(dk, n, 0.f, s);
                if (e == hipSuccess) e = hexi_launch_fill_f32(dv, n, 0.f, s);
            }
        } else {
            e = desc->dtype == HEXI_F32 ? hexi_launch_bwd_f32(a, s) : hexi_launch_bwd_bf16(a, s);
        }
    }
    if (e != hipSuccess) return fail(HEXI_EHIP, "backward launch failed: %s", hipGetErrorString(e));
    return HEXI_OK;
}

static int a2a_call(bool pack, const void* x, void* packed, void* y, int64_t s, int32_t n_heads_total, int32_t head_dim,
                    int32_t elem_bytes, int64_t stride_tok, int32_t n_ranks, const int32_t* heads_per_rank,
                    const int32_t* head_list, void* hip_stream)
{
    if (s < 0 || n_heads_total < 1 || n_heads_total > 65535 || head_dim < 1) return fail(HEXI_EINVAL, "bad sizes s=%lld heads=%d d=%d", (long long)s, n_heads_total, head_dim);
    if (elem_bytes != 2 && elem_bytes != 4) return fail(HEXI_EUNSUPPORTED, "elem_bytes %d", elem_bytes);
    if (n_ranks < 0 || n_ranks > HEXI_A2A_MAX_RANKS || (n_ranks > 0 && !heads_per_rank)) return fail(HEXI_EINVAL, "bad n_ranks %d or null table", n_ranks);
    const int64_t row_bytes = (int64_t)head_dim * elem_bytes;
    if (stride_tok < (int64_t)n_heads_total * head_dim) return fail(HEXI_EINVAL, "token stride %lld smaller than a token", (long long)stride_tok);
    if (row_bytes % 16 || (stride_tok * elem_bytes) % 16 || row_bytes > 65536) return fail(HEXI_EALIGN, "head_dim * elem_bytes and the token stride must be multiples of 16 bytes");
    int n_slots = 0;
    for (int j = 0; j < n_ranks; ++j) {
        if (heads_per_rank[j] < 0) return fail(HEXI_EINVAL, "heads_per_rank[%d] negative", j);
        n_slots += heads_per_rank[j];
        if (n_slots > HEXI_A2A_MAX_SLOTS) return fail(HEXI_EUNSUPPORTED, "more than %d listed heads", HEXI_A2A_MAX_SLOTS);
    }
    if (n_slots > 0 && !head_list) return fail(HEXI_EINVAL, "null head_list");
    std::vector<char> seen(pack ? 0 : n_heads_total, 0);
    for (int i = 0; i < n_slots; ++i) {
        if (head_list[i] < 0 || head_list[i] >= n_heads_total) return fail(HEXI_EINVAL, "head_list[%d] = %d out of range", i, head_list[i]);
        if (!pack) {
            if (seen[head_list[i]]) return fail(HEXI_EINVAL, "head %d listed twice in an unpack", head_list[i]);
            seen[head_list[i]] = true;
        }
    }
    if (s > 0 && n_slots > 0) {
        const void* a = pack ? x : y;
        if (!a || !packed) return fail(HEXI_EINVAL, "null tensor pointer");
        if (!aligned16(a) || !aligned16(packed)) return fail(HEXI_EALIGN, "tensor base pointers must be 16-byte aligned");
    }
    hipError_t e = hexi_launch_a2a(pack, x, packed, y, s, n_heads_total, (int)row_bytes, stride_tok * elem_bytes, n_ranks,
                                   heads_per_rank, head_list, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(HEXI_EHIP, "a2a launch failed: %s", hipGetErrorString(e));
    return HEXI_OK;
}

HEXI_EXPORT int hexi_a2a_pack(const void* x, void* packed, int64_t s, int32_t n_heads_total, int32_t head_dim, int32_t elem_bytes,
                              int64_t x_stride_tok, int32_t n_ranks, const int32_t* heads_per_rank, const int32_t* head_list,
                              void* hip_stream)
{
    return a2a_call(true, x, packed, nullptr, s, n_heads_total, head_dim, elem_bytes, x_stride_tok, n_ranks, heads_per_rank, head_list, hip_stream);
}

HEXI_EXPORT int hexi_a2a_unpack(const void* packed, void* y, int64_t s, int32_t n_heads_total, int32_t head_dim, int32_t elem_bytes,
                                int64_t y_stride_tok, int32_t n_ranks, const int32_t* heads_per_rank, const int32_t* head_list,
                                void* hip_stream)
{
    return a2a_call(false, nullptr, const_cast<void*>(packed), y, s, n_heads_total, head_dim, elem_bytes, y_stride_tok, n_ranks, heads_per_rank, head_list, hip_stream);
}
