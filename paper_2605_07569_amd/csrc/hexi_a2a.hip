// Head redistribution either side of the ring (HexiSeq Sec. 3.2, "Heterogeneous A2A with per-rank split
// tables", "Sub-ring KV exchange": non-contiguous head slices are packed into contiguous buffers): gather
// x[s][N][d] into one contiguous [s][n_j][d] part per destination rank, and the inverse scatter.  Pure data
// movement, HBM-bound: every 16-byte piece is read once and written once.
#include "hexi_internal.h"

namespace {

typedef unsigned int u4 __attribute__((ext_vector_type(4)));   // one 16-byte piece

// One slot per (rank, head of that rank's list), in send-buffer order.
struct A2ATable {
    int n_slots;
    unsigned short head[HEXI_A2A_MAX_SLOTS];        // head index in x
    unsigned short n_j[HEXI_A2A_MAX_SLOTS];         // heads of the slot's rank
    unsigned short local[HEXI_A2A_MAX_SLOTS];       // index of the head within its rank's list
    unsigned short heads_before[HEXI_A2A_MAX_SLOTS];   // heads of all earlier ranks
};

constexpr int TOKENS_PER_BLOCK = 16;

// A block moves TOKENS_PER_BLOCK tokens x all slots.  A token is n_slots rows of cpr 16-byte pieces; a thread
// owns fixed pieces of the token (piece p = thread + 256 m: slot p / cpr, piece p % cpr of the row), looks its
// slot up once, and then walks the block's tokens: from one token to the next the x address advances by the
// token stride and the packed address by the rank's n_j rows.  Consecutive threads take consecutive pieces of
// a row, then consecutive slots, so both sides are accessed in runs of whole rows (the packed side in runs of a
// whole rank's heads).
template <bool PACK>
__global__ void __launch_bounds__(256) a2a_kernel(const A2ATable tb, const u4* __restrict__ x, u4* __restrict__ packed, u4* __restrict__ y,
                                                  const long long s, const int cpr, const long long x_stride_pieces)
{
    const long long t0 = (long long)blockIdx.x * TOKENS_PER_BLOCK;
    const int n_tok = (int)(s - t0 < TOKENS_PER_BLOCK ? s - t0 : TOKENS_PER_BLOCK);
    const unsigned per_token = (unsigned)tb.n_slots * (unsigned)cpr;
    constexpr int UNROLL = 8;
    for (unsigned p = threadIdx.x; p < per_token; p += 256) {
        const unsigned slot = p / (unsigned)cpr, c = p - slot * (unsigned)cpr;
        const long long n_j = tb.n_j[slot];
        long long in_x = t0 * x_stride_pieces + (long long)tb.head[slot] * cpr + c;
        long long in_p = (((long long)tb.heads_before[slot] * s + t0 * n_j) + tb.local[slot]) * cpr + c;
        const long long step_p = n_j * cpr;
        for (int tl = 0; tl < n_tok; tl += UNROLL) {
            u4 val[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (tl + u < n_tok) val[u] = __builtin_nontemporal_load(PACK ? &x[in_x + u * x_stride_pieces] : &packed[in_p + u * step_p]);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (tl + u < n_tok) {
                    if (PACK) __builtin_nontemporal_store(val[u], &packed[in_p + u * step_p]);
                    else __builtin_nontemporal_store(val[u], &y[in_x + u * x_stride_pieces]);
                }
            in_x += UNROLL * x_stride_pieces;
            in_p += UNROLL * step_p;
        }
    }
}

}  // namespace

hipError_t hexi_launch_a2a(bool pack, const void* x, void* packed, void* y, long long s, int n_heads_total, int row_bytes,
                           long long x_stride_bytes, int n_ranks, const int* heads_per_rank, const int* head_list, hipStream_t st)
{
    A2ATable tb;
    int slot = 0, before = 0;
    for (int j = 0; j < n_ranks; ++j) {
        for (int i = 0; i < heads_per_rank[j]; ++i, ++slot) {
            tb.head[slot] = (unsigned short)head_list[slot];
            tb.n_j[slot] = (unsigned short)heads_per_rank[j];
            tb.local[slot] = (unsigned short)i;
            tb.heads_before[slot] = (unsigned short)before;
        }
        before += heads_per_rank[j];
    }
    tb.n_slots = slot;
    if (slot == 0 || s == 0) return hipSuccess;
    const unsigned grid = (unsigned)((s + TOKENS_PER_BLOCK - 1) / TOKENS_PER_BLOCK);
    if (pack)
        a2a_kernel<true><<<grid, 256, 0, st>>>(tb, static_cast<const u4*>(x), static_cast<u4*>(packed), nullptr, s, row_bytes / 16,
                                               x_stride_bytes / 16);
    else
        a2a_kernel<false><<<grid, 256, 0, st>>>(tb, nullptr, static_cast<u4*>(packed), static_cast<u4*>(y), s, row_bytes / 16,
                                                x_stride_bytes / 16);
    return hipGetLastError();
}
