// als_solve_rows orchestration: classify the rows of the requested range by their number of
// stored entries, then run the kernels each class needs (paper Algorithm 1 lines 3-10; long rows
// are cut into segments in the spirit of Section 4.3).  Nothing here waits for the GPU: the class
// counts stay in device memory, every row kernel walks its list with a grid-stride loop bounded by
// the count it reads there, and grids are sized from the counts of the previous call on the same
// matrix when there was one (a hint: a wrong or missing hint costs speed, never correctness).
#include "als_internal.h"

namespace als {

als_status launch_primal_fused(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                               const als_params *prm, als_table *X, int64_t r0, const int32_t *row_list,
                               const int32_t *count_dev, StepGrid g, hipStream_t s);
als_status launch_primal_long(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                              const als_params *prm, als_table *X, const LongRow *long_rows,
                              const Segment *segs, const int32_t *counters, int64_t seg_capacity, StepGrid g_long,
                              StepGrid g_seg, hipStream_t s);
als_status launch_dual_prepare(als_ctx *ctx, const als_table *V, const float *G, const als_params *prm,
                               hipStream_t s);
als_status launch_dual_rows(als_ctx *ctx, const als_csr *Y, als_table *X, int64_t r0, int64_t r1, int dual_max,
                            const als_params *prm, const int32_t *const lists[10], const int32_t *const counts_dev[10],
                            const int64_t caps[10], const int hints[10], hipStream_t s);
als_status launch_cg_free(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G, const als_params *prm,
                          als_table *X, int64_t r0, const int32_t *const lists[10], const int32_t *const counts_dev[10],
                          const int64_t caps[10], const int hints[10], hipStream_t s);
int dual_supported_max_k(int d);

constexpr int DEFAULT_SPLIT = 512;
constexpr int SEG_CAPACITY = 32768;  // segments whose partial statistics the workspace holds ((d*d + d) floats each)
constexpr int MAX_SEGS_PER_ROW = 128;

StepGrid step_grid(const als_ctx *ctx, int64_t capacity, int64_t hint, int per_cu) {
    StepGrid g = {0u, 0u};
    if (capacity <= 0) return g;
    if (hint > 0) g.known = (unsigned)std::min<int64_t>(hint, capacity);
    g.rest = (unsigned)std::min<int64_t>(capacity - g.known, (int64_t)ctx->num_cu * per_cu);
    return g;
}

__global__ void clear_counters_kernel(int32_t *counters, long long *long_stat) {
    const int t = threadIdx.x;
    if (t < 16 && t != 2 && t != 4) counters[t] = 0;  // [2] is the sticky error flag, [4] the CSR check flag
    if (t < 2) long_stat[t] = 0;
}

constexpr int CLS_THREADS = 256, CLS_RPT = 8, CLS_ROWS = CLS_THREADS * CLS_RPT;  // rows per workgroup
struct ListOffsets { int64_t v[11]; };  // start of each dual class list (and the end of the last), passed by value

// Entries and rows beyond the requested split threshold, summed per workgroup and added with one atomic
// each (integer sums: the order does not matter).
__global__ __launch_bounds__(CLS_THREADS) void long_stat_kernel(const int64_t *__restrict__ indptr, int64_t r0,
                                                               int64_t r1, int64_t split,
                                                               unsigned long long *__restrict__ long_stat) {
    __shared__ unsigned long long red[2][CLS_THREADS / 64];
    unsigned long long ent = 0, cnt = 0;
    const int64_t u0 = r0 + (int64_t)blockIdx.x * CLS_ROWS;
#pragma unroll
    for (int i = 0; i < CLS_RPT; ++i) {
        const int64_t u = u0 + (int64_t)i * CLS_THREADS + threadIdx.x;
        if (u < r1) {
            const int64_t k = indptr[u + 1] - indptr[u];
            if (k > split) {
                ent += (unsigned long long)k;
                cnt += 1;
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        ent += __shfl_xor(ent, off);
        cnt += __shfl_xor(cnt, off);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        red[0][wave] = ent;
        red[1][wave] = cnt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long e = 0, c = 0;
        for (int w = 0; w < CLS_THREADS / 64; ++w) {
            e += red[0][w];
            c += red[1][w];
        }
        if (c) {
            atomicAdd(&long_stat[0], e);
            atomicAdd(&long_stat[1], c);
        }
    }
}

// The split threshold in use: the requested one, raised until the segments of all long rows fit the
// workspace.  With s >= entries_beyond / (SEG_CAPACITY / 2) the rows longer than s number at most
// SEG_CAPACITY / 2 and their segments (each row: at most k/s + 1) at most SEG_CAPACITY.
__global__ void decide_split_kernel(const unsigned long long *__restrict__ long_stat, int64_t split,
                                    int32_t *__restrict__ counters) {
    const unsigned long long need = (long_stat[0] + SEG_CAPACITY / 2 - 1) / (SEG_CAPACITY / 2);
    unsigned long long s = (unsigned long long)split;
    if (need > s) s = need;
    counters[7] = (int32_t)(s > 0x7fffffffull ? 0x7fffffffull : s);
}

// One workgroup per CLS_ROWS consecutive rows of [r0, r1):
//   k = 0               X[u] = 0
//   0 < k <= dual_max   appended to the dual list of its class: k <= 4, 5..8, else ceil(k/16) in 1..8
//                       (row id relative to r0)
//   dual_max < k <= split  appended to the mid list (primal, one workgroup per row)
//   k > split           becomes a long row cut into balanced segments of about `split` entries
//                       (at most MAX_SEGS_PER_ROW of them); split is the threshold decide_split_kernel left
//                       in counters[7]
// List positions are reserved with one atomic per workgroup and list (counts gathered in LDS), and
// rows keep their order inside a workgroup's slice.  A matrix whose indptr does not fit its nnz can ask
// for more long rows or segments than the workspace holds: those are dropped and the error flag is set.
template <bool BF16>
__global__ __launch_bounds__(CLS_THREADS) void classify_kernel(
    const int64_t *__restrict__ indptr, int64_t r0, int64_t r1, int64_t dual_max, int d,
    void *__restrict__ X, int64_t ldx, int32_t *__restrict__ counters, LongRow *__restrict__ long_rows,
    Segment *__restrict__ segs, int32_t *__restrict__ mid_list, int64_t cap_mid, int32_t *__restrict__ dual_lists,
    ListOffsets list_off) {
    __shared__ int32_t cnt[11], base[11];
    const int t = threadIdx.x;
    if (t < 11) cnt[t] = 0;
    __syncthreads();
    const int64_t split = counters[7];
    const int64_t u0 = r0 + (int64_t)blockIdx.x * CLS_ROWS;
    int cls[CLS_RPT], pos[CLS_RPT];
#pragma unroll
    for (int i = 0; i < CLS_RPT; ++i) {
        const int64_t u = u0 + (int64_t)i * CLS_THREADS + t;  // coalesced indptr reads
        cls[i] = -1;
        pos[i] = 0;
        if (u < r1) {
            const int64_t b = indptr[u], e = indptr[u + 1], k = e - b;
            if (k <= 0) {
                for (int c = 0; c < d; ++c) store_elem<BF16>(X, u * ldx + c, 0.f);
            } else if (k > split) {
                int nseg = (int)((k + split - 1) / split);
                if (nseg > MAX_SEGS_PER_ROW) nseg = MAX_SEGS_PER_ROW;
                const int64_t len = (k + nseg - 1) / nseg;
                const int slot = atomicAdd(&counters[0], 1);
                const int first = atomicAdd(&counters[1], nseg);
                if (slot < SEG_CAPACITY / 2 && first + nseg <= SEG_CAPACITY) {
                    long_rows[slot].row = u;
                    long_rows[slot].seg_first = first;
                    long_rows[slot].nseg = nseg;
                    for (int g = 0; g < nseg; ++g) {
                        const int64_t start = b + g * len, stop = b + (g + 1) * len;
                        segs[first + g].begin = start < e ? start : e;
                        segs[first + g].end = stop < e ? stop : e;
                    }
                } else {
                    atomicOr(&counters[2], 2);
                }
            } else {
                // 0 = mid list, 1..8 = dual classes by ceil(k/16), 9 = k <= 4, 10 = 5 <= k <= 8
                cls[i] = k > dual_max ? 0 : (k <= 4 ? 9 : (k <= 8 ? 10 : (int)((k + 15) / 16)));
                pos[i] = atomicAdd(&cnt[cls[i]], 1);
            }
        }
    }
    __syncthreads();
    if (t < 11 && cnt[t] > 0) base[t] = atomicAdd(&counters[t == 0 ? 3 : (t <= 8 ? 8 + t - 1 : t - 4)], cnt[t]);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < CLS_RPT; ++i) {
        if (cls[i] < 0) continue;
        const int32_t rel = (int32_t)(u0 + (int64_t)i * CLS_THREADS + t - r0);
        const int64_t at = (int64_t)base[cls[i]] + pos[i];
        if (cls[i] == 0) {
            if (at < cap_mid) mid_list[at] = rel;
            else atomicOr(&counters[2], 2);
        } else {
            const int c = cls[i] - 1;  // class ids 1..10 -> lists 0..9
            if (at < list_off.v[c + 1] - list_off.v[c]) dual_lists[list_off.v[c] + at] = rel;
            else atomicOr(&counters[2], 2);
        }
    }
}

// Clamp the counts to what was stored (only a matrix inconsistent with its nnz exceeds a capacity) and copy
// them into the host-visible hint slot, sequence number last.
__global__ void publish_counts_kernel(int32_t *__restrict__ counters, int64_t cap_mid, ListOffsets list_off,
                                      int32_t *__restrict__ hint, uint32_t seq) {
    const int t = threadIdx.x;
    if (t == 0) {
        if (counters[2] & 2) {  // something was dropped: no long rows at all rather than half-written ones
            counters[0] = 0;
            counters[1] = 0;
        }
        if (counters[3] > cap_mid) counters[3] = (int32_t)cap_mid;
        for (int c = 0; c < 10; ++c) {
            const int ci = c < 8 ? 8 + c : c - 3;
            const int64_t cap = list_off.v[c + 1] - list_off.v[c];
            if (counters[ci] > cap) counters[ci] = (int32_t)cap;
        }
    }
    __syncthreads();
    if (t < 16) hint[t] = counters[t];
    __threadfence_system();
    __syncthreads();
    if (t == 0) {
        ((volatile int32_t *)hint)[16] = (int32_t)seq;
        __threadfence_system();
    }
}

als_status launch_solve_rows(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                             const als_params *prm_in, als_table *X, int64_t r0, int64_t r1, hipStream_t s) {
    // ALS_SOLVER_CG_FREE: the rows of the class lists never see an assembled system; longer rows take
    // conjugate gradients on their assembled one
    const bool cg_free = prm_in->solver == ALS_SOLVER_CG_FREE;
    als_params prm_rows = *prm_in;
    if (cg_free) prm_rows.solver = ALS_SOLVER_CG;
    const als_params *prm = &prm_rows;
    const int64_t nrows = r1 - r0;
    if (nrows > INT32_MAX) return fail(ctx, ALS_EINVAL, "row range longer than 2^31-1: call per sub-range");
    const int64_t split = prm->split_nnz > 0 ? prm->split_nnz : DEFAULT_SPLIT;
    int dual_max = 0;
    if (prm->path != ALS_PATH_PRIMAL) {
        dual_max = dual_supported_max_k(V->d);
        if (prm->dual_max_k > 0 && prm->dual_max_k < dual_max) dual_max = prm->dual_max_k;
        if (dual_max > split) dual_max = (int)split;
        // conjugate gradients on the k x k systems run in the one-row-per-wavefront kernels, which exist for d >= 64
        if (prm_in->solver == ALS_SOLVER_CG && V->d < 64) dual_max = 0;
    }
    // list capacities: class c (k > 16(c-1)) holds at most nnz/(16(c-1)+1) rows, the mid list at most
    // nnz/(dual_max+1)
    int64_t off[11];  // lists 0..7: classes by ceil(k/16); list 8: k <= 4; list 9: 5 <= k <= 8
    off[0] = 0;
    for (int c = 1; c <= 10; ++c) {
        int64_t cap = 0;
        if (c <= 8) {
            if (dual_max > 16 * (c - 1)) cap = std::min<int64_t>(nrows, Y->nnz / (16 * (c - 1) + 1) + 1);
        } else if (dual_max > 0) {
            cap = std::min<int64_t>(nrows, Y->nnz / (c == 9 ? 1 : 5) + 1);
        }
        off[c] = off[c - 1] + cap;
    }
    const int64_t cap_mid = std::min<int64_t>(nrows, Y->nnz / (dual_max + 1) + 1);
    const size_t off_seg = (size_t)(SEG_CAPACITY / 2) * sizeof(LongRow);
    const size_t off_lists = off_seg + (size_t)SEG_CAPACITY * sizeof(Segment);
    // + 16 bytes: the row kernels read a wavefront's four list entries with one 16-byte load
    als_status st = ensure(ctx, ctx->lists, off_lists + (size_t)(cap_mid + off[10]) * sizeof(int32_t) + 16);
    if (st != ALS_OK) return st;
    LongRow *long_rows = (LongRow *)ctx->lists.p;
    Segment *segs = (Segment *)((char *)ctx->lists.p + off_seg);
    int32_t *mid_list = (int32_t *)((char *)ctx->lists.p + off_lists);
    int32_t *dual_lists = mid_list + cap_mid;
    int32_t *counters = (int32_t *)((char *)ctx->small.p + SM_COUNTERS);
    unsigned long long *long_stat = (unsigned long long *)((char *)ctx->small.p + SM_LONGSTAT);
    ListOffsets list_off;
    for (int c = 0; c <= 10; ++c) list_off.v[c] = off[c];

    // ---- hint slot of this (matrix, range, class shape): counts of the previous such call, if they have arrived
    int slot = -1, lru = 0;
    for (int i = 0; i < N_HINTS; ++i) {
        const HintSlot &h = ctx->hints[i];
        if (h.seq != 0 && h.indptr == (const void *)Y->indptr && h.rows == Y->rows && h.nnz == Y->nnz && h.r0 == r0 &&
            h.r1 == r1 && h.split == (int32_t)split && h.dual_max == dual_max && h.d == V->d)
            slot = i;
        if (ctx->hints[i].seq < ctx->hints[lru].seq) lru = i;
    }
    int hint[16];
    for (int i = 0; i < 16; ++i) hint[i] = -1;
    if (++ctx->hint_seq == 0) ctx->hint_seq = 1;
    if (slot >= 0) {
        // whatever call with this key the GPU has finished last left its counts here (the host may be several
        // calls ahead of the GPU: the hint need not come from the call just before this one)
        const volatile int32_t *hc = ctx->hint_counts + (size_t)slot * HINT_INTS;
        const uint32_t stamp = (uint32_t)hc[16];
        if (stamp != 0 && stamp - ctx->hints[slot].first_seq < 0x80000000u)
            for (int i = 0; i < 16; ++i) hint[i] = hc[i];
    } else {
        slot = lru;
        ctx->hints[slot].first_seq = ctx->hint_seq;
    }
    HintSlot &hs = ctx->hints[slot];
    hs.indptr = Y->indptr; hs.rows = Y->rows; hs.nnz = Y->nnz; hs.r0 = r0; hs.r1 = r1;
    hs.split = (int32_t)split; hs.dual_max = dual_max; hs.d = V->d;
    hs.seq = ctx->hint_seq;

    timer_begin(ctx, T_CLASSIFY, s);
    hipLaunchKernelGGL(clear_counters_kernel, dim3(1), dim3(64), 0, s, counters, (long long *)long_stat);
    const unsigned cblocks = (unsigned)((nrows + CLS_ROWS - 1) / CLS_ROWS);
    hipLaunchKernelGGL(long_stat_kernel, dim3(cblocks), dim3(CLS_THREADS), 0, s, Y->indptr, r0, r1, split, long_stat);
    hipLaunchKernelGGL(decide_split_kernel, dim3(1), dim3(1), 0, s, (const unsigned long long *)long_stat, split,
                       counters);
    if (V->dtype == ALS_BF16)
        hipLaunchKernelGGL(classify_kernel<true>, dim3(cblocks), dim3(CLS_THREADS), 0, s, Y->indptr, r0, r1,
                           (int64_t)dual_max, V->d, X->data, X->ld, counters, long_rows, segs, mid_list, cap_mid,
                           dual_lists, list_off);
    else
        hipLaunchKernelGGL(classify_kernel<false>, dim3(cblocks), dim3(CLS_THREADS), 0, s, Y->indptr, r0, r1,
                           (int64_t)dual_max, V->d, X->data, X->ld, counters, long_rows, segs, mid_list, cap_mid,
                           dual_lists, list_off);
    hipLaunchKernelGGL(publish_counts_kernel, dim3(1), dim3(64), 0, s, counters, cap_mid, list_off,
                       ctx->hint_counts_dev + (size_t)slot * HINT_INTS, hs.seq);
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());

    if (dual_max > 0 && !cg_free) {
        if ((st = launch_dual_prepare(ctx, V, G, prm, s)) != ALS_OK) return st;
    }
    // segments: at most 2 nnz / split + 1 of them exist, and never more than the workspace holds
    const int64_t seg_capacity = std::min<int64_t>(SEG_CAPACITY, 2 * (Y->nnz / split) + 2);
    const StepGrid g_long = step_grid(ctx, std::min<int64_t>(SEG_CAPACITY / 2, Y->nnz / split + 1), hint[0], 4);
    const StepGrid g_seg = step_grid(ctx, seg_capacity, hint[1], 8);
    if ((st = launch_primal_long(ctx, Y, V, G, prm, X, long_rows, segs, counters, seg_capacity, g_long, g_seg, s)) != ALS_OK)
        return st;
    if ((st = launch_primal_fused(ctx, Y, V, G, prm, X, r0, mid_list, counters + 3, step_grid(ctx, cap_mid, hint[3], 8),
                                  s)) != ALS_OK)
        return st;
    if (dual_max > 0) {
        const int32_t *lists[10], *counts_dev[10];
        int64_t caps[10];
        int hints[10];
        for (int c = 0; c < 10; ++c) {
            lists[c] = dual_lists + off[c];
            const int ci = c < 8 ? 8 + c : c - 3;  // counters [5], [6]: the two small classes
            counts_dev[c] = counters + ci;
            caps[c] = off[c + 1] - off[c];
            hints[c] = hint[ci];
        }
        st = cg_free ? launch_cg_free(ctx, Y, V, G, prm, X, r0, lists, counts_dev, caps, hints, s)
                     : launch_dual_rows(ctx, Y, X, r0, r1, dual_max, prm, lists, counts_dev, caps, hints, s);
        if (st != ALS_OK) return st;
    }
    return ALS_OK;
}

// ---------------------------------------------------------------------------------------------- validation
__global__ __launch_bounds__(256) void check_csr_kernel(const int64_t *__restrict__ indptr,
                                                        const int32_t *__restrict__ indices, int64_t rows,
                                                        int64_t cols, int64_t nnz, int32_t *__restrict__ flag) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    bool bad = false;
    if (t == 0) bad = indptr[0] != 0 || indptr[rows] != nnz;
    for (int64_t u = t; u < rows; u += stride) bad |= indptr[u + 1] < indptr[u];
    for (int64_t p = t; p < nnz; p += stride) bad |= indices[p] < 0 || indices[p] >= cols;
    if (bad) atomicOr(flag, 1);
}

als_status launch_check_csr(als_ctx *ctx, const als_csr *Y, int32_t *flag_dev, hipStream_t s) {
    int64_t work = std::max<int64_t>(Y->rows, Y->nnz);
    unsigned blocks = (unsigned)std::min<int64_t>(4096, std::max<int64_t>(1, (work + 255) / 256));
    hipLaunchKernelGGL(check_csr_kernel, dim3(blocks), dim3(256), 0, s, Y->indptr, Y->indices, Y->rows, Y->cols,
                       Y->nnz, flag_dev);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

}  // namespace als
