// als_solve_rows orchestration: classify the rows of the requested range by their number of
// stored entries, then run the kernels each class needs (paper Algorithm 1 lines 3-10; long rows
// are cut into segments in the spirit of Section 4.3).
#include "als_internal.h"

namespace als {

als_status launch_primal_fused(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                               const als_params *prm, als_table *X, int64_t r0, const int32_t *row_list,
                               int64_t nitems, hipStream_t s);
als_status launch_primal_long(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                              const als_params *prm, als_table *X, const LongRow *long_rows, int n_long,
                              const Segment *segs, int n_seg, hipStream_t s);
als_status launch_dual_prepare(als_ctx *ctx, const als_table *V, const float *G, const als_params *prm,
                               hipStream_t s);
als_status launch_dual_rows(als_ctx *ctx, const als_csr *Y, als_table *X, int64_t r0, int64_t r1, int dual_max,
                            const int32_t *const lists[10], const int counts[10], hipStream_t s);
int dual_supported_max_k(int d);

constexpr int DEFAULT_SPLIT = 512;

__global__ void clear_counters_kernel(int32_t *counters) {
    const int t = threadIdx.x;
    if (t < 16 && t != 2 && t != 4) counters[t] = 0;  // [2] is the sticky error flag, [4] the CSR check flag
}

constexpr int CLS_THREADS = 256, CLS_RPT = 8, CLS_ROWS = CLS_THREADS * CLS_RPT;  // rows per workgroup
constexpr int MAX_SEGS_PER_ROW = 128;
struct ListOffsets { int64_t v[10]; };  // start of each dual class list, passed by value

// One workgroup per CLS_ROWS consecutive rows of [r0, r1):
//   k = 0               X[u] = 0
//   0 < k <= dual_max   appended to the dual list of its class: k <= 4, 5..8, else ceil(k/16) in 1..8
//                       (row id relative to r0)
//   dual_max < k <= split  appended to the mid list (primal, one workgroup per row)
//   k > split           becomes a long row cut into balanced segments of about `split` entries
//                       (at most MAX_SEGS_PER_ROW of them)
// List positions are reserved with one atomic per workgroup and list (counts gathered in LDS), and
// rows keep their order inside a workgroup's slice.
template <bool BF16>
__global__ __launch_bounds__(CLS_THREADS) void classify_kernel(
    const int64_t *__restrict__ indptr, int64_t r0, int64_t r1, int64_t split, int64_t dual_max, int d,
    void *__restrict__ X, int64_t ldx, int32_t *__restrict__ counters, LongRow *__restrict__ long_rows,
    Segment *__restrict__ segs, int32_t *__restrict__ mid_list, int32_t *__restrict__ dual_lists,
    ListOffsets list_off) {
    __shared__ int32_t cnt[11], base[11];
    const int t = threadIdx.x;
    if (t < 11) cnt[t] = 0;
    __syncthreads();
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
                long_rows[slot].row = u;
                long_rows[slot].seg_first = first;
                long_rows[slot].nseg = nseg;
                for (int g = 0; g < nseg; ++g) {
                    const int64_t start = b + g * len, stop = b + (g + 1) * len;
                    segs[first + g].begin = start < e ? start : e;
                    segs[first + g].end = stop < e ? stop : e;
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
        int32_t *list = cls[i] == 0 ? mid_list : dual_lists + list_off.v[cls[i] - 1];  // class ids 1..10 -> lists 0..9
        list[base[cls[i]] + pos[i]] = rel;
    }
}

als_status launch_solve_rows(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                             const als_params *prm, als_table *X, int64_t r0, int64_t r1, hipStream_t s) {
    const int64_t nrows = r1 - r0;
    if (nrows > INT32_MAX) return fail(ctx, ALS_EINVAL, "row range longer than 2^31-1: call per sub-range");
    const int64_t split = prm->split_nnz > 0 ? prm->split_nnz : DEFAULT_SPLIT;
    int dual_max = 0;
    if (prm->path != ALS_PATH_PRIMAL) {
        dual_max = dual_supported_max_k(V->d);
        if (prm->dual_max_k > 0 && prm->dual_max_k < dual_max) dual_max = prm->dual_max_k;
        if (dual_max > split) dual_max = (int)split;
    }
    // capacities: rows longer than split number at most nnz/split, their segments at most twice that
    const int64_t cap_long = Y->nnz / split + 1, cap_seg = 2 * (Y->nnz / split) + 2;
    if (cap_seg > INT32_MAX) return fail(ctx, ALS_EINVAL, "split_nnz too small for this matrix");
    // list capacities: class c (k > 16(c-1)) holds at most nnz/(16(c-1)+1) rows, the mid list at most
    // nnz/(dual_max+1); offsets go to the device through a small table in the context's scratch
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
    const size_t off_seg = (size_t)cap_long * sizeof(LongRow);
    const size_t off_lists = off_seg + (size_t)cap_seg * sizeof(Segment);
    // + 16 bytes: the row kernels read a wavefront's four list entries with one 16-byte load
    als_status st = ensure(ctx, ctx->lists, off_lists + (size_t)(cap_mid + off[10]) * sizeof(int32_t) + 16);
    if (st != ALS_OK) return st;
    LongRow *long_rows = (LongRow *)ctx->lists.p;
    Segment *segs = (Segment *)((char *)ctx->lists.p + off_seg);
    int32_t *mid_list = (int32_t *)((char *)ctx->lists.p + off_lists);
    int32_t *dual_lists = mid_list + cap_mid;
    int32_t *counters = (int32_t *)((char *)ctx->small.p + SM_COUNTERS);
    ListOffsets list_off;
    for (int c = 0; c < 10; ++c) list_off.v[c] = off[c];

    timer_begin(ctx, T_CLASSIFY, s);
    hipLaunchKernelGGL(clear_counters_kernel, dim3(1), dim3(64), 0, s, counters);
    const unsigned cblocks = (unsigned)((nrows + CLS_ROWS - 1) / CLS_ROWS);
    if (V->dtype == ALS_BF16)
        hipLaunchKernelGGL(classify_kernel<true>, dim3(cblocks), dim3(CLS_THREADS), 0, s, Y->indptr, r0, r1, split,
                           (int64_t)dual_max, V->d, X->data, X->ld, counters, long_rows, segs, mid_list, dual_lists,
                           list_off);
    else
        hipLaunchKernelGGL(classify_kernel<false>, dim3(cblocks), dim3(CLS_THREADS), 0, s, Y->indptr, r0, r1, split,
                           (int64_t)dual_max, V->d, X->data, X->ld, counters, long_rows, segs, mid_list, dual_lists,
                           list_off);
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());
    ALS_HIP(ctx, hipMemcpyAsync(ctx->host_counters, counters, 16 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    // the shared factorisation and the table transform need no counts: enqueue them before waiting
    if (dual_max > 0) {
        if ((st = launch_dual_prepare(ctx, V, G, prm, s)) != ALS_OK) return st;
    }
    ALS_HIP(ctx, hipStreamSynchronize(s));
    const int n_long = ctx->host_counters[0], n_seg = ctx->host_counters[1], n_mid = ctx->host_counters[3];
    if (n_long > cap_long || n_seg > cap_seg)
        return fail(ctx, ALS_EINVAL, "CSR structure inconsistent with nnz (run als_check_csr)");

    // From here on the work of the row classes is independent (disjoint output rows): the primal and
    // long-row kernels go to side stream 2 while the dual classes use the caller's stream and side
    // streams 0 and 1; everything is joined back into the caller's stream before returning.
    const bool side = ctx->use_side_streams;
    if (side && (st = side_fork(ctx, s)) != ALS_OK) return st;
    hipStream_t s_primal = side ? ctx->side[2] : s;
    if ((st = launch_primal_long(ctx, Y, V, G, prm, X, long_rows, n_long, segs, n_seg, s_primal)) != ALS_OK) return st;
    if ((st = launch_primal_fused(ctx, Y, V, G, prm, X, r0, mid_list, n_mid, s_primal)) != ALS_OK) return st;
    if (dual_max > 0) {
        const int32_t *lists[10];
        int counts[10];
        for (int c = 0; c < 10; ++c) {
            lists[c] = dual_lists + off[c];
            counts[c] = ctx->host_counters[c < 8 ? 8 + c : c - 3];  // [5], [6]: the two small classes
        }
        if ((st = launch_dual_rows(ctx, Y, X, r0, r1, dual_max, lists, counts, s)) != ALS_OK) return st;
    }
    if (side && (st = side_join(ctx, 2, s)) != ALS_OK) return st;
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
