// als_solve_rows orchestration: classify the rows of the requested range by their number of
// stored entries, then run the kernels each class needs (paper Algorithm 1 lines 3-10; long rows
// are cut into segments in the spirit of Section 4.3).
#include "als_internal.h"

namespace als {

als_status launch_primal_fused(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                               const als_params *prm, als_table *X, int64_t r0, const int64_t *row_list,
                               int64_t nitems, int64_t k_lo, int64_t k_hi, hipStream_t s);
als_status launch_primal_long(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                              const als_params *prm, als_table *X, const LongRow *long_rows, int n_long,
                              const Segment *segs, int n_seg, hipStream_t s);
als_status launch_dual(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G, const als_params *prm,
                       als_table *X, int64_t r0, int64_t r1, int dual_max_k, hipStream_t s);
int dual_supported_max_k(int d);

constexpr int DEFAULT_SPLIT = 2048;

__global__ void clear_counters_kernel(int32_t *counters) {
    if (threadIdx.x < 2) counters[threadIdx.x] = 0;
    if (threadIdx.x == 3) counters[3] = 0;
}

// One thread per row of [r0, r1): empty rows get X[u] = 0; rows with k > split become a long row
// with ceil(k/split) balanced segments; rows with mid_lo < k <= split are appended to mid_list.
template <bool BF16>
__global__ __launch_bounds__(256) void classify_kernel(const int64_t *__restrict__ indptr, int64_t r0, int64_t r1,
                                                       int64_t split, int64_t mid_lo, int d, void *__restrict__ X,
                                                       int64_t ldx, int32_t *__restrict__ counters,
                                                       LongRow *__restrict__ long_rows, Segment *__restrict__ segs,
                                                       int64_t *__restrict__ mid_list) {
    const int64_t u = r0 + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (u >= r1) return;
    const int64_t b = indptr[u], e = indptr[u + 1], k = e - b;
    if (k <= 0) {
        for (int c = 0; c < d; ++c) store_elem<BF16>(X, u * ldx + c, 0.f);
        return;
    }
    if (k > split) {
        const int nseg = (int)((k + split - 1) / split);
        const int64_t len = (k + nseg - 1) / nseg;
        const int slot = atomicAdd(&counters[0], 1);
        const int first = atomicAdd(&counters[1], nseg);
        long_rows[slot].row = u;
        long_rows[slot].seg_first = first;
        long_rows[slot].nseg = nseg;
        for (int g = 0; g < nseg; ++g) {
            segs[first + g].begin = b + g * len;
            const int64_t stop = b + (g + 1) * len;
            segs[first + g].end = stop < e ? stop : e;
        }
    } else if (mid_list && k > mid_lo) {
        const int slot = atomicAdd(&counters[3], 1);
        mid_list[slot] = u;
    }
}

als_status launch_solve_rows(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                             const als_params *prm, als_table *X, int64_t r0, int64_t r1, hipStream_t s) {
    const int64_t nrows = r1 - r0;
    const int64_t split = prm->split_nnz > 0 ? prm->split_nnz : DEFAULT_SPLIT;
    int dual_max = 0;
    if (prm->path != ALS_PATH_PRIMAL) {
        dual_max = dual_supported_max_k(V->d);
        if (prm->dual_max_k > 0 && prm->dual_max_k < dual_max) dual_max = prm->dual_max_k;
        if (dual_max > split) dual_max = (int)split;
    }
    // capacities: rows longer than split number at most nnz/split, their segments at most twice that
    const int64_t cap_long = Y->nnz / split + 1, cap_seg = 2 * (Y->nnz / split) + 2;
    const int64_t cap_mid = dual_max > 0 ? Y->nnz / (dual_max + 1) + 1 : 0;
    if (cap_seg > INT32_MAX) return fail(ctx, ALS_EINVAL, "split_nnz too small for this matrix");
    const size_t off_seg = (size_t)cap_long * sizeof(LongRow);
    const size_t off_mid = off_seg + (size_t)cap_seg * sizeof(Segment);
    als_status st = ensure(ctx, ctx->lists, off_mid + (size_t)cap_mid * sizeof(int64_t));
    if (st != ALS_OK) return st;
    LongRow *long_rows = (LongRow *)ctx->lists.p;
    Segment *segs = (Segment *)((char *)ctx->lists.p + off_seg);
    int64_t *mid_list = dual_max > 0 ? (int64_t *)((char *)ctx->lists.p + off_mid) : nullptr;
    int32_t *counters = (int32_t *)((char *)ctx->small.p + SM_COUNTERS);

    // Short rows first: the dual kernels need nothing from the classification, and their closing
    // table transform passes over every row of the range, so the classifier (which zeroes the empty
    // rows) and the primal kernels must come after it.
    if (dual_max > 0) {
        if ((st = launch_dual(ctx, Y, V, G, prm, X, r0, r1, dual_max, s)) != ALS_OK) return st;
    }
    timer_begin(ctx, T_CLASSIFY, s);
    hipLaunchKernelGGL(clear_counters_kernel, dim3(1), dim3(64), 0, s, counters);
    const unsigned cblocks = (unsigned)((nrows + 255) / 256);
    if (V->dtype == ALS_BF16)
        hipLaunchKernelGGL(classify_kernel<true>, dim3(cblocks), dim3(256), 0, s, Y->indptr, r0, r1, split,
                           (int64_t)dual_max, V->d, X->data, X->ld, counters, long_rows, segs, mid_list);
    else
        hipLaunchKernelGGL(classify_kernel<false>, dim3(cblocks), dim3(256), 0, s, Y->indptr, r0, r1, split,
                           (int64_t)dual_max, V->d, X->data, X->ld, counters, long_rows, segs, mid_list);
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());
    ALS_HIP(ctx, hipMemcpyAsync(ctx->host_counters, counters, 4 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    ALS_HIP(ctx, hipStreamSynchronize(s));
    const int n_long = ctx->host_counters[0], n_seg = ctx->host_counters[1], n_mid = ctx->host_counters[3];
    if (n_long > cap_long || n_seg > cap_seg || n_mid > cap_mid)
        return fail(ctx, ALS_EINVAL, "CSR structure inconsistent with nnz (run als_check_csr)");

    if (dual_max > 0) {
        st = launch_primal_fused(ctx, Y, V, G, prm, X, r0, mid_list, n_mid, dual_max, split, s);
    } else {
        st = launch_primal_fused(ctx, Y, V, G, prm, X, r0, nullptr, nrows, 0, split, s);
    }
    if (st != ALS_OK) return st;
    return launch_primal_long(ctx, Y, V, G, prm, X, long_rows, n_long, segs, n_seg, s);
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
