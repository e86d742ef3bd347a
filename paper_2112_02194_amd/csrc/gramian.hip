// Gramian G = V^T V of an embedding table (paper Section 3, the remark after Eq. 4; Algorithm 1
// line 2): a tall-skinny contraction over the table's rows on the fp32 matrix cores.
//
// Each wavefront walks a strided set of row groups; a lane fetches NC consecutive columns of one
// row with a single vector load and feeds them as both MFMA operands (see Geo<> for the column
// interleave), accumulating all (d/TM)^2 output tiles in registers.  The four wavefronts of a
// workgroup are summed through LDS in a fixed order, every workgroup writes one fp32 partial
// Gramian, and two further kernels add the partials in fp64 in a fixed order, so the result is
// reproducible bit for bit.  The grid grows with the table so that no fp32 summation chain inside
// the matrix core is longer than GRAM_CHAIN steps: on a 1e8-row table chains of 12 000 steps showed a
// relative error of 1.3e-5 on the diagonal (sums of squares), all of one sign.
#include <mutex>

#include "als_internal.h"

namespace als {

constexpr int GRAM_THREADS = 256;
constexpr int GRAM_CHAIN = 256;         // MFMA steps a wavefront accumulates in fp32
constexpr int GRAM_MAX_BLOCKS = 65536;  // beyond rows = 65536 * 4 * KS * GRAM_CHAIN the chains grow
constexpr int GRAM_SLICES = 64;         // fp64 partial sums of the second stage

template <int D, bool BF16>
__global__ __launch_bounds__(GRAM_THREADS, 2) void gramian_partial_kernel(const void *__restrict__ V, int64_t rows,
                                                                       int64_t ld, float *__restrict__ partials) {
    using G = Geo<D>;
    constexpr int NC = G::NC, TM = G::TM, KS = G::KS, ACC = G::ACC;
    typedef typename AccT<ACC>::type acc_t;
    __shared__ float red[D * D];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane % TM, kk = lane / TM;
    const int64_t wave_id = (int64_t)blockIdx.x * (GRAM_THREADS / 64) + wave;
    const int64_t nwaves = (int64_t)gridDim.x * (GRAM_THREADS / 64);

    acc_t acc[NC][NC];
#pragma unroll
    for (int i = 0; i < NC; ++i)
#pragma unroll
        for (int j = 0; j < NC; ++j)
#pragma unroll
            for (int v = 0; v < ACC; ++v) acc[i][j][v] = 0.f;

    // Rows r0 + kk, r0 advancing by nwaves*KS per MFMA step, in batches of U steps.  The loads of the next
    // batch are issued before the MFMAs of the current one (two register sets used alternately), so that
    // a wavefront always has a batch of rows in flight while the matrix core works.
    constexpr int U = 4;
    const int64_t step = nwaves * KS, batch = step * U;
    auto issue = [&](int64_t r0, float (&x)[U][NC]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t r = r0 + u * step + kk;
            if (r < rows) {
                load_vec<NC, BF16>(V, r * ld + NC * m, x[u]);
            } else {
#pragma unroll
                for (int c = 0; c < NC; ++c) x[u][c] = 0.f;
            }
        }
    };
    auto consume = [&](float (&x)[U][NC]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < NC; ++i)
#pragma unroll
                for (int j = i; j < NC; ++j)  // upper tiles only; the result is symmetric
                    acc[i][j] = mfma<D>(x[u][i], x[u][j], acc[i][j]);
    };
    float xa[U][NC], xb[U][NC];
    int64_t r0 = wave_id * KS;
    issue(r0, xa);
    for (; r0 < rows; r0 += 2 * batch) {
        issue(r0 + batch, xb);  // past the end: zeros, no loads
        consume(xa);
        issue(r0 + 2 * batch, xa);
        if (r0 + batch < rows) consume(xb);
    }

    // fixed-order sum of the four wavefronts through LDS
    for (int w = 0; w < GRAM_THREADS / 64; ++w) {
        if (wave == w) {
#pragma unroll
            for (int i = 0; i < NC; ++i)
#pragma unroll
                for (int j = i; j < NC; ++j)
#pragma unroll
                    for (int v = 0; v < ACC; ++v) {
                        const int r = NC * acc_row<D>(v, lane) + i, c = NC * m + j;
                        if (w == 0) red[r * D + c] = acc[i][j][v];
                        else red[r * D + c] += acc[i][j][v];
                    }
        }
        __syncthreads();
    }
    float *out = partials + (int64_t)blockIdx.x * D * D;
    for (int e = threadIdx.x; e < D * D; e += GRAM_THREADS) {
        const int r = e / D, c = e % D;
        // tile (i,j) with i<=j was computed, where i = r % NC, j = c % NC; otherwise mirror
        const bool have = (r % NC) <= (c % NC);
        out[e] = have ? red[r * D + c] : red[c * D + r];
    }
}

// Stage 2: slice y of gridDim.y adds the partials b = y, y + gridDim.y, ... in fp64.
template <int D>
__global__ __launch_bounds__(256) void gramian_slice_kernel(const float *__restrict__ partials, int nblocks,
                                                            double *__restrict__ slices) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= D * D) return;
    double s = 0.0;
#pragma unroll 4
    for (int b = blockIdx.y; b < nblocks; b += gridDim.y) s += (double)partials[(int64_t)b * D * D + e];
    slices[(int64_t)blockIdx.y * D * D + e] = s;
}

// Stage 3: the slices in order.
template <int D>
__global__ __launch_bounds__(256) void gramian_reduce_kernel(const double *__restrict__ slices, int nslices,
                                                             float *__restrict__ G) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= D * D) return;
    double s = 0.0;
    for (int b = 0; b < nslices; ++b) s += slices[(int64_t)b * D * D + e];
    G[e] = (float)s;
}

template <int D> static int gramian_blocks(int64_t rows) {
    const int64_t per_block = (int64_t)(GRAM_THREADS / 64) * Geo<D>::KS * GRAM_CHAIN;
    return (int)std::min<int64_t>(GRAM_MAX_BLOCKS, std::max<int64_t>(1, (rows + per_block - 1) / per_block));
}

// The three launches; `work` holds nblocks fp32 partials followed by nslices fp64 slices.
template <int D, bool BF16>
static void gramian_enqueue(const als_table *V, float *G, void *work, int nblocks, int nslices, hipStream_t s) {
    float *partials = (float *)work;
    double *slices = (double *)((char *)work + (size_t)nblocks * D * D * sizeof(float));
    hipLaunchKernelGGL((gramian_partial_kernel<D, BF16>), dim3(nblocks), dim3(GRAM_THREADS), 0, s, V->data, V->rows,
                       V->ld, partials);
    hipLaunchKernelGGL((gramian_slice_kernel<D>), dim3((D * D + 255) / 256, nslices), dim3(256), 0, s,
                       (const float *)partials, nblocks, slices);
    hipLaunchKernelGGL((gramian_reduce_kernel<D>), dim3((D * D + 255) / 256), dim3(256), 0, s,
                       (const double *)slices, nslices, G);
}

template <int D, bool BF16>
static als_status gramian_typed(als_ctx *ctx, const als_table *V, float *G, hipStream_t s) {
    const int nblocks = gramian_blocks<D>(V->rows);
    const int nslices = std::min(nblocks, GRAM_SLICES);
    als_status st = ensure(ctx, ctx->gram_partials, (size_t)nblocks * D * D * sizeof(float) +
                                                        (size_t)nslices * D * D * sizeof(double));
    if (st != ALS_OK) return st;
    timer_begin(ctx, T_GRAMIAN, s);
    gramian_enqueue<D, BF16>(V, G, ctx->gram_partials.p, nblocks, nslices, s);
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

als_status launch_gramian(als_ctx *ctx, const als_table *V, float *G, hipStream_t s) {
    const bool bf = V->dtype == ALS_BF16;
    switch (V->d) {
        case 16: return bf ? gramian_typed<16, true>(ctx, V, G, s) : gramian_typed<16, false>(ctx, V, G, s);
        case 32: return bf ? gramian_typed<32, true>(ctx, V, G, s) : gramian_typed<32, false>(ctx, V, G, s);
        case 64: return bf ? gramian_typed<64, true>(ctx, V, G, s) : gramian_typed<64, false>(ctx, V, G, s);
        case 128: return bf ? gramian_typed<128, true>(ctx, V, G, s) : gramian_typed<128, false>(ctx, V, G, s);
    }
    return fail(ctx, ALS_EDTYPE, "unsupported d");
}

// ---------------------------------------------------------------------------------------------- no allocation
// als_gramian_static: the same kernels with their partial sums in a file-scope device array instead of
// the context's workspace, for callers that cannot allocate.  Every GPU holds its own copy of the array
// at its own address; the address is looked up once per device (with that device current) and kept.
// Nothing in the array has to start at zero: every partial and slice that is read has been written by
// the same call.  Calls that overlap on one GPU share the array and race.
constexpr int STATIC_BLOCKS = 128;   // 262 144 rows at d = 128 (2048 rows per workgroup)
constexpr int STATIC_SLICES = 16;
constexpr size_t STATIC_BYTES = (size_t)STATIC_BLOCKS * 128 * 128 * sizeof(float) +
                                (size_t)STATIC_SLICES * 128 * 128 * sizeof(double);
static __device__ __align__(256) unsigned char scratch[STATIC_BYTES];

constexpr int STATIC_MAX_DEVICES = 64;
static void *scratch_ptr[STATIC_MAX_DEVICES];  // per device, null until looked up
static std::mutex scratch_mutex;

// Device address of this GPU's copy of the array; `device` must be current.
hipError_t gramian_static_setup(int device) {
    if (device < 0 || device >= STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_ptr[device]) return hipSuccess;
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    scratch_ptr[device] = p;
    return hipSuccess;
}

template <int D, bool BF16>
static als_status gramian_static_typed(const als_table *V, float *G, void *work, hipStream_t s) {
    const int nblocks = gramian_blocks<D>(V->rows);  // <= STATIC_BLOCKS: the caller has checked the row count
    gramian_enqueue<D, BF16>(V, G, work, nblocks, std::min(nblocks, STATIC_SLICES), s);
    return hipGetLastError() == hipSuccess ? ALS_OK : ALS_EHIP;
}

als_status launch_gramian_static(int device, const als_table *V, float *G, hipStream_t s) {
    if (gramian_static_setup(device) != hipSuccess) return ALS_EHIP;
    void *work = scratch_ptr[device];
    const bool bf = V->dtype == ALS_BF16;
    switch (V->d) {
        case 16: return bf ? gramian_static_typed<16, true>(V, G, work, s) : gramian_static_typed<16, false>(V, G, work, s);
        case 32: return bf ? gramian_static_typed<32, true>(V, G, work, s) : gramian_static_typed<32, false>(V, G, work, s);
        case 64: return bf ? gramian_static_typed<64, true>(V, G, work, s) : gramian_static_typed<64, false>(V, G, work, s);
        case 128: return bf ? gramian_static_typed<128, true>(V, G, work, s) : gramian_static_typed<128, false>(V, G, work, s);
    }
    return ALS_EDTYPE;
}

}  // namespace als
