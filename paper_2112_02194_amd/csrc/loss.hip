// The objective of the paper's Eq. 3:
//     sum_{(u,i,y)} (y - <w_u,h_i>)^2 + alpha * sum_u sum_i <w_u,h_i>^2 + lambda*(|W|_F^2 + |H|_F^2).
// The observed term is a gather-and-dot over the stored entries; the all-pairs term equals
// <W^T W, H^T H>_F (sum over a,b of G_W[a][b]*G_H[a][b]) and the norms are the Gramians' traces.
// Products are fp32, every sum across entries is fp64, summed in a fixed order.
#include "als_internal.h"

namespace als {

constexpr int LOSS_THREADS = 256;
constexpr int LOSS_MAX_BLOCKS = 2048;

// A group of LPE = D/4 lanes owns one stored entry at a time (each lane 4 columns); a wavefront
// walks the rows assigned to it.
template <int D, bool BF16>
__global__ __launch_bounds__(LOSS_THREADS) void loss_observed_kernel(
    const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices, const float *__restrict__ values,
    int64_t rows, const void *__restrict__ W, int64_t ldw, const void *__restrict__ H, int64_t ldh,
    double *__restrict__ block_sums) {
    constexpr int LPE = D / 4, EPW = 64 / LPE;  // lanes per entry, entries per wave step
    __shared__ double red[LOSS_THREADS / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPE, grp = lane / LPE;
    const int64_t wave_id = (int64_t)blockIdx.x * (LOSS_THREADS / 64) + wave;
    const int64_t nwaves = (int64_t)gridDim.x * (LOSS_THREADS / 64);
    double total = 0.0;
    for (int64_t u = wave_id; u < rows; u += nwaves) {
        const int64_t b = indptr[u], e = indptr[u + 1];
        if (e == b) continue;
        float w[4];
        load_vec<4, BF16>(W, u * ldw + 4 * sub, w);
        for (int64_t p0 = b; p0 < e; p0 += EPW) {
            const int64_t p = p0 + grp;
            float dot = 0.f, y = 0.f;
            if (p < e) {
                float h[4];
                load_vec<4, BF16>(H, (int64_t)indices[p] * ldh + 4 * sub, h);
                dot = w[0] * h[0] + w[1] * h[1] + w[2] * h[2] + w[3] * h[3];
                y = values ? values[p] : 1.f;
            }
#pragma unroll
            for (int off = LPE / 2; off >= 1; off >>= 1) dot += __shfl_xor(dot, off);
            if (p < e && sub == 0) {
                const float r = y - dot;
                total += (double)r * (double)r;
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) total += __shfl_xor(total, off);
    if (lane == 0) red[wave] = total;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int w = 0; w < LOSS_THREADS / 64; ++w) s += red[w];
        block_sums[blockIdx.x] = s;
    }
}

// One workgroup: adds the per-block sums and the Gramian terms in fp64.
__global__ __launch_bounds__(256) void loss_final_kernel(const double *__restrict__ block_sums, int nblocks,
                                                         const float *__restrict__ GW, const float *__restrict__ GH,
                                                         int d, double alpha, double lambda, double *__restrict__ out) {
    __shared__ double red[256];
    double s = 0.0;
    for (int b = threadIdx.x; b < nblocks; b += 256) s += block_sums[b];
    double pairs = 0.0, norms = 0.0;
    for (int e = threadIdx.x; e < d * d; e += 256) {
        pairs += (double)GW[e] * (double)GH[e];
        if (e / d == e % d) norms += (double)GW[e] + (double)GH[e];
    }
    red[threadIdx.x] = s + alpha * pairs + lambda * norms;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = red[0];
}

// Plain device-to-device copy of `bytes` bytes (a multiple of 16): the known-size kernel against
// which hardware traffic counters are calibrated when profiling.
__global__ __launch_bounds__(256) void copy_probe_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst,
                                                         int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

als_status launch_copy_probe(als_ctx *ctx, const void *src, void *dst, int64_t bytes, hipStream_t s) {
    const int64_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)std::min<int64_t>(8192, std::max<int64_t>(1, (n16 + 255) / 256));
    hipLaunchKernelGGL(copy_probe_kernel, dim3(blocks), dim3(256), 0, s, (const float4 *)src, (float4 *)dst, n16);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

template <int D, bool BF16>
static als_status loss_typed(als_ctx *ctx, const als_csr *Y, const als_table *W, const als_table *H,
                             const float *GW, const float *GH, const als_params *prm, double *out_dev,
                             hipStream_t s) {
    int nblocks = (int)std::min<int64_t>(LOSS_MAX_BLOCKS, std::max<int64_t>(1, (Y->rows + 15) / 16));
    als_status st = ensure(ctx, ctx->loss_partials, (size_t)LOSS_MAX_BLOCKS * sizeof(double));
    if (st != ALS_OK) return st;
    hipLaunchKernelGGL((loss_observed_kernel<D, BF16>), dim3(nblocks), dim3(LOSS_THREADS), 0, s, Y->indptr,
                       Y->indices, Y->values, Y->rows, W->data, W->ld, H->data, H->ld,
                       (double *)ctx->loss_partials.p);
    hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(256), 0, s, (const double *)ctx->loss_partials.p, nblocks, GW,
                       GH, (int)D, (double)prm->alpha, (double)prm->lambda, out_dev);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

als_status launch_loss(als_ctx *ctx, const als_csr *Y, const als_table *W, const als_table *H, const float *GW,
                       const float *GH, const als_params *prm, double *out_dev, hipStream_t s) {
    const bool bf = W->dtype == ALS_BF16;
    switch (W->d) {
        case 16: return bf ? loss_typed<16, true>(ctx, Y, W, H, GW, GH, prm, out_dev, s) : loss_typed<16, false>(ctx, Y, W, H, GW, GH, prm, out_dev, s);
        case 32: return bf ? loss_typed<32, true>(ctx, Y, W, H, GW, GH, prm, out_dev, s) : loss_typed<32, false>(ctx, Y, W, H, GW, GH, prm, out_dev, s);
        case 64: return bf ? loss_typed<64, true>(ctx, Y, W, H, GW, GH, prm, out_dev, s) : loss_typed<64, false>(ctx, Y, W, H, GW, GH, prm, out_dev, s);
        case 128: return bf ? loss_typed<128, true>(ctx, Y, W, H, GW, GH, prm, out_dev, s) : loss_typed<128, false>(ctx, Y, W, H, GW, GH, prm, out_dev, s);
    }
    return fail(ctx, ALS_EDTYPE, "unsupported d");
}

}  // namespace als
