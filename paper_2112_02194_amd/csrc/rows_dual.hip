// Dual (k x k) form of the row update of the paper's Eq. 4 for rows with few stored entries.
//
// With B = alpha*G + lambda*I = L L^T (one shared d x d factorisation per half-epoch) and
// z_i = L^{-1} v_i, the normal equations of a row with entries I (|I| = k) become
//     A = B + V_I^T V_I = L (I_d + Z_I^T Z_I) L^T ,
// and the push-through identity (I_d + Z^T Z)^{-1} Z^T = Z^T (I_k + Z Z^T)^{-1} gives
//     x_u = A^{-1} V_I^T y = L^{-T} Z_I^T t ,   (I_k + Z_I Z_I^T) t = y .
// This is the same minimiser of Eq. 3 as the d x d system (exact algebra, no approximation), but
// costs O(k^2 d + k^3) per row instead of O(k d^2 + d^3), and the k x k matrix has eigenvalues in
// [1, 1 + k/alpha], so fp32 is comfortable.  Steps:
//   factor_kernel     B -> L^{-1} in fp64 (one workgroup), stored fp32
//   transform_kernel  Z = V L^{-T}   (fp32 MFMA, table-sized workspace)
//   dual_wave_kernel  one wavefront per row: gather Z_I straight into MFMA operand registers,
//                     S = I + Z_I Z_I^T on the matrix cores, Cholesky + two triangular solves with
//                     one lane per row of S, r = Z_I^T t by a cross-lane reduction
//   transform_kernel  X = R L^{-1}   (rows r -> L^{-T} r), rounding to the table's element type
#include "als_internal.h"

namespace als {

// ---------------------------------------------------------------------------------------------- factor
// One workgroup.  a (fp64, LDS): entry (r,c) at a[c*LD + r].  Outputs Linv (row-major, zeros above
// the diagonal) and its transpose LinvT, both fp32 [D*D].
template <int D>
__global__ __launch_bounds__(256) void factor_kernel(const float *__restrict__ G, float alpha, float lambda,
                                                     float *__restrict__ Linv, float *__restrict__ LinvT,
                                                     int32_t *__restrict__ err_flag) {
    constexpr int LD = D + 1, T = 256;
    extern __shared__ double fa[];
    double *a = fa, *col = fa + D * LD;
    const int t = threadIdx.x, tx = t & 31, ty = t >> 5;
    for (int e = t; e < D * D; e += T) {
        const int r = e / D, c = e % D;
        a[c * LD + r] = (double)alpha * (double)G[e] + (r == c ? (double)lambda : 0.0);
    }
    __syncthreads();
    for (int k = 0; k < D; ++k) {
        const double pivot = a[k * LD + k];
        if (t == 0 && !(pivot > 0.0)) atomicOr(err_flag, 1);
        const double rinv = 1.0 / sqrt(pivot);
        __syncthreads();
        for (int i = k + t; i < D; i += T) a[k * LD + i] = (i == k) ? sqrt(pivot) : a[k * LD + i] * rinv;
        __syncthreads();
        for (int j = k + 1 + ty; j < D; j += T / 32) {
            const double cj = a[k * LD + j];
            for (int i = j + tx; i < D; i += 32) a[j * LD + i] -= a[k * LD + i] * cj;
        }
        __syncthreads();
    }
    // in-place inverse of the lower triangle, last column first:
    //   inv[j][j] = 1/L[j][j];  inv[i][j] = -( sum_{p=j+1..i} inv[i][p] * L[p][j] ) * inv[j][j]   (i > j)
    for (int j = D - 1; j >= 0; --j) {
        for (int i = j + t; i < D; i += T) col[i] = a[j * LD + i];
        __syncthreads();
        const double dj = 1.0 / col[j];
        for (int i = j + t; i < D; i += T) {
            double s = 0.0;
            for (int p = j + 1; p <= i; ++p) s += a[p * LD + i] * col[p];
            a[j * LD + i] = (i == j) ? dj : -s * dj;
        }
        __syncthreads();
    }
    for (int e = t; e < D * D; e += T) {
        const int r = e / D, c = e % D;
        const float v = r >= c ? (float)a[c * LD + r] : 0.f;
        Linv[r * D + c] = v;
        LinvT[c * D + r] = v;
    }
}

// ---------------------------------------------------------------------------------------------- transform
// Out[r][:] = In[r][:] * M for rows r in [r0, r1), M fp32 [D x D] row-major.  In may be bf16 or
// fp32, Out fp32 or bf16; Out may be the same buffer as In (a workgroup reads its whole row tile
// into LDS before it writes).  Wavefront w owns output column tile w % NCT for the row sub-tiles
// of its group and keeps its slice of M in registers.
template <int D, bool IN_BF16, bool OUT_BF16>
__global__ __launch_bounds__(256) void transform_kernel(const void *__restrict__ In, int64_t ldi,
                                                        void *__restrict__ Out, int64_t ldo,
                                                        const float *__restrict__ M, int64_t r0, int64_t r1) {
    using GE = Geo<D>;
    constexpr int TM = GE::TM, KS = GE::KS, ACC = GE::ACC;
    constexpr int NCT = D / TM, RG = 4 / NCT, RT = 64, NSUB = RT / TM, LD = D + 1, NS = D / KS;
    typedef typename AccT<ACC>::type acc_t;
    __shared__ float At[RT * LD];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane % TM, kq = lane / TM;
    const int J = wave % NCT, rg = wave / NCT;
    float breg[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) breg[s] = M[(KS * s + kq) * D + TM * J + m];

    const int64_t ntiles = (r1 - r0 + RT - 1) / RT;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t base = r0 + tile * RT;
        __syncthreads();  // previous tile's operand reads are done
        for (int e = threadIdx.x; e < RT * (D / 4); e += 256) {
            const int row = e / (D / 4), c4 = e % (D / 4);
            float x[4] = {0.f, 0.f, 0.f, 0.f};
            if (base + row < r1) load_vec<4, IN_BF16>(In, (base + row) * ldi + 4 * c4, x);
#pragma unroll
            for (int c = 0; c < 4; ++c) At[row * LD + 4 * c4 + c] = x[c];
        }
        __syncthreads();
        for (int sub = rg; sub < NSUB; sub += RG) {
            acc_t acc;
#pragma unroll
            for (int v = 0; v < ACC; ++v) acc[v] = 0.f;
#pragma unroll
            for (int s = 0; s < NS; ++s) acc = mfma<D>(At[(sub * TM + m) * LD + KS * s + kq], breg[s], acc);
#pragma unroll
            for (int v = 0; v < ACC; ++v) {
                const int64_t r = base + sub * TM + acc_row<D>(v, lane);
                if (r < r1) store_elem<OUT_BF16>(Out, r * ldo + TM * J + m, acc[v]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------- dual rows
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float readlane_f(float v, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

// x + (x rotated by N lanes inside each row of 16 lanes)
template <int N> __device__ __forceinline__ float add_row_ror(float x) {
    const int r = __builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x120 + N, 0xf, 0xf, false);
    return x + __int_as_float(r);
}

// One wavefront per row u with k_lo < k <= k_hi <= 16*KT stored entries.
//   lane (a = lane%16, q = lane/16) loads, for entry e = 16*t + a and j < D/16, the four columns
//   (4j+q)*4.. of z_e; the same register is the A and the B operand of v_mfma_f32_16x16x4, so tile
//   (t1,t2) accumulates S[16*t1 + .][16*t2 + .] over all d columns.
//   sbuf (LDS, per wavefront): K x (K+1) floats.
template <int D, int KT>
__global__ __launch_bounds__(256) void dual_wave_kernel(const int64_t *__restrict__ indptr,
                                                        const int32_t *__restrict__ indices,
                                                        const float *__restrict__ values,
                                                        const float *__restrict__ Z, float *__restrict__ R,
                                                        int64_t ldr, int64_t r0, int64_t r1, int k_lo, int k_hi) {
    constexpr int K = 16 * KT, KP = K + 1, NJ = D / 16;
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *sbuf = lds + wave * K * KP;
    const int64_t u = r0 + (int64_t)blockIdx.x * 4 + wave;
    if (u >= r1) return;  // no workgroup barrier below: wavefronts are independent
    const int64_t b = indptr[u];
    const int k = (int)(indptr[u + 1] - b);
    if (k <= k_lo || k > k_hi) return;
    const int a = lane & 15, q = lane >> 4;

    float4 z[KT][NJ];
#pragma unroll
    for (int t = 0; t < KT; ++t) {
        const int e = 16 * t + a;
        const int64_t idx = e < k ? (int64_t)indices[b + e] : -1;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (idx >= 0) z[t][j] = *(const float4 *)(Z + idx * D + (4 * j + q) * 4);
            else z[t][j] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    float yv = 0.f;  // lane e holds the label of entry e
    if (lane < k) yv = values ? values[b + lane] : 1.f;

    floatx4 acc[KT][KT];
#pragma unroll
    for (int t1 = 0; t1 < KT; ++t1)
#pragma unroll
        for (int t2 = 0; t2 <= t1; ++t2) acc[t1][t2] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int t1 = 0; t1 < KT; ++t1)
#pragma unroll
            for (int t2 = 0; t2 <= t1; ++t2) {
                acc[t1][t2] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[t1][j].x, z[t2][j].x, acc[t1][t2], 0, 0, 0);
                acc[t1][t2] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[t1][j].y, z[t2][j].y, acc[t1][t2], 0, 0, 0);
                acc[t1][t2] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[t1][j].z, z[t2][j].z, acc[t1][t2], 0, 0, 0);
                acc[t1][t2] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[t1][j].w, z[t2][j].w, acc[t1][t2], 0, 0, 0);
            }
    // S = I + Z_I Z_I^T into LDS (lower block triangle; diagonal tiles in full)
#pragma unroll
    for (int t1 = 0; t1 < KT; ++t1)
#pragma unroll
        for (int t2 = 0; t2 <= t1; ++t2)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * t1 + 4 * q + v, jc = 16 * t2 + a;
                sbuf[i * KP + jc] = acc[t1][t2][v] + (i == jc ? 1.f : 0.f);
            }
    wave_sync();
    // lane i owns row i of S; entries right of the diagonal are never used
    const int myrow = lane < K ? lane : K - 1;
    float s[K];
#pragma unroll
    for (int c = 0; c < K; ++c) s[c] = sbuf[myrow * KP + c];
    wave_sync();
    // right-looking Cholesky, one column per step; lane i ends with L[i][c] in s[c] (c <= i)
    float myrinv = 1.f;
#pragma unroll
    for (int c = 0; c < K; ++c) {
        if (c < k) {
            const float pivot = readlane_f(s[c], c);
            const float rinv = 1.0f / sqrtf(pivot);
            const float lc = s[c] * rinv;
            s[c] = lc;
            myrinv = lane == c ? rinv : myrinv;
#pragma unroll
            for (int i = c + 1; i < K; ++i) s[i] -= lc * readlane_f(lc, i);
        }
    }
    // L w = y (lane i ends with w_i); rows beyond k are identity rows with zero right-hand side
#pragma unroll
    for (int c = 0; c < K; ++c) {
        if (c < k) {
            const float wc = readlane_f(yv, c) * readlane_f(myrinv, c);
            yv = lane > c ? yv - s[c] * wc : (lane == c ? wc : yv);
        }
    }
    // L^T t = w: lane i needs column i of L, read back transposed through LDS
#pragma unroll
    for (int c = 0; c < K; ++c) sbuf[myrow * KP + c] = s[c];
    wave_sync();
#pragma unroll
    for (int c = K - 1; c >= 0; --c) {
        if (c < k) {
            const float tc = readlane_f(yv, c) * readlane_f(myrinv, c);
            const float lt = sbuf[c * KP + myrow];  // L[c][lane], meaningful for lane <= c
            yv = lane < c ? yv - lt * tc : (lane == c ? tc : yv);
        }
    }
    // r = Z_I^T t: scale this lane's pieces by t_e, add over the tiles, then over the 16 lanes a
    float4 rp[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) rp[j] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int t = 0; t < KT; ++t) {
        const float te = __shfl(yv, 16 * t + a);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            rp[j].x += te * z[t][j].x; rp[j].y += te * z[t][j].y;
            rp[j].z += te * z[t][j].z; rp[j].w += te * z[t][j].w;
        }
    }
    float4 out = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        float4 v = rp[j];
        v.x = add_row_ror<8>(v.x); v.y = add_row_ror<8>(v.y); v.z = add_row_ror<8>(v.z); v.w = add_row_ror<8>(v.w);
        v.x = add_row_ror<4>(v.x); v.y = add_row_ror<4>(v.y); v.z = add_row_ror<4>(v.z); v.w = add_row_ror<4>(v.w);
        v.x = add_row_ror<2>(v.x); v.y = add_row_ror<2>(v.y); v.z = add_row_ror<2>(v.z); v.w = add_row_ror<2>(v.w);
        v.x = add_row_ror<1>(v.x); v.y = add_row_ror<1>(v.y); v.z = add_row_ror<1>(v.z); v.w = add_row_ror<1>(v.w);
        out = (a == j) ? v : out;
    }
    if (a < NJ) *(float4 *)(R + u * ldr + (4 * a + q) * 4) = out;
}

// ---------------------------------------------------------------------------------------------- launchers
int dual_supported_max_k(int d) { return d < 64 ? d : 64; }

template <int D, int KT>
static void launch_dual_class(const als_csr *Y, const float *Z, float *R, int64_t ldr, int64_t r0, int64_t r1,
                              int dual_max, hipStream_t s) {
    const int k_lo = 16 * (KT - 1), k_hi = std::min(16 * KT, dual_max);
    if (k_hi <= k_lo) return;
    constexpr size_t lds = 4 * (16 * KT) * (16 * KT + 1) * sizeof(float);
    const unsigned blocks = (unsigned)((r1 - r0 + 3) / 4);
    hipLaunchKernelGGL((dual_wave_kernel<D, KT>), dim3(blocks), dim3(256), lds, s, Y->indptr, Y->indices, Y->values, Z,
                       R, ldr, r0, r1, k_lo, k_hi);
}

template <int D, bool BF16>
static als_status dual_typed(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                             const als_params *prm, als_table *X, int64_t r0, int64_t r1, int dual_max,
                             hipStream_t s) {
    als_status st = ensure(ctx, ctx->ztable, (size_t)V->rows * D * sizeof(float));
    if (st != ALS_OK) return st;
    float *R = (float *)X->data;
    int64_t ldr = X->ld;
    if (BF16) {
        st = ensure(ctx, ctx->rtable, (size_t)(r1 - r0) * D * sizeof(float));
        if (st != ALS_OK) return st;
        R = (float *)ctx->rtable.p - r0 * D;  // row u lives at rtable[(u - r0) * D]
        ldr = D;
    }
    float *Linv = (float *)((char *)ctx->small.p + SM_FACTOR), *LinvT = Linv + 128 * 128;
    int32_t *err = (int32_t *)((char *)ctx->small.p + SM_COUNTERS) + 2;
    float *Z = (float *)ctx->ztable.p;
    constexpr size_t factor_lds = (size_t)(D * (D + 1) + D) * sizeof(double);
    ALS_HIP(ctx, hipFuncSetAttribute((const void *)factor_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)factor_lds));
    timer_begin(ctx, T_TRANSFORM, s);
    hipLaunchKernelGGL(factor_kernel<D>, dim3(1), dim3(256), factor_lds, s, G, prm->alpha, prm->lambda, Linv, LinvT,
                       err);
    const unsigned tblocks = (unsigned)std::min<int64_t>(2048, std::max<int64_t>(1, (V->rows + 63) / 64));
    hipLaunchKernelGGL((transform_kernel<D, BF16, false>), dim3(tblocks), dim3(256), 0, s, V->data, V->ld, (void *)Z,
                       (int64_t)D, (const float *)LinvT, (int64_t)0, V->rows);
    timer_end(ctx, s);
    timer_begin(ctx, T_DUAL, s);
    launch_dual_class<D, 1>(Y, Z, R, ldr, r0, r1, dual_max, s);
    launch_dual_class<D, 2>(Y, Z, R, ldr, r0, r1, dual_max, s);
    launch_dual_class<D, 3>(Y, Z, R, ldr, r0, r1, dual_max, s);
    launch_dual_class<D, 4>(Y, Z, R, ldr, r0, r1, dual_max, s);
    timer_end(ctx, s);
    timer_begin(ctx, T_TRANSFORM, s);
    const unsigned xblocks = (unsigned)std::min<int64_t>(2048, std::max<int64_t>(1, (r1 - r0 + 63) / 64));
    hipLaunchKernelGGL((transform_kernel<D, false, BF16>), dim3(xblocks), dim3(256), 0, s, (const void *)R, ldr,
                       X->data, X->ld, (const float *)Linv, r0, r1);
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

als_status launch_dual(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G, const als_params *prm,
                       als_table *X, int64_t r0, int64_t r1, int dual_max, hipStream_t s) {
    const bool bf = V->dtype == ALS_BF16;
    switch (V->d) {
        case 16: return bf ? dual_typed<16, true>(ctx, Y, V, G, prm, X, r0, r1, dual_max, s) : dual_typed<16, false>(ctx, Y, V, G, prm, X, r0, r1, dual_max, s);
        case 32: return bf ? dual_typed<32, true>(ctx, Y, V, G, prm, X, r0, r1, dual_max, s) : dual_typed<32, false>(ctx, Y, V, G, prm, X, r0, r1, dual_max, s);
        case 64: return bf ? dual_typed<64, true>(ctx, Y, V, G, prm, X, r0, r1, dual_max, s) : dual_typed<64, false>(ctx, Y, V, G, prm, X, r0, r1, dual_max, s);
        case 128: return bf ? dual_typed<128, true>(ctx, Y, V, G, prm, X, r0, r1, dual_max, s) : dual_typed<128, false>(ctx, Y, V, G, prm, X, r0, r1, dual_max, s);
    }
    return fail(ctx, ALS_EDTYPE, "unsupported d");
}

}  // namespace als
