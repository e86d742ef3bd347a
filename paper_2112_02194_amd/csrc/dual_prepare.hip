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
//   row kernels       by class of k (fixed by measurement on MI355X): all gather Z_I straight into MFMA
//                     operand registers, form S = I + Z_I Z_I^T on the matrix cores, solve the k x k
//                     system on the vector ALU, then r = Z_I^T t
//       dual_small_kernel  k <= 4 and 5 <= k <= 8: several rows share one 16-entry MFMA tile
//       dual_rows_kernel   8 < k <= 16: four rows per wavefront, one lane per row of S, DPP broadcasts
//       dual_multi_kernel  16 < k <= 32: four rows per wavefront, two rows of S per lane, DPP only
//       dual_wide_kernel   32 < k <= 128 (d >= 64; k <= 64 at d = 64): one row per wavefront, S as a
//                          lower triangle in LDS, blocked elimination with MFMA trailing updates
//   transform_kernel  X = R L^{-1}   (rows r -> L^{-T} r), rounding to the table's element type
#include "dual_common.h"

namespace als {

void launch_dual_small4(int d, const als_csr *Y, const void *Z, bool zb16, float *R, int64_t ldr, int64_t r0,
                        const int32_t *list, const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s);
void launch_dual_small8(int d, const als_csr *Y, const void *Z, bool zb16, float *R, int64_t ldr, int64_t r0,
                        const int32_t *list, const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s);
void launch_dual_multi2(int d, const als_csr *Y, const void *Z, bool zb16, float *R, int64_t ldr, int64_t r0,
                        const int32_t *list, const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s);
#define ALS_DECL_WIDE(kt)                                                                                          \
    als_status launch_dual_wide##kt(als_ctx *ctx, int d, const als_csr *Y, const void *Z, bool zb16, float *R,     \
                                    int64_t ldr, int64_t r0, const int32_t *list, const int32_t *count_dev,        \
                                    StepGrid g, int32_t *err, const WideSolver &ws, hipStream_t s);
ALS_DECL_WIDE(3) ALS_DECL_WIDE(4) ALS_DECL_WIDE(5) ALS_DECL_WIDE(6) ALS_DECL_WIDE(7) ALS_DECL_WIDE(8)
#undef ALS_DECL_WIDE

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
// Out[r][:] = In[r][:] * M for rows r in [r0, r1) (only rows with 0 < k <= k_max stored entries when
// indptr is given), M fp32 [D x D] row-major and triangular: UPPER = true means M[j][c] = 0 for j > c
// (M = L^{-T}), UPPER = false means M[j][c] = 0 for j < c (M = L^{-1}).  In may be bf16 or fp32, Out
// fp32 or bf16; Out may be the same buffer as In (a wavefront reads its rows completely before it
// writes them, and no other wavefront touches them).
//
// A wavefront owns TM table rows at a time and all D output columns.  Lane (m, kq) streams along row
// m: for the contraction block kb (TM input columns) it holds the BW = TM/KS consecutive columns
// TM*kb + BW*kq .. of its row, loaded straight from global memory as 16-byte pieces; step i of the
// block contracts column TM*kb + BW*kq + i (A and B operands only have to agree on that mapping).
// The transposed matrix sits in LDS (one copy per workgroup, MT[c][j], padded rows) and supplies the
// B operands; blocks that only meet zeros of the triangular matrix are skipped.
template <int D> struct XfCfg {
    using GE = Geo<D>;
    static constexpr int TM = GE::TM, KS = GE::KS, NB = D / TM, BW = TM / KS, MLD = D + 4;
    static constexpr size_t LDS_BYTES = (size_t)D * MLD * sizeof(float);
};

template <int D, bool IN_BF16, bool OUT_BF16, bool UPPER>
__global__ __launch_bounds__(256) void transform_kernel(const void *In, int64_t ldi, void *Out, int64_t ldo,
                                                        const float *__restrict__ M, int64_t r0, int64_t r1,
                                                        const int64_t *__restrict__ indptr, int64_t k_max) {
    using C = XfCfg<D>;
    constexpr int TM = C::TM, NB = C::NB, BW = C::BW, MLD = C::MLD, ACC = Geo<D>::ACC;
    typedef typename AccT<ACC>::type acc_t;
    extern __shared__ float MT[];  // MT[c * MLD + j] = M[j][c]
    for (int e = threadIdx.x; e < D * D; e += 256) {
        const int j = e / D, c = e % D;
        MT[c * MLD + j] = M[e];
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane % TM, kq = lane / TM;
    const int64_t ntiles = (r1 - r0 + TM - 1) / TM;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < ntiles; tile += nwaves) {
        const int64_t base = r0 + tile * TM, row = base + m;
        float a[NB][BW];
#pragma unroll
        for (int kb = 0; kb < NB; ++kb)
#pragma unroll
            for (int i4 = 0; i4 < BW / 4; ++i4) {
                float x[4] = {0.f, 0.f, 0.f, 0.f};
                if (row < r1) load_vec<4, IN_BF16>(In, row * ldi + TM * kb + BW * kq + 4 * i4, x);
#pragma unroll
                for (int c = 0; c < 4; ++c) a[kb][4 * i4 + c] = x[c];
            }
        // which of this lane's ACC output rows are written (only rows solved in the dual form)
        bool keep[ACC];
#pragma unroll
        for (int v = 0; v < ACC; ++v) {
            const int64_t r = base + acc_row<D>(v, lane);
            keep[v] = r < r1;
            if (keep[v] && indptr) {
                const int64_t k = indptr[r + 1] - indptr[r];
                keep[v] = k > 0 && k <= k_max;
            }
        }
#pragma unroll
        for (int J = 0; J < NB; ++J) {
            acc_t acc;
#pragma unroll
            for (int v = 0; v < ACC; ++v) acc[v] = 0.f;
#pragma unroll
            for (int kb = 0; kb < NB; ++kb) {
                if (UPPER ? (kb <= J) : (kb >= J)) {  // compile-time after unrolling
                    const float *bp = MT + (TM * J + m) * MLD + TM * kb + BW * kq;
#pragma unroll
                    for (int i4 = 0; i4 < BW / 4; ++i4) {
                        const float4 b = *(const float4 *)(bp + 4 * i4);
                        acc = mfma<D>(a[kb][4 * i4 + 0], b.x, acc);
                        acc = mfma<D>(a[kb][4 * i4 + 1], b.y, acc);
                        acc = mfma<D>(a[kb][4 * i4 + 2], b.z, acc);
                        acc = mfma<D>(a[kb][4 * i4 + 3], b.w, acc);
                    }
                }
            }
            // acc[v] = Out[base + acc_row(v)][TM*J + m]
#pragma unroll
            for (int v = 0; v < ACC; ++v)
                if (keep[v]) store_elem<OUT_BF16>(Out, (base + acc_row<D>(v, lane)) * ldo + TM * J + m, acc[v]);
            __builtin_amdgcn_sched_barrier(0);  // keep the next column tile's operand reads from piling up
        }
    }
}

// ---------------------------------------------------------------------------------------------- transform, bf16 output
// The same product for bf16 tables (d >= 32), where both passes write bf16 (Z and X): on the bf16 matrix cores,
// which turns the pass from matrix-core-bound (fp32 instruction) into HBM-bound.  M is cut once per workgroup
// into hi = bf16(M) and lo = bf16(M - hi) (LDS, transposed); bf16 input rows are exact operands (two products
// per step: x hi + x lo), fp32 input rows (the dual solutions R) are cut the same way (three products,
// dropping lo lo).  The error of the cut, 2^-17 relative, is far below the bf16 rounding of the output.
// The roles of the operands are swapped against transform_kernel: the matrix supplies the M dimension
// (output columns) and the table rows the N dimension, so that a lane ends up with 16 consecutive output
// columns of ONE table row (the output columns are assigned to the instruction's row index in the order
// that makes them consecutive) and stores them as two 16-byte pieces.
template <int D> struct Xf16Cfg {
    static constexpr int MLD = D + 8;  // bf16 elements per LDS row (rows stay 16-byte aligned)
    static constexpr size_t LDS_BYTES = (size_t)2 * D * MLD * sizeof(uint16_t);
};

template <int D, bool IN_BF16, bool UPPER>
__global__ __launch_bounds__(256, 2) void transform16_kernel(const void *__restrict__ In, int64_t ldi,
                                                          uint16_t *__restrict__ Out, int64_t ldo,
                                                          const float *__restrict__ M, int64_t r0, int64_t r1,
                                                          const int64_t *__restrict__ indptr, int64_t k_max) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    constexpr int MLD = Xf16Cfg<D>::MLD, NKB = D / 16, NJB = D / 32;
    extern __shared__ uint16_t mt[];  // hi: mt[c * MLD + j] = bf16(M[j][c]); lo: the same at offset D * MLD
    auto rne = [](float x, float y) { return __builtin_bit_cast(uint32_t, __builtin_convertvector((floatx2){x, y}, bf16x2)); };
    for (int e = threadIdx.x; e < D * D; e += 256) {
        const int j = e / D, c = e % D;
        const float v = M[e];
        const uint32_t h = rne(v, 0.f) & 0xffffu;
        mt[c * MLD + j] = (uint16_t)h;
        mt[D * MLD + c * MLD + j] = (uint16_t)(rne(v - __uint_as_float(h << 16), 0.f) & 0xffffu);
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, kq = lane >> 5;
    // output column (inside a block of 32) that this lane supplies as row n of the matrix operand
    const int pi = 16 * ((n >> 2) & 1) + 4 * (n >> 3) + (n & 3);
    const int64_t ntiles = (r1 - r0 + 31) / 32;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < ntiles; tile += nwaves) {
        const int64_t row = r0 + tile * 32 + n;
        bool keep = row < r1;
        if (keep && indptr) {  // only rows solved in the dual form are written
            const int64_t k = indptr[row + 1] - indptr[row];
            keep = k > 0 && k <= k_max;
        }
        // this lane's share of its row: columns 16 kb + 8 kq .., as bf16 operands (hi and, for fp32 input, lo)
        bf16x8 xh[NKB], xl[IN_BF16 ? 1 : NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            if constexpr (IN_BF16) {
                u32x4 w = {0u, 0u, 0u, 0u};
                if (row < r1) w = *(const u32x4 *)((const uint16_t *)In + row * ldi + 16 * kb + 8 * kq);
                xh[kb] = __builtin_bit_cast(bf16x8, w);
            } else {
                float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                if (row < r1) {
                    const float4 p = *(const float4 *)((const float *)In + row * ldi + 16 * kb + 8 * kq);
                    const float4 q4 = *(const float4 *)((const float *)In + row * ldi + 16 * kb + 8 * kq + 4);
                    x[0] = p.x; x[1] = p.y; x[2] = p.z; x[3] = p.w; x[4] = q4.x; x[5] = q4.y; x[6] = q4.z; x[7] = q4.w;
                }
                u32x4 h, l;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    h[w] = rne(x[2 * w], x[2 * w + 1]);
                    l[w] = rne(x[2 * w] - __uint_as_float(h[w] << 16), x[2 * w + 1] - __uint_as_float(h[w] & 0xffff0000u));
                }
                xh[kb] = __builtin_bit_cast(bf16x8, h);
                xl[kb] = __builtin_bit_cast(bf16x8, l);
            }
        }
#pragma unroll
        for (int J = 0; J < NJB; ++J) {
            floatx16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            const uint16_t *mrow = mt + (32 * J + pi) * MLD + 8 * kq;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                if (UPPER ? (kb <= 2 * J + 1) : (kb >= 2 * J)) {  // compile-time after unrolling: other steps only meet zeros
                    const bf16x8 mh = *(const bf16x8 *)(mrow + 16 * kb), ml = *(const bf16x8 *)(mrow + D * MLD + 16 * kb);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(mh, xh[kb], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ml, xh[kb], acc, 0, 0, 0);
                    if constexpr (!IN_BF16) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(mh, xl[kb], acc, 0, 0, 0);
                }
            }
            // acc[v] = Out[row][32 J + 16 kq + v]
            if (keep) {
                u32x4 lo4, hi4;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    lo4[w] = rne(acc[2 * w], acc[2 * w + 1]);
                    hi4[w] = rne(acc[8 + 2 * w], acc[8 + 2 * w + 1]);
                }
                u32x4 *dst = (u32x4 *)(Out + row * ldo + 32 * J + 16 * kq);
                dst[0] = lo4;
                dst[1] = hi4;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------- transform, fp32 tables
// fp32 in, fp32 out (d >= 64), with fp32 accuracy on the bf16 matrix cores: the matrix (once per workgroup, LDS)
// and the table rows (registers) are cut exactly into three bf16 parts each, x = x0 + x1 + x2 with x0 = upper
// 16 bits of x and so on, and a product keeps the six terms m0 x0, m0 x1, m1 x0, m0 x2, m2 x0, m1 x1 (what is
// dropped is below the rounding of an fp32 product): 0.375 of the fp32 instruction's matrix-core time, which
// leaves the pass to the table read and write (used for X = R L^-1: 24.5 against 29.0 ms per epoch on the 50M-row
// configuration; for Z = V L^-T the fp32 kernel above measured faster, 24.4 against 25.9 ms).  The matrix core's running sum is not rounded to nearest, so
// only the six products of one 16-column step are summed there, from zero and small terms first; the steps are
// summed on the vector units.  Operand roles and the store layout are those of transform16_kernel.  All of a
// tile's input is in registers before its first store, so In == Out is fine.
constexpr int XFS_THREADS = 512;
template <int D> struct XfsCfg {
    static constexpr int MLD = D + 8;  // bf16 elements per LDS row
    static constexpr size_t LDS_BYTES = (size_t)3 * D * MLD * sizeof(uint16_t);
};

template <int D, bool UPPER>
__global__ __launch_bounds__(XFS_THREADS, 2) void transform_split_kernel(const float *In, int64_t ldi, float *Out,
                                                                         int64_t ldo, const float *__restrict__ M,
                                                                         int64_t r0, int64_t r1,
                                                                         const int64_t *__restrict__ indptr, int64_t k_max) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr int MLD = XfsCfg<D>::MLD, NKB = D / 16, NJB = D / 32;
    extern __shared__ uint16_t mt[];  // part t: mt[t * D * MLD + c * MLD + j] = part t of M[j][c]
    auto rest = [](float x) { return x - __uint_as_float(__float_as_uint(x) & 0xffff0000u); };
    for (int e = threadIdx.x; e < D * D; e += XFS_THREADS) {
        const int j = e / D, c = e % D;
        float v = M[e];
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            mt[t * D * MLD + c * MLD + j] = (uint16_t)(__float_as_uint(v) >> 16);
            v = rest(v);
        }
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, kq = lane >> 5;
    const int pi = 16 * ((n >> 2) & 1) + 4 * (n >> 3) + (n & 3);  // see transform16_kernel
    const int64_t ntiles = (r1 - r0 + 31) / 32;
    const int64_t nwaves = (int64_t)gridDim.x * (XFS_THREADS / 64);
    for (int64_t tile = (int64_t)blockIdx.x * (XFS_THREADS / 64) + wave; tile < ntiles; tile += nwaves) {
        const int64_t row = r0 + tile * 32 + n;
        bool keep = row < r1;
        if (keep && indptr) {  // only rows solved in the dual form are written
            const int64_t k = indptr[row + 1] - indptr[row];
            keep = k > 0 && k <= k_max;
        }
        // this lane's share of its row: columns 16 kb + 8 kq .., as three bf16 operands each
        bf16x8 xp[3][NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (row < r1) {
                const float4 p = *(const float4 *)(In + row * ldi + 16 * kb + 8 * kq);
                const float4 q4 = *(const float4 *)(In + row * ldi + 16 * kb + 8 * kq + 4);
                x[0] = p.x; x[1] = p.y; x[2] = p.z; x[3] = p.w; x[4] = q4.x; x[5] = q4.y; x[6] = q4.z; x[7] = q4.w;
            }
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                u32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = pack_upper(x[2 * e], x[2 * e + 1]);
                xp[t][kb] = __builtin_bit_cast(bf16x8, w);
                if (t < 2) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[e] = rest(x[e]);
                }
            }
        }
#pragma unroll
        for (int J = 0; J < NJB; ++J) {
            floatx16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            const uint16_t *mrow = mt + (32 * J + pi) * MLD + 8 * kq;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                if (UPPER ? (kb <= 2 * J + 1) : (kb >= 2 * J)) {  // compile-time after unrolling: other steps only meet zeros
                    const bf16x8 m0 = *(const bf16x8 *)(mrow + 16 * kb), m1 = *(const bf16x8 *)(mrow + D * MLD + 16 * kb),
                                 m2 = *(const bf16x8 *)(mrow + 2 * D * MLD + 16 * kb);
                    floatx16 t16;
#pragma unroll
                    for (int v = 0; v < 16; ++v) t16[v] = 0.f;
                    t16 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(m1, xp[1][kb], t16, 0, 0, 0);  // small terms first
                    t16 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(m2, xp[0][kb], t16, 0, 0, 0);
                    t16 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(m0, xp[2][kb], t16, 0, 0, 0);
                    t16 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(m1, xp[0][kb], t16, 0, 0, 0);
                    t16 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(m0, xp[1][kb], t16, 0, 0, 0);
                    t16 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(m0, xp[0][kb], t16, 0, 0, 0);
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[v] += t16[v];
                }
            }
            // acc[v] = Out[row][32 J + 16 kq + v]
            if (keep) {
                float4 *dst = (float4 *)(Out + row * ldo + 32 * J + 16 * kq);
#pragma unroll
                for (int w = 0; w < 4; ++w) dst[w] = make_float4(acc[4 * w], acc[4 * w + 1], acc[4 * w + 2], acc[4 * w + 3]);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the next column block's operand reads from piling up
        }
    }
}

// ---------------------------------------------------------------------------------------------- launchers
int dual_supported_max_k(int d) { return d < 128 ? (d < 64 ? d : 64) : 128; }

// bf16 tables with d >= 32: Z is stored as bf16 too (one more rounding, to the tables' own element type, of a
// table that is only ever used to solve rows whose result is rounded to bf16 anyway; half the gather
// traffic, and a row piece is a matrix-core operand as loaded).  At d = 16 a row is shorter than one
// 32-column matrix-core step and Z stays fp32.
template <int D, bool BF16> constexpr bool z_is_bf16() { return BF16 && D >= 32; }

// Part 1 (needs no row classification): factorise B and build Z = V L^{-T}.
template <int D, bool BF16>
static als_status dual_prepare_typed(als_ctx *ctx, const als_table *V, const float *G, const als_params *prm,
                                     hipStream_t s) {
    constexpr bool ZB = z_is_bf16<D, BF16>();
    als_status st = ensure(ctx, ctx->ztable, (size_t)V->rows * D * (ZB ? 2 : 4));
    if (st != ALS_OK) return st;
    float *Linv = (float *)((char *)ctx->small.p + SM_FACTOR), *LinvT = Linv + 128 * 128;
    int32_t *err = (int32_t *)((char *)ctx->small.p + SM_COUNTERS) + 2;
    constexpr size_t factor_lds = (size_t)(D * (D + 1) + D) * sizeof(double);
    static const hipError_t attr_f = hipFuncSetAttribute((const void *)factor_kernel<D>,
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)factor_lds);
    ALS_HIP(ctx, attr_f);
    timer_begin(ctx, T_TRANSFORM, s);
    hipLaunchKernelGGL(factor_kernel<D>, dim3(1), dim3(256), factor_lds, s, G, prm->alpha, prm->lambda, Linv, LinvT,
                       err);
    const unsigned tblocks = (unsigned)std::min<int64_t>(1024, std::max<int64_t>(1, (V->rows + 127) / 128));
    if constexpr (ZB) {
        static const hipError_t attr_t = hipFuncSetAttribute((const void *)transform16_kernel<D, true, true>,
                                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                                             (int)Xf16Cfg<D>::LDS_BYTES);  // once per process
        ALS_HIP(ctx, attr_t);
        hipLaunchKernelGGL((transform16_kernel<D, true, true>), dim3(tblocks), dim3(256), Xf16Cfg<D>::LDS_BYTES, s, V->data,
                           V->ld, (uint16_t *)ctx->ztable.p, (int64_t)D, (const float *)LinvT, (int64_t)0, V->rows,
                           (const int64_t *)nullptr, (int64_t)0);
    } else {
        static const hipError_t attr_t = hipFuncSetAttribute((const void *)transform_kernel<D, BF16, false, true>,
                                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                                             (int)XfCfg<D>::LDS_BYTES);  // once per process
        ALS_HIP(ctx, attr_t);
        hipLaunchKernelGGL((transform_kernel<D, BF16, false, true>), dim3(tblocks), dim3(256), XfCfg<D>::LDS_BYTES, s,
                           V->data, V->ld, ctx->ztable.p, (int64_t)D, (const float *)LinvT, (int64_t)0, V->rows,
                           (const int64_t *)nullptr, (int64_t)0);
    }
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

// Part 2: the row kernels of the k-classes, then X = R L^{-1} on the rows they solved.  Every class is
// launched (its kernel finds the length of its list in device memory); `caps` bounds the lists, `hints` holds
// the lengths seen by the previous call on the same matrix, or -1.
template <int D, bool BF16>
static als_status dual_rows_typed(als_ctx *ctx, const als_csr *Y, als_table *X, int64_t r0, int64_t r1,
                                  int dual_max, const als_params *prm, const int32_t *const lists[10],
                                  const int32_t *const counts_dev[10], const int64_t caps[10], const int hints[10],
                                  hipStream_t s) {
    float *R = (float *)X->data;
    int64_t ldr = X->ld;
    if (BF16) {
        als_status st = ensure(ctx, ctx->rtable, (size_t)(r1 - r0) * D * sizeof(float));
        if (st != ALS_OK) return st;
        R = (float *)ctx->rtable.p - r0 * D;  // row u lives at rtable[(u - r0) * D]
        ldr = D;
    }
    const float *Linv = (const float *)((char *)ctx->small.p + SM_FACTOR);
    int32_t *err = (int32_t *)((char *)ctx->small.p + SM_COUNTERS) + 2;
    const void *Z = ctx->ztable.p;
    constexpr bool zb16 = z_is_bf16<D, BF16>();
    als_status stb = ALS_OK;
    // workgroups of class `cls` whose kernel takes `rpw` rows per step
    auto grid = [&](int cls, int rpw) {
        const int64_t cap = (caps[cls] + rpw - 1) / rpw;
        const int64_t hint = hints[cls] < 0 ? -1 : ((int64_t)hints[cls] + rpw - 1) / rpw;
        return step_grid(ctx, cap, hint, 32);
    };
#define ALS_TIMED_CLASS(slot, cls, rpw, call)           \
    if (caps[cls] > 0 && stb == ALS_OK) {               \
        const StepGrid g = grid(cls, rpw);              \
        timer_begin(ctx, slot, s);                      \
        call;                                           \
        timer_end(ctx, s);                              \
    }
    // conjugate gradients on the k x k systems (Section 4.5's solver): every class goes through the
    // one-row-per-wavefront kernel, the classes up to k = 32 through its smallest instance
    const WideSolver ws = {prm->solver == ALS_SOLVER_CG, prm->cg_max_iters > 0 ? prm->cg_max_iters : 2 * D,
                           prm->cg_tol > 0.f ? prm->cg_tol : 1e-6f};
    if (ws.cg) {
        if constexpr (D < 64) return fail(ctx, ALS_EINVAL, "conjugate gradients on the dual systems need d >= 64");
        ALS_TIMED_CLASS(T_DUAL_CLASS0 + 1, 1, 1, (stb = launch_dual_wide3(ctx, D, Y, Z, zb16, R, ldr, r0, lists[1], counts_dev[1], g, err, ws, s)))
        ALS_TIMED_CLASS(T_DUAL_CLASS0, 0, 1, (stb = launch_dual_wide3(ctx, D, Y, Z, zb16, R, ldr, r0, lists[0], counts_dev[0], g, err, ws, s)))
        ALS_TIMED_CLASS(T_SMALL8, 9, 1, (stb = launch_dual_wide3(ctx, D, Y, Z, zb16, R, ldr, r0, lists[9], counts_dev[9], g, err, ws, s)))
        ALS_TIMED_CLASS(T_SMALL4, 8, 1, (stb = launch_dual_wide3(ctx, D, Y, Z, zb16, R, ldr, r0, lists[8], counts_dev[8], g, err, ws, s)))
    } else {
    ALS_TIMED_CLASS(T_DUAL_CLASS0 + 1, 1, 4, (launch_dual_multi2(D, Y, Z, zb16, R, ldr, r0, lists[1], counts_dev[1], g, err, s)))
    ALS_TIMED_CLASS(T_DUAL_CLASS0, 0, 4, (launch_dual_k16(D, Y, Z, zb16, R, ldr, r0, lists[0], counts_dev[0], g, err, s)))
    // 5 <= k <= 8 and k <= 4: several rows per MFMA tile
    ALS_TIMED_CLASS(T_SMALL8, 9, 8, (launch_dual_small8(D, Y, Z, zb16, R, ldr, r0, lists[9], counts_dev[9], g, err, s)))
    ALS_TIMED_CLASS(T_SMALL4, 8, 16, (launch_dual_small4(D, Y, Z, zb16, R, ldr, r0, lists[8], counts_dev[8], g, err, s)))
    }
    ALS_TIMED_CLASS(T_DUAL_CLASS0 + 2, 2, 1, (stb = launch_dual_wide3(ctx, D, Y, Z, zb16, R, ldr, r0, lists[2], counts_dev[2], g, err, ws, s)))
    ALS_TIMED_CLASS(T_DUAL_CLASS0 + 3, 3, 1, (stb = launch_dual_wide4(ctx, D, Y, Z, zb16, R, ldr, r0, lists[3], counts_dev[3], g, err, ws, s)))
    ALS_TIMED_CLASS(T_DUAL_CLASS0 + 4, 4, 1, (stb = launch_dual_wide5(ctx, D, Y, Z, zb16, R, ldr, r0, lists[4], counts_dev[4], g, err, ws, s)))
    ALS_TIMED_CLASS(T_DUAL_CLASS0 + 5, 5, 1, (stb = launch_dual_wide6(ctx, D, Y, Z, zb16, R, ldr, r0, lists[5], counts_dev[5], g, err, ws, s)))
    ALS_TIMED_CLASS(T_DUAL_CLASS0 + 6, 6, 1, (stb = launch_dual_wide7(ctx, D, Y, Z, zb16, R, ldr, r0, lists[6], counts_dev[6], g, err, ws, s)))
    ALS_TIMED_CLASS(T_DUAL_CLASS0 + 7, 7, 1, (stb = launch_dual_wide8(ctx, D, Y, Z, zb16, R, ldr, r0, lists[7], counts_dev[7], g, err, ws, s)))
#undef ALS_TIMED_CLASS
    if (stb != ALS_OK) return stb;
    timer_begin(ctx, T_TRANSFORM_X, s);
    const unsigned xblocks = (unsigned)std::min<int64_t>(1024, std::max<int64_t>(1, (r1 - r0 + 127) / 128));
    if constexpr (zb16) {
        static const hipError_t attr_x = hipFuncSetAttribute((const void *)transform16_kernel<D, false, false>,
                                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                                             (int)Xf16Cfg<D>::LDS_BYTES);  // once per process
        ALS_HIP(ctx, attr_x);
        hipLaunchKernelGGL((transform16_kernel<D, false, false>), dim3(xblocks), dim3(256), Xf16Cfg<D>::LDS_BYTES, s,
                           (const void *)R, ldr, (uint16_t *)X->data, X->ld, Linv, r0, r1, Y->indptr, (int64_t)dual_max);
    } else if constexpr (!BF16 && D >= 64) {
        static const hipError_t attr_x = hipFuncSetAttribute((const void *)transform_split_kernel<D, false>,
                                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                                             (int)XfsCfg<D>::LDS_BYTES);  // once per process
        ALS_HIP(ctx, attr_x);
        const unsigned sblocks = (unsigned)std::min<int64_t>(512, std::max<int64_t>(1, (r1 - r0 + 255) / 256));
        hipLaunchKernelGGL((transform_split_kernel<D, false>), dim3(sblocks), dim3(XFS_THREADS), XfsCfg<D>::LDS_BYTES, s,
                           (const float *)R, ldr, (float *)X->data, X->ld, Linv, r0, r1, Y->indptr, (int64_t)dual_max);
    } else {
        static const hipError_t attr_x = hipFuncSetAttribute((const void *)transform_kernel<D, false, BF16, false>,
                                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                                             (int)XfCfg<D>::LDS_BYTES);  // once per process
        ALS_HIP(ctx, attr_x);
        hipLaunchKernelGGL((transform_kernel<D, false, BF16, false>), dim3(xblocks), dim3(256), XfCfg<D>::LDS_BYTES, s,
                           (const void *)R, ldr, X->data, X->ld, Linv, r0, r1, Y->indptr, (int64_t)dual_max);
    }
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

als_status launch_dual_prepare(als_ctx *ctx, const als_table *V, const float *G, const als_params *prm,
                               hipStream_t s) {
    const bool bf = V->dtype == ALS_BF16;
    switch (V->d) {
        case 16: return bf ? dual_prepare_typed<16, true>(ctx, V, G, prm, s) : dual_prepare_typed<16, false>(ctx, V, G, prm, s);
        case 32: return bf ? dual_prepare_typed<32, true>(ctx, V, G, prm, s) : dual_prepare_typed<32, false>(ctx, V, G, prm, s);
        case 64: return bf ? dual_prepare_typed<64, true>(ctx, V, G, prm, s) : dual_prepare_typed<64, false>(ctx, V, G, prm, s);
        case 128: return bf ? dual_prepare_typed<128, true>(ctx, V, G, prm, s) : dual_prepare_typed<128, false>(ctx, V, G, prm, s);
    }
    return fail(ctx, ALS_EDTYPE, "unsupported d");
}

als_status launch_dual_rows(als_ctx *ctx, const als_csr *Y, als_table *X, int64_t r0, int64_t r1, int dual_max,
                            const als_params *prm, const int32_t *const lists[10], const int32_t *const counts[10],
                            const int64_t caps[10], const int hints[10], hipStream_t s) {
    const bool bf = X->dtype == ALS_BF16;
    switch (X->d) {
        case 16: return bf ? dual_rows_typed<16, true>(ctx, Y, X, r0, r1, dual_max, prm, lists, counts, caps, hints, s) : dual_rows_typed<16, false>(ctx, Y, X, r0, r1, dual_max, prm, lists, counts, caps, hints, s);
        case 32: return bf ? dual_rows_typed<32, true>(ctx, Y, X, r0, r1, dual_max, prm, lists, counts, caps, hints, s) : dual_rows_typed<32, false>(ctx, Y, X, r0, r1, dual_max, prm, lists, counts, caps, hints, s);
        case 64: return bf ? dual_rows_typed<64, true>(ctx, Y, X, r0, r1, dual_max, prm, lists, counts, caps, hints, s) : dual_rows_typed<64, false>(ctx, Y, X, r0, r1, dual_max, prm, lists, counts, caps, hints, s);
        case 128: return bf ? dual_rows_typed<128, true>(ctx, Y, X, r0, r1, dual_max, prm, lists, counts, caps, hints, s) : dual_rows_typed<128, false>(ctx, Y, X, r0, r1, dual_max, prm, lists, counts, caps, hints, s);
    }
    return fail(ctx, ALS_EDTYPE, "unsupported d");
}

}  // namespace als
