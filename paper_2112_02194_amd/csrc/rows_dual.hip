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
//   dual_rows_kernel  one wavefront per 4 / 2 / 1 rows (k <= 16 / 32 / 64): gather Z_I straight into
//                     MFMA operand registers, S = I + Z_I Z_I^T on the matrix cores, Cholesky + two
//                     triangular solves with one lane per row of S, then r = Z_I^T t
//   dual_wide_kernel  one wavefront per row with 64 < k <= 128 (d = 128 only): S tile by tile into a
//                     packed triangle in LDS, elimination with two rows of S per lane
//   transform_kernel  X = R L^{-1}   (rows r -> L^{-T} r), rounding to the table's element type
#include <cstdlib>
#include <type_traits>

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
__global__ __launch_bounds__(256) void transform_kernel(const void *__restrict__ In, int64_t ldi,
                                                        void *__restrict__ Out, int64_t ldo,
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

// ---------------------------------------------------------------------------------------------- dual rows
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int B, int E, class F> __device__ __forceinline__ void static_for(F &&f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// Value of lane C of this lane's group of GW consecutive lanes (GW = 16: DPP row broadcast,
// GW = 32: LDS-crossbar swizzle, GW = 64: scalar read of the lane).
template <int GW, int C> __device__ __forceinline__ float group_bcast(float x) {
    if constexpr (GW == 16) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + C, 0xf, 0xf, true));
    } else if constexpr (GW == 32) {
        return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), C << 5));
    } else {
        return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), C));
    }
}

// x + (x rotated by N lanes inside each row of 16 lanes)
template <int N> __device__ __forceinline__ float add_row_ror(float x) {
    const int r = __builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x120 + N, 0xf, 0xf, false);
    return x + __int_as_float(r);
}

template <int D, int K, bool RG> struct DualCfg {
    static constexpr int KT = K / 16;                       // 16-entry tiles per row
    static constexpr int GW = K <= 16 ? 16 : (K <= 32 ? 32 : 64);  // lanes that share one row's k x k system
    static constexpr int RPW = 64 / GW;                     // rows per wavefront
    static constexpr int KP = K + 4;                        // LDS row stride of S (keeps rows 16-byte aligned)
    static constexpr int NJ = D / 16;                       // float4 loads per lane and entry
    static constexpr bool ZBUF = !RG && K <= 32;            // r = Z_I^T t through an LDS copy of Z_I
    static constexpr int ZLD = D + 4;
    static constexpr int SB_FLOATS = RPW * K * KP;
    static constexpr int ZB_FLOATS = ZBUF ? K * ZLD : 0;
    static constexpr int TAIL = 64 + 128 + 4 + (RG ? 64 * (K / 16 > 1 ? K / 16 : 1) : 0);  // tbuf[64], colbuf[2][64],
                                                                                          // ybuf[2][2], ids (RG)
    static constexpr int LDS_FLOATS = (SB_FLOATS > ZB_FLOATS ? SB_FLOATS : ZB_FLOATS) + TAIL;
};

// One wavefront (= one workgroup) solves RPW rows taken from `list` (row ids relative to r0), all
// with at most K stored entries:
//   1. per row, lane (a = lane%16, q = lane/16) loads for entry e = 16t + a and j < D/16 the four
//      columns (4j+q)*4.. of z_e; the same register is the A and the B operand of
//      v_mfma_f32_16x16x4, so tile (t1,t2) accumulates S[16 t1 + .][16 t2 + .] over all d columns;
//      S = I + Z_I Z_I^T goes to LDS;
//   2. lane i of a row's group of GW lanes owns row i of S: right-looking Cholesky with the column
//      broadcast inside the group, then L w = y, then L^T t = w with L read back transposed;
//   3. r = Z_I^T t, either from an LDS copy of Z_I with one lane per output column pair, or (K > 32)
//      by a cross-lane reduction of the lanes' own pieces.
template <int D, int K, bool RG>
__global__ __launch_bounds__(64) void dual_rows_kernel(const int64_t *__restrict__ indptr,
                                                       const int32_t *__restrict__ indices,
                                                       const float *__restrict__ values,
                                                       const float *__restrict__ Z, float *__restrict__ R,
                                                       int64_t ldr, int64_t r0, const int32_t *__restrict__ list,
                                                       int count, int32_t *__restrict__ err_flag) {
    using C = DualCfg<D, K, RG>;
    constexpr int KT = C::KT, GW = C::GW, RPW = C::RPW, KP = C::KP, NJ = C::NJ, ZLD = C::ZLD;
    extern __shared__ float lds[];
    float *sb = lds, *zb = lds, *tb = lds + (C::LDS_FLOATS - C::TAIL);
    const int lane = threadIdx.x;
    const int a = lane & 15, q = lane >> 4;
    const int grp = lane / GW, gi = lane % GW;
    const int myrow = gi < K ? gi : K - 1;  // K = 48: lanes 48..63 shadow row 47

    int64_t u[RPW], b[RPW];
    int k[RPW], kmax = 0;
#pragma unroll
    for (int p = 0; p < RPW; ++p) {
        const int item = blockIdx.x * RPW + p;
        u[p] = -1; b[p] = 0; k[p] = 0;
        if (item < count) {
            u[p] = r0 + list[item];
            b[p] = indptr[u[p]];
            k[p] = (int)(indptr[u[p] + 1] - b[p]);
        }
        kmax = k[p] > kmax ? k[p] : kmax;
    }

    // ---- 1. gather + S tiles
    float4 z[RPW][KT][NJ];
#pragma unroll
    for (int p = 0; p < RPW; ++p)
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const int e = 16 * t + a;
            const int64_t idx = e < k[p] ? (int64_t)indices[b[p] + e] : -1;
            if constexpr (RG) {
                if (q == 0) ((int32_t *)(tb + 196))[p * K + e] = (int32_t)idx;  // kept for the second gather
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if (idx >= 0) z[p][t][j] = *(const float4 *)(Z + idx * D + (4 * j + q) * 4);
                else z[p][t][j] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    int myk = 0;
    int64_t myb = 0;
#pragma unroll
    for (int p = 0; p < RPW; ++p) {
        myk = grp == p ? k[p] : myk;
        myb = grp == p ? b[p] : myb;
    }
    float yv = 0.f;  // lane i of a group holds the label of entry i
    if (gi < myk) yv = values ? values[myb + gi] : 1.f;

#pragma unroll
    for (int p = 0; p < RPW; ++p) {
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
                    acc[t1][t2] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][t1][j].x, z[p][t2][j].x, acc[t1][t2], 0, 0, 0);
                    acc[t1][t2] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][t1][j].y, z[p][t2][j].y, acc[t1][t2], 0, 0, 0);
                    acc[t1][t2] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][t1][j].z, z[p][t2][j].z, acc[t1][t2], 0, 0, 0);
                    acc[t1][t2] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][t1][j].w, z[p][t2][j].w, acc[t1][t2], 0, 0, 0);
                }
        // lower block triangle of S = I + Z_I Z_I^T (diagonal tiles in full)
#pragma unroll
        for (int t1 = 0; t1 < KT; ++t1)
#pragma unroll
            for (int t2 = 0; t2 <= t1; ++t2)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int i = 16 * t1 + 4 * q + v, jc = 16 * t2 + a;
                    sb[(p * K + i) * KP + jc] = acc[t1][t2][v] + (i == jc ? 1.f : 0.f);
                }
    }
    wave_sync();

    // ---- 2. Cholesky and the two triangular solves; entries right of the diagonal are never used
    float s[K];
    {
        const float4 *row = (const float4 *)(sb + (grp * K + myrow) * KP);
#pragma unroll
        for (int c4 = 0; c4 < K / 4; ++c4) {
            const float4 v = row[c4];
            s[4 * c4] = v.x; s[4 * c4 + 1] = v.y; s[4 * c4 + 2] = v.z; s[4 * c4 + 3] = v.w;
        }
    }
    wave_sync();
    bool bad = false;
    if constexpr (GW == 16) {
        // k <= 16: Cholesky S = L L^T, column broadcast by DPP inside the 16-lane group
        float myrinv = 1.f;
        static_for<0, K>([&](auto cc) {
            constexpr int c = decltype(cc)::value;
            if (c < kmax) {  // steps beyond every row's k only meet identity rows
                const float pivot = group_bcast<GW, c>(s[c]);
                bad |= !(pivot > 0.f);
                float rinv = __builtin_amdgcn_rsqf(pivot);
                rinv = rinv * (1.5f - 0.5f * pivot * rinv * rinv);  // one Newton step on the hardware estimate
                const float lc = s[c] * rinv;
                s[c] = lc;
                myrinv = myrow == c ? rinv : myrinv;
                static_for<c + 1, K>([&](auto ii) {
                    constexpr int i = decltype(ii)::value;
                    s[i] -= lc * group_bcast<GW, i>(lc);
                });
            }
        });
        static_for<0, K>([&](auto cc) {  // L w = y
            constexpr int c = decltype(cc)::value;
            if (c < kmax) {
                const float wc = group_bcast<GW, c>(yv) * group_bcast<GW, c>(myrinv);
                yv = myrow > c ? yv - s[c] * wc : (myrow == c ? wc : yv);
            }
        });
        {
            float4 *row = (float4 *)(sb + (grp * K + myrow) * KP);
#pragma unroll
            for (int c4 = 0; c4 < K / 4; ++c4)
                row[c4] = make_float4(s[4 * c4], s[4 * c4 + 1], s[4 * c4 + 2], s[4 * c4 + 3]);
        }
        wave_sync();
        static_for<0, K>([&](auto cc) {  // L^T t = w
            constexpr int c = K - 1 - decltype(cc)::value;
            if (c < kmax) {
                const float tc = group_bcast<GW, c>(yv) * group_bcast<GW, c>(myrinv);
                const float lt = sb[(grp * K + c) * KP + myrow];  // L[c][myrow], meaningful for myrow <= c
                yv = myrow < c ? yv - lt * tc : (myrow == c ? tc : yv);
            }
        });
    } else {
        // 16 < k <= 64: S = M D M^T (M unit lower, D the pivots), one column per step.  Every lane
        // publishes its entry of the column in LDS (double-buffered by step parity), then reads the
        // pivot and the whole column back with broadcast reads; u = M^{-1} y rides along.
        float *colbuf = tb + 64, *yb = tb + 64 + 128;
        float rp_mine = 1.f;
        static_for<0, K>([&](auto cc) {
            constexpr int c = decltype(cc)::value;
            if (c < kmax) {
                float *cb = colbuf + (c & 1) * 64;
                cb[lane] = s[c];  // S'[row][c] as it stands (column c is final)
                if (gi == c) yb[(c & 1) * 2 + grp] = yv;
                wave_sync();
                const float pivot = cb[grp * GW + c];
                const float uc = yb[(c & 1) * 2 + grp];
                bad |= !(pivot > 0.f);
                float rp = __builtin_amdgcn_rcpf(pivot);
                rp = rp * (2.f - pivot * rp);  // one Newton step on the hardware reciprocal
                rp_mine = myrow == c ? rp : rp_mine;
                const float f = myrow > c ? s[c] * rp : 0.f;  // M[row][c]; rows above stay as they are
                yv -= f * uc;
                static_for<(c + 1) / 4, K / 4>([&](auto jj) {
                    constexpr int j4 = decltype(jj)::value;
                    const float4 col = *(const float4 *)(cb + grp * GW + 4 * j4);
                    if constexpr (4 * j4 + 0 > c) s[4 * j4 + 0] -= f * col.x;
                    if constexpr (4 * j4 + 1 > c) s[4 * j4 + 1] -= f * col.y;
                    if constexpr (4 * j4 + 2 > c) s[4 * j4 + 2] -= f * col.z;
                    if constexpr (4 * j4 + 3 > c) s[4 * j4 + 3] -= f * col.w;
                });
            }
        });
        // t_c = (u_c - sum_{R>c} S'[R][c] t_R) / pivot_c with lane c owning unknown c: the factor is
        // read back transposed through LDS, t_c is broadcast inside the group
        {
            float4 *row = (float4 *)(sb + (grp * K + myrow) * KP);
#pragma unroll
            for (int c4 = 0; c4 < K / 4; ++c4)
                row[c4] = make_float4(s[4 * c4], s[4 * c4 + 1], s[4 * c4 + 2], s[4 * c4 + 3]);
        }
        wave_sync();
#pragma unroll
        for (int c = 0; c < K; ++c) s[c] = sb[(grp * K + c) * KP + myrow];  // S'[c][myrow], used for myrow < c
        static_for<0, K>([&](auto cc) {
            constexpr int c = K - 1 - decltype(cc)::value;
            if (c < kmax) {
                const float tc = group_bcast<GW, c>(yv * rp_mine);
                yv = myrow < c ? yv - s[c] * tc : (myrow == c ? tc : yv);
            }
        });
    }
    if (bad && myk > 0) atomicOr(err_flag, 1);

    // ---- 3. r = Z_I^T t
    if constexpr (RG) {
        // gather the row's entries a second time (they are still in the caches), one lane per pair of
        // output columns, so that no copy of Z_I has to stay in registers or LDS during the solve
        constexpr int CPL = D >= 128 ? 2 : 1;
        tb[lane] = yv;  // lane grp*GW + i holds t_i
        wave_sync();
#pragma unroll
        for (int p = 0; p < RPW; ++p) {
            if (u[p] >= 0 && lane * CPL < D) {
                float r0v = 0.f, r1v = 0.f;
                const int32_t *ix = (const int32_t *)(tb + 196) + p * K;
                const int kp8 = (k[p] + 7) & ~7;  // padded entries have t = 0 and id -1 (row 0 is read instead)
                for (int e0 = 0; e0 < kp8; e0 += 8) {
                    float2 zz[8];
                    float te[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int id = ix[e0 + i];
                        te[i] = tb[p * GW + e0 + i];
                        const float *zr = Z + (int64_t)(id < 0 ? 0 : id) * D + CPL * lane;
                        if constexpr (CPL == 2) zz[i] = *(const float2 *)zr;
                        else zz[i] = make_float2(zr[0], 0.f);
                    }
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        r0v += te[i] * zz[i].x;
                        r1v += te[i] * zz[i].y;
                    }
                }
                if constexpr (CPL == 2) *(float2 *)(R + u[p] * ldr + 2 * lane) = make_float2(r0v, r1v);
                else R[u[p] * ldr + lane] = r0v;
            }
        }
    } else if constexpr (C::ZBUF) {
        constexpr int CPL = D >= 128 ? 2 : 1;  // output columns per lane
        tb[lane] = yv;                         // K <= 32: lane == grp*K + row
#pragma unroll
        for (int p = 0; p < RPW; ++p) {
            wave_sync();  // zb aliases sb and the previous row's copy: all reads of those are done
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int j = 0; j < NJ; ++j) *(float4 *)(zb + (16 * t + a) * ZLD + (4 * j + q) * 4) = z[p][t][j];
            wave_sync();
            if (u[p] >= 0 && lane * CPL < D) {
                float r0v = 0.f, r1v = 0.f;
                for (int e = 0; e < k[p]; ++e) {
                    const float te = tb[p * K + e];
                    if constexpr (CPL == 2) {
                        const float2 zz = *(const float2 *)(zb + e * ZLD + 2 * lane);
                        r0v += te * zz.x;
                        r1v += te * zz.y;
                    } else {
                        r0v += te * zb[e * ZLD + lane];
                    }
                }
                if constexpr (CPL == 2) *(float2 *)(R + u[p] * ldr + 2 * lane) = make_float2(r0v, r1v);
                else R[u[p] * ldr + lane] = r0v;
            }
        }
    } else {
        // scale this lane's pieces by t_e, add over the tiles, then over the 16 lanes a of each q
        float4 rp[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) rp[j] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const float te = __shfl(yv, 16 * t + a);
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                rp[j].x += te * z[0][t][j].x; rp[j].y += te * z[0][t][j].y;
                rp[j].z += te * z[0][t][j].z; rp[j].w += te * z[0][t][j].w;
            }
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            float4 v = rp[j];
            v.x = add_row_ror<8>(v.x); v.y = add_row_ror<8>(v.y); v.z = add_row_ror<8>(v.z); v.w = add_row_ror<8>(v.w);
            v.x = add_row_ror<4>(v.x); v.y = add_row_ror<4>(v.y); v.z = add_row_ror<4>(v.z); v.w = add_row_ror<4>(v.w);
            v.x = add_row_ror<2>(v.x); v.y = add_row_ror<2>(v.y); v.z = add_row_ror<2>(v.z); v.w = add_row_ror<2>(v.w);
            v.x = add_row_ror<1>(v.x); v.y = add_row_ror<1>(v.y); v.z = add_row_ror<1>(v.z); v.w = add_row_ror<1>(v.w);
            if (a == j && u[0] >= 0) *(float4 *)(R + u[0] * ldr + (4 * j + q) * 4) = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------- dual rows, 64 < k <= 128
// One wavefront per row with k <= K = 16*KT entries (KT = 5..8).
//   1. S = I + Z_I Z_I^T tile by tile: the wavefront keeps the 16 entries of tile t1 in registers (B
//      operand) and streams the tiles t2 <= t1 past them (A operand, fetched again from the caches);
//      each finished 16x16 tile goes to LDS, where S is kept as a packed lower triangle.
//   2. Elimination S = M P M^T with lane i owning rows i and 64+i (columns 0..63 of the first, all of
//      the second, in registers): per step the column is published in LDS and read back by broadcast,
//      pivot and right-hand-side entry come straight from the owning lane; u = M^{-1} y rides along.
//   3. Back-substitution with the factor read transposed from LDS, the value just found taken from
//      its lane.
//   4. r = Z_I^T t with one lane per pair of output columns, gathering the entries a second time.
template <int D, int KT> struct WideCfg {
    static constexpr int K = 16 * KT;
    static constexpr int TRI = K * (K + 1) / 2;      // packed lower triangle
    static constexpr int OFF_COL = TRI;              // colbuf[2][K]
    static constexpr int OFF_T = OFF_COL + 2 * K;    // tbuf[K]
    static constexpr int OFF_ID = OFF_T + K;         // ids[K]
    static constexpr int LDS_FLOATS = OFF_ID + K;
};

template <int D, int KT>
__global__ __launch_bounds__(64) void dual_wide_kernel(const int64_t *__restrict__ indptr,
                                                       const int32_t *__restrict__ indices,
                                                       const float *__restrict__ values,
                                                       const float *__restrict__ Z, float *__restrict__ R,
                                                       int64_t ldr, int64_t r0, const int32_t *__restrict__ list,
                                                       int32_t *__restrict__ err_flag) {
    using C = WideCfg<D, KT>;
    constexpr int K = C::K, NJ = D / 16, K1 = K - 64;  // K1 = rows held as "second row" of a lane
    extern __shared__ float lds[];
    float *tri = lds, *colbuf = lds + C::OFF_COL, *tbuf = lds + C::OFF_T;
    int32_t *ids = (int32_t *)(lds + C::OFF_ID);
    const int lane = threadIdx.x, a = lane & 15, q = lane >> 4;
    const int64_t u = r0 + list[blockIdx.x];
    const int64_t b = indptr[u];
    const int k = (int)(indptr[u + 1] - b);  // <= K by the list's class

    // ---- 1. S tiles
    int32_t myid[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t) {
        const int e = 16 * t + a;
        myid[t] = e < k ? indices[b + e] : -1;
        if (q == 0) ids[e] = myid[t];
    }
    // the first RT tiles stay in registers for the whole phase (one round of loads, all in flight
    // together); later tiles are fetched when they are needed
    constexpr int RT = KT < 5 ? KT : 5;
    float4 zres[RT][NJ];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            zres[t][j] = myid[t] >= 0 ? *(const float4 *)(Z + (int64_t)myid[t] * D + (4 * j + q) * 4)
                                      : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int t1 = 0; t1 < KT; ++t1) {
        float4 zb[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (t1 < RT) zb[j] = zres[t1 < RT ? t1 : 0][j];
            else zb[j] = myid[t1] >= 0 ? *(const float4 *)(Z + (int64_t)myid[t1] * D + (4 * j + q) * 4)
                                       : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int t2 = 0; t2 <= t1; ++t2) {
            floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                float4 za;
                if (t2 == t1) za = zb[j];
                else if (t2 < RT) za = zres[t2 < RT ? t2 : 0][j];
                else za = myid[t2] >= 0 ? *(const float4 *)(Z + (int64_t)myid[t2] * D + (4 * j + q) * 4)
                                        : make_float4(0.f, 0.f, 0.f, 0.f);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(za.x, zb[j].x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(za.y, zb[j].y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(za.z, zb[j].z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(za.w, zb[j].w, acc, 0, 0, 0);
            }
            // acc[v] = S[Rr][c], Rr = 16*t1 + a, c = 16*t2 + 4q + v (S is symmetric); keep c <= Rr
            const int Rr = 16 * t1 + a;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int c = 16 * t2 + 4 * q + v;
                if (c <= Rr) tri[Rr * (Rr + 1) / 2 + c] = acc[v] + (c == Rr ? 1.f : 0.f);
            }
        }
    }
    wave_sync();

    // ---- 2. elimination; lane i owns rows i (columns 0..63) and 64+i (all columns, if 64+i < K)
    const int ra = lane, rb = 64 + lane;
    const bool hasb = rb < K;
    float s0[64], s1[K];
#pragma unroll
    for (int c = 0; c < 64; ++c) s0[c] = c <= ra ? tri[ra * (ra + 1) / 2 + c] : 0.f;
#pragma unroll
    for (int c = 0; c < K; ++c) s1[c] = (hasb && c <= rb) ? tri[rb * (rb + 1) / 2 + c] : 0.f;
    float y0 = 0.f, y1 = 0.f;
    if (ra < k) y0 = values ? values[b + ra] : 1.f;
    if (rb < k) y1 = values ? values[b + rb] : 1.f;
    float rp0 = 1.f, rp1 = 1.f;
    bool bad = false;
    wave_sync();
    static_for<0, K>([&](auto cc) {
        constexpr int c = decltype(cc)::value;
        if (c < k) {  // the remaining rows are identity rows with zero right-hand side
            float *cb = colbuf + (c & 1) * K;
            float pivot, uc;
            if constexpr (c < 64) {
                cb[lane] = s0[c];
                if (hasb) cb[64 + lane] = s1[c];
                pivot = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s0[c]), c));
                uc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(y0), c));
            } else {
                if (hasb) cb[64 + lane] = s1[c];
                pivot = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s1[c]), c - 64));
                uc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(y1), c - 64));
            }
            bad |= !(pivot > 0.f);
            float rp = __builtin_amdgcn_rcpf(pivot);
            rp = rp * (2.f - pivot * rp);  // one Newton step on the hardware reciprocal
            float f0 = 0.f;
            if constexpr (c < 64) {
                rp0 = ra == c ? rp : rp0;
                f0 = ra > c ? s0[c] * rp : 0.f;
                y0 -= f0 * uc;
            }
            rp1 = rb == c ? rp : rp1;
            const float f1 = rb > c ? s1[c] * rp : 0.f;  // lanes without a second row hold zeros in s1
            y1 -= f1 * uc;
            wave_sync();
            static_for<(c + 1) / 4, K / 4>([&](auto jj) {
                constexpr int j4 = decltype(jj)::value;
                const float4 col = *(const float4 *)(cb + 4 * j4);
                if constexpr (4 * j4 + 0 > c) { if constexpr (4 * j4 + 0 < 64 && c < 64) s0[4 * j4 + 0] -= f0 * col.x; s1[4 * j4 + 0] -= f1 * col.x; }
                if constexpr (4 * j4 + 1 > c) { if constexpr (4 * j4 + 1 < 64 && c < 64) s0[4 * j4 + 1] -= f0 * col.y; s1[4 * j4 + 1] -= f1 * col.y; }
                if constexpr (4 * j4 + 2 > c) { if constexpr (4 * j4 + 2 < 64 && c < 64) s0[4 * j4 + 2] -= f0 * col.z; s1[4 * j4 + 2] -= f1 * col.z; }
                if constexpr (4 * j4 + 3 > c) { if constexpr (4 * j4 + 3 < 64 && c < 64) s0[4 * j4 + 3] -= f0 * col.w; s1[4 * j4 + 3] -= f1 * col.w; }
            });
        }
    });
    if (bad && lane == 0) atomicOr(err_flag, 1);

    // ---- 3. t_c = (u_c - sum_{Rr>c} S'[Rr][c] t_Rr) / pivot_c; the factor goes back to the packed triangle
#pragma unroll
    for (int c = 0; c < 64; ++c)
        if (c <= ra) tri[ra * (ra + 1) / 2 + c] = s0[c];
#pragma unroll
    for (int c = 0; c < K; ++c)
        if (hasb && c <= rb) tri[rb * (rb + 1) / 2 + c] = s1[c];
    wave_sync();
    {
        float t0 = 0.f, t1v = 0.f;
#pragma unroll 4
        for (int Rr = (k < K ? k : K) - 1; Rr >= 64; --Rr) {
            const float tR = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(y1 * rp1), Rr - 64));
            t1v = rb == Rr ? tR : t1v;
            const int base = Rr * (Rr + 1) / 2;
            if (rb < Rr) y1 -= tri[base + rb] * tR;
            y0 -= tri[base + ra] * tR;
        }
#pragma unroll 4
        for (int Rr = (k < 64 ? k : 64) - 1; Rr >= 0; --Rr) {
            const float tR = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(y0 * rp0), Rr));
            t0 = ra == Rr ? tR : t0;
            if (ra < Rr) y0 -= tri[Rr * (Rr + 1) / 2 + ra] * tR;
        }
        tbuf[ra] = t0;
        if (hasb) tbuf[rb] = t1v;
    }
    wave_sync();

    // ---- 4. r = Z_I^T t, one lane per pair of output columns (second gather of the row's entries)
    {
        float r0v = 0.f, r1v = 0.f;
        const int kp8 = (k + 7) & ~7;  // padded entries have t = 0 and id -1 (row 0 is read instead)
        for (int e0 = 0; e0 < kp8; e0 += 8) {
            float2 zz[8];
            float te[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int id = ids[e0 + i];
                te[i] = tbuf[e0 + i];
                zz[i] = *(const float2 *)(Z + (int64_t)(id < 0 ? 0 : id) * D + 2 * lane);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                r0v += te[i] * zz[i].x;
                r1v += te[i] * zz[i].y;
            }
        }
        *(float2 *)(R + u * ldr + 2 * lane) = make_float2(r0v, r1v);
    }
}

// ---------------------------------------------------------------------------------------------- launchers
int dual_supported_max_k(int d) { return d < 128 ? (d < 64 ? d : 64) : 128; }

static bool regather_default(int K) {
    // bit i set = class i (K = 16*(i+1)) gathers its entries a second time for r = Z_I^T t instead of
    // keeping them in registers; measured faster only for K = 64 (register pressure).  The
    // environment variable is a tuning knob for experiments.
    const char *e = getenv("ALS_DUAL_REGATHER");
    const int mask = e ? atoi(e) : 8;
    return (mask >> (K / 16 - 1)) & 1;
}

template <int D, int K>
static void launch_dual_class(const als_csr *Y, const float *Z, float *R, int64_t ldr, int64_t r0,
                              const int32_t *list, int count, int32_t *err, hipStream_t s) {
    if (count <= 0) return;
    if (regather_default(K)) {
        using C = DualCfg<D, K, true>;
        const unsigned blocks = (unsigned)((count + C::RPW - 1) / C::RPW);
        hipLaunchKernelGGL((dual_rows_kernel<D, K, true>), dim3(blocks), dim3(64), C::LDS_FLOATS * sizeof(float), s,
                           Y->indptr, Y->indices, Y->values, Z, R, ldr, r0, list, count, err);
        return;
    }
    using C = DualCfg<D, K, false>;
    const unsigned blocks = (unsigned)((count + C::RPW - 1) / C::RPW);
    hipLaunchKernelGGL((dual_rows_kernel<D, K, false>), dim3(blocks), dim3(64), C::LDS_FLOATS * sizeof(float), s, Y->indptr,
                       Y->indices, Y->values, Z, R, ldr, r0, list, count, err);
}

// Part 1 (needs no row classification): factorise B and build Z = V L^{-T}.
template <int D, bool BF16>
static als_status dual_prepare_typed(als_ctx *ctx, const als_table *V, const float *G, const als_params *prm,
                                     hipStream_t s) {
    als_status st = ensure(ctx, ctx->ztable, (size_t)V->rows * D * sizeof(float));
    if (st != ALS_OK) return st;
    float *Linv = (float *)((char *)ctx->small.p + SM_FACTOR), *LinvT = Linv + 128 * 128;
    int32_t *err = (int32_t *)((char *)ctx->small.p + SM_COUNTERS) + 2;
    constexpr size_t factor_lds = (size_t)(D * (D + 1) + D) * sizeof(double);
    ALS_HIP(ctx, hipFuncSetAttribute((const void *)factor_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)factor_lds));
    timer_begin(ctx, T_TRANSFORM, s);
    hipLaunchKernelGGL(factor_kernel<D>, dim3(1), dim3(256), factor_lds, s, G, prm->alpha, prm->lambda, Linv, LinvT,
                       err);
    const unsigned tblocks = (unsigned)std::min<int64_t>(1024, std::max<int64_t>(1, (V->rows + 127) / 128));
    ALS_HIP(ctx, hipFuncSetAttribute((const void *)transform_kernel<D, BF16, false, true>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)XfCfg<D>::LDS_BYTES));
    hipLaunchKernelGGL((transform_kernel<D, BF16, false, true>), dim3(tblocks), dim3(256), XfCfg<D>::LDS_BYTES, s, V->data, V->ld,
                       ctx->ztable.p, (int64_t)D, (const float *)LinvT, (int64_t)0, V->rows,
                       (const int64_t *)nullptr, (int64_t)0);
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

// Part 2: the row kernels of the four k-classes, then X = R L^{-1} on the rows they solved.
template <int D, int KT>
static als_status launch_big_class(als_ctx *ctx, const als_csr *Y, const float *Z, float *R, int64_t ldr, int64_t r0,
                                   const int32_t *list, int count, int32_t *err, hipStream_t s) {
    if (count <= 0) return ALS_OK;
    if constexpr (D == 128) {
        using C = WideCfg<D, KT>;
        auto kern = dual_wide_kernel<D, KT>;
        ALS_HIP(ctx, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)(C::LDS_FLOATS * sizeof(float))));
        hipLaunchKernelGGL(kern, dim3((unsigned)count), dim3(64), C::LDS_FLOATS * sizeof(float), s, Y->indptr,
                           Y->indices, Y->values, Z, R, ldr, r0, list, err);
        return ALS_OK;
    } else {
        return fail(ctx, ALS_EINVAL, "rows with more than 64 entries take the dual form only for d = 128");
    }
}

template <int D, bool BF16>
static als_status dual_rows_typed(als_ctx *ctx, const als_csr *Y, als_table *X, int64_t r0, int64_t r1,
                                  int dual_max, const int32_t *const lists[8], const int counts[8], hipStream_t s) {
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
    const float *Z = (const float *)ctx->ztable.p;
    // Independent classes run concurrently: the two largest on the caller's stream, 32 < k <= 64 on
    // side stream 0, the workgroup kernels (k > 64) on side stream 1.  The caller has forked the side
    // streams; they are joined before the closing transform, which reads every class's result.
    als_status stb = ALS_OK;
    const bool side = ctx->use_side_streams;
    hipStream_t s_mid = side ? ctx->side[0] : s, s_big = side ? ctx->side[1] : s;
#define ALS_TIMED_CLASS(cls, strm, call)            \
    if (counts[cls] > 0 && stb == ALS_OK) {         \
        hipStream_t cs = strm;                      \
        timer_begin(ctx, T_DUAL_CLASS0 + cls, cs);  \
        call;                                       \
        timer_end(ctx, cs);                         \
    }
    ALS_TIMED_CLASS(1, s, (launch_dual_class<D, 32>(Y, Z, R, ldr, r0, lists[1], counts[1], err, cs)))
    ALS_TIMED_CLASS(0, s, (launch_dual_class<D, 16>(Y, Z, R, ldr, r0, lists[0], counts[0], err, cs)))
    ALS_TIMED_CLASS(2, s_mid, (launch_dual_class<D, 48>(Y, Z, R, ldr, r0, lists[2], counts[2], err, cs)))
    ALS_TIMED_CLASS(3, s_mid, (launch_dual_class<D, 64>(Y, Z, R, ldr, r0, lists[3], counts[3], err, cs)))
    ALS_TIMED_CLASS(4, s_big, (stb = launch_big_class<D, 5>(ctx, Y, Z, R, ldr, r0, lists[4], counts[4], err, cs)))
    ALS_TIMED_CLASS(5, s_big, (stb = launch_big_class<D, 6>(ctx, Y, Z, R, ldr, r0, lists[5], counts[5], err, cs)))
    ALS_TIMED_CLASS(6, s_big, (stb = launch_big_class<D, 7>(ctx, Y, Z, R, ldr, r0, lists[6], counts[6], err, cs)))
    ALS_TIMED_CLASS(7, s_big, (stb = launch_big_class<D, 8>(ctx, Y, Z, R, ldr, r0, lists[7], counts[7], err, cs)))
#undef ALS_TIMED_CLASS
    if (side && stb == ALS_OK) stb = side_join(ctx, 0, s);
    if (side && stb == ALS_OK) stb = side_join(ctx, 1, s);
    if (stb != ALS_OK) return stb;
    timer_begin(ctx, T_TRANSFORM, s);
    const unsigned xblocks = (unsigned)std::min<int64_t>(1024, std::max<int64_t>(1, (r1 - r0 + 127) / 128));
    ALS_HIP(ctx, hipFuncSetAttribute((const void *)transform_kernel<D, false, BF16, false>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)XfCfg<D>::LDS_BYTES));
    hipLaunchKernelGGL((transform_kernel<D, false, BF16, false>), dim3(xblocks), dim3(256), XfCfg<D>::LDS_BYTES, s, (const void *)R, ldr,
                       X->data, X->ld, Linv, r0, r1, Y->indptr, (int64_t)dual_max);
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
                            const int32_t *const lists[8], const int counts[8], hipStream_t s) {
    const bool bf = X->dtype == ALS_BF16;
    switch (X->d) {
        case 16: return bf ? dual_rows_typed<16, true>(ctx, Y, X, r0, r1, dual_max, lists, counts, s) : dual_rows_typed<16, false>(ctx, Y, X, r0, r1, dual_max, lists, counts, s);
        case 32: return bf ? dual_rows_typed<32, true>(ctx, Y, X, r0, r1, dual_max, lists, counts, s) : dual_rows_typed<32, false>(ctx, Y, X, r0, r1, dual_max, lists, counts, s);
        case 64: return bf ? dual_rows_typed<64, true>(ctx, Y, X, r0, r1, dual_max, lists, counts, s) : dual_rows_typed<64, false>(ctx, Y, X, r0, r1, dual_max, lists, counts, s);
        case 128: return bf ? dual_rows_typed<128, true>(ctx, Y, X, r0, r1, dual_max, lists, counts, s) : dual_rows_typed<128, false>(ctx, Y, X, r0, r1, dual_max, lists, counts, s);
    }
    return fail(ctx, ALS_EDTYPE, "unsupported d");
}

}  // namespace als
