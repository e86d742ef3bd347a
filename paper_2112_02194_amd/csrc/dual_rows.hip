// Dual row update for rows with 8 < k <= 16 stored entries: four rows per wavefront, one lane per row of
// the k x k system, gathered entries kept in registers and copied to LDS for r = Z_I^T t.  The algebra
// is in the header comment of dual_prepare.hip.
#include "dual_common.h"

namespace als {

template <int D> struct DualCfg {
    static constexpr int K = 16;                            // one 16-entry tile per row
    static constexpr int GW = 16;                           // lanes that share one row's k x k system
    static constexpr int RPW = 64 / GW;                     // rows per wavefront (4: read as one int4)
    static constexpr int KP = K + 4;                        // LDS row stride of S (keeps rows 16-byte aligned)
    static constexpr int NJ = D / 16;                       // float4 loads per lane and entry
    static constexpr int ZLD = D + 4;                       // row stride of the LDS copy of Z_I
    static constexpr int SB_FLOATS = RPW * K * KP;
    static constexpr int ZB_FLOATS = K * ZLD;
    static constexpr int TAIL = 64;                         // tbuf[64]
    static constexpr int LDS_FLOATS = (SB_FLOATS > ZB_FLOATS ? SB_FLOATS : ZB_FLOATS) + TAIL;
};

// One wavefront (= one workgroup) solves four rows taken from `list` (row ids relative to r0), all
// with at most 16 stored entries:
//   1. per row, lane (a = lane%16, q = lane/16) loads for entry a and j < D/16 the four columns
//      (4j+q)*4.. of z_a; the same register is the A and the B operand of v_mfma_f32_16x16x4, so the
//      tile accumulates S over all d columns; S = I + Z_I Z_I^T goes to LDS;
//   2. lane i of a row's group of 16 lanes owns row i of S: right-looking Cholesky with the column
//      broadcast by DPP inside the group, then L w = y, then L^T t = w with L read back transposed;
//   3. r = Z_I^T t with one lane per pair of output columns, from an LDS copy of Z_I.
template <int D, bool ZB>
__device__ __forceinline__ void dual_rows_step(const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                                               const float *__restrict__ values, const void *__restrict__ Z,
                                               float *__restrict__ R, int64_t ldr, int64_t r0,
                                               const int32_t *__restrict__ list, int count,
                                               int32_t *__restrict__ err_flag, int blk, float *lds) {
    using C = DualCfg<D>;
    constexpr int K = C::K, KT = 1, GW = C::GW, RPW = C::RPW, KP = C::KP, NJ = z_pieces<D, ZB>();
    constexpr int ZLDB = D * ZT<ZB>::ES + 16;  // row stride in bytes of the LDS copy of Z_I
    float *sb = lds, *tb = lds + (C::LDS_FLOATS - C::TAIL);
    char *zb = (char *)lds;
    const int lane = opaque_tid();
    const int a = lane & 15, q = lane >> 4;
    const int grp = lane / GW, gi = lane % GW;
    const int myrow = gi;

    // Row descriptors, then column ids, then table rows: each stage is issued for all four rows before the
    // next one starts, so that a wavefront waits for three memory round trips, not for three per row.
    // (Loads are unconditional on clamped addresses; what does not exist is masked afterwards.)
    int64_t u[RPW], b[RPW];
    int k[RPW], kmax = 0, rel[RPW];
    {
        // one 16-byte read of the wavefront's four list entries; past the end of the list (its workspace is
        // padded for this) the first entry stands in
        const ListQuad r4 = *(const ListQuad *)(list + (int64_t)blk * RPW);
        const int first = blk * RPW;
        rel[0] = r4.x;
        rel[1] = first + 1 < count ? r4.y : r4.x;
        rel[2] = first + 2 < count ? r4.z : r4.x;
        rel[3] = first + 3 < count ? r4.w : r4.x;
    }
    int64_t b1[RPW];
#pragma unroll
    for (int p = 0; p < RPW; ++p) {
        b[p] = indptr[r0 + rel[p]];
        b1[p] = indptr[r0 + rel[p] + 1];
    }
#pragma unroll
    for (int p = 0; p < RPW; ++p) {
        const bool have = blk * RPW + p < count;
        u[p] = have ? r0 + rel[p] : -1;
        k[p] = have ? (int)(b1[p] - b[p]) : 0;
        kmax = k[p] > kmax ? k[p] : kmax;
    }

    // ---- 1. gather + S tiles
    int64_t idx[RPW];
#pragma unroll
    for (int p = 0; p < RPW; ++p) {
        const int32_t id = indices[b[p] + (a < k[p] ? a : 0)];  // rows of this class have k >= 1: always in range
        idx[p] = a < k[p] ? (int64_t)id : -1;
    }
    float4 z[RPW][KT][NJ];
#pragma unroll
    for (int p = 0; p < RPW; ++p) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) z[p][0][j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (idx[p] >= 0) {  // one masked region per tile, not one per load
#pragma unroll
            for (int j = 0; j < NJ; ++j) z[p][0][j] = load_piece<D, ZB>(Z, idx[p], j, q);
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
        if constexpr (ZB) {  // bf16 rows are matrix-core operands as loaded
            acc[0][0] = mfma_pieces_bf16<NJ>(z[p][0], z[p][0], acc[0][0]);
        } else if constexpr (NJ >= 2) {  // split products on the bf16 matrix cores (dual_common.h)
#pragma unroll
            for (int h = 0; h < NJ / 2; ++h) {
                const SplitOperand zs = split_operand(z[p][0][2 * h], z[p][0][2 * h + 1]);
                acc[0][0] = split_mfma(zs, zs, acc[0][0]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][0][j].x, z[p][0][j].x, acc[0][0], 0, 0, 0);
                acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][0][j].y, z[p][0][j].y, acc[0][0], 0, 0, 0);
                acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][0][j].z, z[p][0][j].z, acc[0][0], 0, 0, 0);
                acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][0][j].w, z[p][0][j].w, acc[0][0], 0, 0, 0);
            }
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
    {
        // k <= 16: Cholesky S = L L^T, column broadcast by DPP inside the 16-lane group
        float myrinv = 1.f;
        static_for<0, K>([&](auto cc) {
            constexpr int c = decltype(cc)::value;
            if (c < kmax) {  // steps beyond every row's k only meet identity rows
                const float pivot = group_bcast<GW, c>(s[c]);
                bad |= !(pivot > 0.f);
                float rinv = __builtin_amdgcn_rsqf(pivot);
                rinv = rinv * (1.5f - 0.5f * pivot * rinv * rinv);  // one Newton step on the hardware estimate
                float lc = s[c] * rinv;
                float nlc = -lc;
                dpp_settle(lc);  // just written, read through DPP below
                s[c] = lc;
                myrinv = myrow == c ? rinv : myrinv;
                static_for<c + 1, K>([&](auto ii) {  // s[i] -= L[row][c] L[i][c], broadcast fused into the multiply-add
                    constexpr int i = decltype(ii)::value;
                    fmac_bcast16<i>(s[i], lc, nlc);
                });
                if constexpr (c + 1 < K) dpp_settle(s[c + 1]);  // the next step's pivot is read through DPP
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
    }
    if (bad && myk > 0) atomicOr(err_flag, 1);

    // ---- 3. r = Z_I^T t
    {
        constexpr int CPL = D >= 128 ? 2 : 1;  // output columns per lane
        tb[lane] = yv;                         // lane == 16*grp + row
#pragma unroll
        for (int p = 0; p < RPW; ++p) {
            wave_sync();  // zb aliases sb and the previous row's copy: all reads of those are done
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int j = 0; j < NJ; ++j) *(float4 *)(zb + (16 * t + a) * ZLDB + (4 * j + q) * 16) = z[p][t][j];
            wave_sync();
            if (u[p] >= 0 && lane * CPL < D) {
                // four slots at a time (slots past the row's k hold t = 0 and zero entries): the LDS reads of a
                // group are issued together, one round trip per group instead of one per entry
                float r0v = 0.f, r1v = 0.f;
#pragma unroll
                for (int h = 0; h < K / 4; ++h) {
                    if (4 * h < k[p]) {  // uniform
                        const float4 tq = *(const float4 *)(tb + p * K + 4 * h);
                        const float te[4] = {tq.x, tq.y, tq.z, tq.w};
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            const int e = 4 * h + x;
                            float zz[CPL];
                            row_cols<ZB, CPL>(zb + e * ZLDB, lane, zz);
                            r0v += te[x] * zz[0];
                            if constexpr (CPL == 2) r1v += te[x] * zz[1];
                        }
                    }
                }
                if constexpr (CPL == 2) *(float2 *)(R + u[p] * ldr + 2 * lane) = make_float2(r0v, r1v);
                else R[u[p] * ldr + lane] = r0v;
            }
        }
    }
}

// The two launch forms of a step kernel (see StepGrid): one step per workgroup, or a grid-stride walk from
// step first_blk to the end of the list.
template <int D, bool ZB, bool LOOP>
__global__ __launch_bounds__(64) void dual_rows_kernel(const int64_t *__restrict__ indptr,
                                                       const int32_t *__restrict__ indices,
                                                       const float *__restrict__ values,
                                                       const void *__restrict__ Z, float *__restrict__ R,
                                                       int64_t ldr, int64_t r0, const int32_t *__restrict__ list,
                                                       const int32_t *__restrict__ count_ptr, int first_blk,
                                                       int32_t *__restrict__ err_flag) {
    extern __shared__ float lds[];
    const int count = *count_ptr;
    int blk = first_blk + blockIdx.x;
    if constexpr (!LOOP) {
        if (blk * DualCfg<D>::RPW < count) dual_rows_step<D, ZB>(indptr, indices, values, Z, R, ldr, r0, list, count, err_flag, blk, lds);
    } else {
        for (; blk * DualCfg<D>::RPW < count; blk += gridDim.x) {
            dual_rows_step<D, ZB>(opaque(indptr), opaque(indices), opaque(values), opaque(Z), opaque(R), opaque(ldr), opaque(r0),
                              opaque(list), opaque(count), opaque(err_flag), blk, opaque(lds));
            wave_sync();  // the next step reuses the LDS buffers
        }
    }
}

template <int D, bool ZB>
static void launch_rows_typed(const als_csr *Y, const void *Z, float *R, int64_t ldr, int64_t r0, const int32_t *list,
                              const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s) {
    using C = DualCfg<D>;
    if (g.known > 0)
        hipLaunchKernelGGL((dual_rows_kernel<D, ZB, false>), dim3(g.known), dim3(64), C::LDS_FLOATS * sizeof(float), s,
                           Y->indptr, Y->indices, Y->values, Z, R, ldr, r0, list, count_dev, 0, err);
    if (g.rest > 0)
        hipLaunchKernelGGL((dual_rows_kernel<D, ZB, true>), dim3(g.rest), dim3(64), C::LDS_FLOATS * sizeof(float), s,
                           Y->indptr, Y->indices, Y->values, Z, R, ldr, r0, list, count_dev, (int)g.known, err);
}

void launch_dual_k16(int d, const als_csr *Y, const void *Z, bool zb16, float *R, int64_t ldr, int64_t r0,
                     const int32_t *list, const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s) {
#define ALS_ROWS_CASE(dd)                                                                             \
    case dd:                                                                                          \
        if (zb16 && dd >= 32) launch_rows_typed<dd, (dd >= 32)>(Y, Z, R, ldr, r0, list, count_dev, g, err, s); \
        else launch_rows_typed<dd, false>(Y, Z, R, ldr, r0, list, count_dev, g, err, s);              \
        break;
    switch (d) { ALS_ROWS_CASE(16) ALS_ROWS_CASE(32) ALS_ROWS_CASE(64) ALS_ROWS_CASE(128) }
#undef ALS_ROWS_CASE
}

}  // namespace als
