// Dual row update for rows with 16 < k <= 32 stored entries.  The algebra is in the header comment of
// dual_prepare.hip.  The kernel is written for M rows of S per lane (k <= 16*M); M = 2 is the one in
// use (for 32 < k <= 48, M = 3 was measured slower than the one-row-per-wavefront kernel).
#include "dual_common.h"

#define MULTI_M 2

namespace als {

// Four rows per wavefront, one per group of 16 lanes; lane i of a group owns the M rows i, 16+i, ..
// of its row's k x k system (k <= K = 16*M), so every broadcast of the elimination stays inside a DPP
// row and needs no LDS.
//   1. per row: gather its M tiles into registers, S = I + Z_I Z_I^T tile by tile, packed lower
//      triangle to LDS; the column ids go to LDS for the second gather;
//   2. lanes load their rows; elimination S = M P M^T (unit lower M, pivots P) one column per step with
//      u = M^{-1} y riding along;
//   3. the factor goes back to LDS and is read transposed; back-substitution column by column;
//   4. r = Z_I^T t with one lane per pair of output columns, gathering the entries a second time.
template <int C> __device__ __forceinline__ float bcast16(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + C, 0xf, 0xf, true));
}

template <int D, int M> struct MultiCfg {
    static constexpr int K = 16 * M, TRI = K * (K + 1) / 2;
    static constexpr int OFF_T = 4 * TRI, OFF_ID = OFF_T + 4 * K, OFF_DUMP = OFF_ID + 4 * K;
    static constexpr int OFF_PARTS = OFF_DUMP + 64;  // one dump slot per lane for stores that must not land
    // bf16 Z only: t cut into three bf16 parts plus a block of zeros, [4][4 rows][K]; the finished rows r are
    // staged in the (by then free) triangle area
    static constexpr int LDS_FLOATS = OFF_PARTS;
    static constexpr int LDS_FLOATS_RESIDENT = OFF_PARTS + 16 * K;
    static_assert(4 * TRI >= 4 * D, "the triangle area stages four rows of r");
};

// bf16 Z with two tiles per row: the gathered tiles stay in registers (4 rows x 2 tiles x D/32 operands of
// four registers) until r = Z_I^T t is formed from them on the matrix cores, so nothing is gathered twice.
template <int D, int M, bool ZB> constexpr bool multi_resident() { return ZB && M == 2; }

// One step: the four rows list[4 blk .. 4 blk + 3] (blk * 4 < count).
template <int D, int M, bool ZB>
__device__ __forceinline__ void dual_multi_step(const int64_t *__restrict__ indptr,
                                                const int32_t *__restrict__ indices,
                                                const float *__restrict__ values, const void *__restrict__ Z,
                                                float *__restrict__ R, int64_t ldr, int64_t r0,
                                                const int32_t *__restrict__ list, int count,
                                                int32_t *__restrict__ err_flag, int blk, float *lds) {
    using C = MultiCfg<D, M>;
    constexpr int K = C::K, TRI = C::TRI, NJ = z_pieces<D, ZB>(), CPL = D >= 128 ? 2 : 1;
    float *tri = lds, *tbuf = lds + C::OFF_T;
    int32_t *ids = (int32_t *)(lds + C::OFF_ID);
    // Accesses to the packed triangle are never put under a lane-dependent branch (a branch per element costs
    // more than the access): reads go to an in-range address and are selected afterwards, stores of entries
    // that do not exist go to the lane's dump slot.
    const int lane = opaque_tid(), a = lane & 15, q = lane >> 4;  // MFMA view: entry a of a tile, column group q
    float *dump = lds + C::OFF_DUMP + lane;
    const int g = lane >> 4, i = lane & 15;                         // solver view: system g, lane i of its group

    // Row descriptors of all four rows first (one 16-byte read of the list entries - the list's workspace is
    // padded for it; past the end of the list the first entry stands in - then the four indptr pairs
    // together): one wait per stage instead of one per row.
    int64_t u[4], b[4], b1[4];
    int k[4], kmax = 0, rel[4];
    {
        const ListQuad r4 = *(const ListQuad *)(list + (int64_t)blk * 4);
        const int first = blk * 4;
        rel[0] = r4.x;
        rel[1] = first + 1 < count ? r4.y : r4.x;
        rel[2] = first + 2 < count ? r4.z : r4.x;
        rel[3] = first + 3 < count ? r4.w : r4.x;
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        b[p] = indptr[r0 + rel[p]];
        b1[p] = indptr[r0 + rel[p] + 1];
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const bool have = blk * 4 + p < count;
        u[p] = have ? r0 + rel[p] : -1;  // past the end of the list: the step's first row once more, not stored
        k[p] = (int)(b1[p] - b[p]);
        kmax = k[p] > kmax ? k[p] : kmax;
    }

    // ---- 1. S of every row, packed lower triangle in LDS
    // the column ids of all four rows first: one wait, not one per row.  A slot past the row's k holds the id of
    // the row's first entry with the top bit set: no load for the products, and a harmless, in-range row of the
    // row's own for the second gather (where such a slot meets t = 0)
    int32_t idv[4][M];
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int t = 0; t < M; ++t) {
            const int e = 16 * t + a;
            const int32_t id = indices[b[p] + (e < k[p] ? e : 0)];  // clamped: unconditional load
            idv[p][t] = e < k[p] ? id : (id | (int32_t)0x80000000);
        }
    constexpr bool RES = multi_resident<D, M, ZB>();
    float4 zkeep[RES ? 4 : 1][M][NJ];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        float4 zrow[M][NJ];
        float4 (&z)[M][NJ] = RES ? zkeep[RES ? p : 0] : zrow;
#pragma unroll
        for (int t = 0; t < M; ++t) {
            const int e = 16 * t + a;
            const int32_t id = idv[p][t];
            if (!RES && q == 0) ids[p * K + e] = id & 0x7fffffff;
            if (t < M - 1) {  // every row of the class has more than 16 (M - 1) entries: these tiles are full
#pragma unroll
                for (int j = 0; j < NJ; ++j) z[t][j] = load_piece<D, ZB>(Z, id & 0x7fffffff, j, q);
            } else {
#pragma unroll
                for (int j = 0; j < NJ; ++j) z[t][j] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (id >= 0) {  // one masked region per tile, not one per load
#pragma unroll
                    for (int j = 0; j < NJ; ++j) z[t][j] = load_piece<D, ZB>(Z, id, j, q);
                }
            }
        }
        SplitOperand zs[M][NJ / 2 > 0 ? NJ / 2 : 1];
        if constexpr (!ZB && NJ >= 2) {
#pragma unroll
            for (int t = 0; t < M; ++t)
#pragma unroll
                for (int h = 0; h < NJ / 2; ++h) zs[t][h] = split_operand(z[t][2 * h], z[t][2 * h + 1]);
        }
        __builtin_amdgcn_s_setprio(1);  // matrix-core work first: other wavefronts fill in with vector work
#pragma unroll
        for (int t1 = 0; t1 < M; ++t1)
#pragma unroll
            for (int t2 = 0; t2 <= t1; ++t2) {
                floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
                if constexpr (ZB) {  // bf16 rows are matrix-core operands as loaded
                    acc = mfma_pieces_bf16<NJ>(z[t2], z[t1], acc);
                } else if constexpr (NJ >= 2) {
#pragma unroll
                    for (int h = 0; h < NJ / 2; ++h) acc = split_mfma(zs[t2][h], zs[t1][h], acc);
                } else {
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(z[t2][j].x, z[t1][j].x, acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(z[t2][j].y, z[t1][j].y, acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(z[t2][j].z, z[t1][j].z, acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(z[t2][j].w, z[t1][j].w, acc, 0, 0, 0);
                    }
                }
                // acc[v] = S[Rr][c], Rr = 16*t1 + a, c = 16*t2 + 4q + v (S is symmetric); keep c <= Rr
                const int Rr = 16 * t1 + a;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int c = 16 * t2 + 4 * q + v;
                    float *dst = tri + p * TRI + Rr * (Rr + 1) / 2 + c;
                    if (t2 == t1) dst = c <= Rr ? dst : dump;  // compile-time test: only diagonal tiles have c > Rr
                    *dst = acc[v] + (c == Rr ? 1.f : 0.f);
                }
            }
        __builtin_amdgcn_s_setprio(0);
    }
    wave_sync();

    // ---- 2. elimination, lane i of group g owns rows 16*bk + i of system g
    float s[M][K], y[M], rpm[M];
    int myk = 0;
    int64_t myb = 0;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        myk = g == p ? k[p] : myk;
        myb = g == p ? b[p] : myb;
    }
#pragma unroll
    for (int bk = 0; bk < M; ++bk) {
        const int Rr = 16 * bk + i;
#pragma unroll
        for (int c = 0; c < 16 * (bk + 1); ++c) {
            const float v = tri[g * TRI + Rr * (Rr + 1) / 2 + c];  // c > Rr reads the next row: in range, unused
            s[bk][c] = (c < 16 * bk || c <= Rr) ? v : 0.f;
        }
        y[bk] = 0.f;
        if (Rr < myk) y[bk] = values ? values[myb + Rr] : 1.f;
        rpm[bk] = 1.f;
    }
    bool bad = false;
    dpp_settle(s[0][0], s[1][0]);
    static_for<0, K>([&](auto cc) {
        constexpr int c = decltype(cc)::value;
        constexpr int cb = c / 16, ci = c % 16;
        if (c < kmax) {  // steps beyond every row's k only meet identity rows
            const float pivot = bcast16<ci>(s[cb][c]);
            const float uc = bcast16<ci>(y[cb]);
            bad |= !(pivot > 0.f);
            float rp = __builtin_amdgcn_rcpf(pivot);
            rp = rp * (2.f - pivot * rp);  // one Newton step on the hardware reciprocal
            float nf[M];  // -M[Rr][c]
            static_for<cb, M>([&](auto bb) {
                constexpr int bk = decltype(bb)::value;
                const int Rr = 16 * bk + i;
                rpm[bk] = Rr == c ? rp : rpm[bk];
                nf[bk] = Rr > c ? -(s[bk][c] * rp) : 0.f;  // rows above stay as they are
                y[bk] += nf[bk] * uc;
            });
            // S'[Rr][j] -= M[Rr][c] S'[j][c]: the broadcast of S'[j][c] from the lane that owns row j rides on
            // the multiply-add (column c is final since the previous step and has settled)
            static_for<c + 1, K>([&](auto jj) {
                constexpr int j = decltype(jj)::value;
                constexpr int jb = j / 16, ji = j % 16;
                static_for<jb, M>([&](auto bb) {
                    constexpr int bk = decltype(bb)::value;
                    fmac_bcast16<ji>(s[bk][j], s[jb][c], nf[bk]);
                });
            });
            if constexpr (c + 1 < K) {  // the next step reads column c + 1 through DPP
                if constexpr ((c + 1) / 16 == 0) dpp_settle(s[0][c + 1], s[1][c + 1]);
                else dpp_settle(s[M - 1][c + 1]);
            }
        }
    });
    if (bad && myk > 0) atomicOr(err_flag, 1);

    // ---- 3. factor back to LDS, read transposed (lt[bk][Rr] = S'[Rr][16*bk + i]), back-substitution
#pragma unroll
    for (int bk = 0; bk < M; ++bk) {
        const int Rr = 16 * bk + i;
#pragma unroll
        for (int c = 0; c < 16 * (bk + 1); ++c) {
            float *dst = tri + g * TRI + Rr * (Rr + 1) / 2 + c;
            if (c >= 16 * bk) dst = c <= Rr ? dst : dump;
            *dst = s[bk][c];
        }
    }
    wave_sync();
#pragma unroll
    for (int bk = 0; bk < M; ++bk) {
        const int col = 16 * bk + i;
#pragma unroll
        for (int Rr = 16 * bk; Rr < K; ++Rr) {
            const float v = tri[g * TRI + Rr * (Rr + 1) / 2 + col];  // col > Rr reads a later row: in range, unused
            s[bk][Rr] = (Rr >= 16 * (bk + 1) || Rr > col) ? v : 0.f;
        }
    }
    float t[M];
#pragma unroll
    for (int bk = 0; bk < M; ++bk) t[bk] = 0.f;
    static_for<0, K>([&](auto cc) {
        constexpr int c = K - 1 - decltype(cc)::value;
        constexpr int cb = c / 16, ci = c % 16;
        if (c < kmax) {
            const float tc = bcast16<ci>(y[cb] * rpm[cb]);
            t[cb] = i == ci ? tc : t[cb];
            static_for<0, cb + 1>([&](auto bb) {
                constexpr int bk = decltype(bb)::value;
                y[bk] -= s[bk][c] * tc;  // zero unless row c lies below column 16*bk + i
            });
        }
    });
    if constexpr (RES) {
        // ---- 4. r = Z_I^T t from the tiles in registers (zt_times_t, dual_common.h); parts[x][row][e]: part
        // x of t, x = 3 a block of zeros; the finished rows are staged in the triangle area for 8-byte stores
        float *parts = lds + C::OFF_PARTS;
#pragma unroll
        for (int bk = 0; bk < M; ++bk) {
            float x1, x2;
            t_parts(t[bk], x1, x2);
            const int e = g * K + 16 * bk + i;
            parts[e] = t[bk];
            parts[4 * K + e] = x1;
            parts[8 * K + e] = x2;
            parts[12 * K + e] = 0.f;
        }
        const SelOperands sel = make_sel(lane);
        wave_sync();
        const float *mine = parts + (a < 3 ? a : 3) * 4 * K + 4 * q;
        float *rbuf = tri;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const bf16x8 top[1] = {t_operand(mine + p * K, true)};
            floatx4 out[2 * NJ];
#pragma unroll
            for (int x = 0; x < 2 * NJ; ++x) out[x] = floatx4{0.f, 0.f, 0.f, 0.f};
            zt_times_t<2, NJ>([&](int tt, int j) { return __builtin_bit_cast(bf16x8, zkeep[RES ? p : 0][tt][j]); }, top, sel, out);
#pragma unroll
            for (int x = 0; x < 2 * NJ; ++x)
                *(q == 0 ? rbuf + p * D + column_of_result(x >> 1, x & 1, a) : dump) = out[x][0] + out[x][1] + out[x][2];
        }
        wave_sync();
        const bool col_ok = lane * CPL < D;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            if (u[p] >= 0 && col_ok) {
                if constexpr (CPL == 2) *(float2 *)(R + u[p] * ldr + 2 * lane) = *(const float2 *)(rbuf + p * D + 2 * lane);
                else R[u[p] * ldr + lane] = rbuf[p * D + lane];
            }
        }
        return;
    }
#pragma unroll
    for (int bk = 0; bk < M; ++bk) tbuf[g * K + 16 * bk + i] = t[bk];
    wave_sync();

    // ---- 4. r = Z_I^T t (second gather of the row's entries); the four rows advance together, EPR
    // entries each per round.  Per round: first the ids and t of all rows from LDS with 16-byte reads,
    // then the loads, then the products - no wait and no lane-dependent branch between two loads.
    {
        float r0v[4] = {0.f, 0.f, 0.f, 0.f}, r1v[4] = {0.f, 0.f, 0.f, 0.f};
        const bool col_ok = lane * CPL < D;
        const int zlane = col_ok ? lane : 0;  // lanes without a column (d = 32) read column 0
        // entries per row and round (measured: 16 eight-byte loads in flight are best at d = 128, 32 four-byte
        // loads at d <= 64)
        constexpr int EPR = CPL == 2 ? 4 : 8, NQ = EPR / 4;
        const int kmaxr = (kmax + EPR - 1) / EPR * EPR;  // padded entries have t = 0 and the id of the row's first entry
        for (int e0 = 0; e0 < kmaxr; e0 += EPR) {
            int4 idq[4][NQ];
            float4 teq[4][NQ];
#pragma unroll
            for (int p = 0; p < 4; ++p)
#pragma unroll
                for (int h = 0; h < NQ; ++h) {
                    idq[p][h] = *(const int4 *)(ids + p * K + e0 + 4 * h);
                    teq[p][h] = *(const float4 *)(tbuf + p * K + e0 + 4 * h);
                }
            float zz[4][EPR][CPL];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                if (e0 < k[p]) {  // uniform
#pragma unroll
                    for (int h = 0; h < NQ; ++h) {
                        const int id[4] = {idq[p][h].x, idq[p][h].y, idq[p][h].z, idq[p][h].w};
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            row_cols<ZB, CPL>((const char *)Z + (int64_t)id[x] * D * ZT<ZB>::ES, zlane, zz[p][4 * h + x]);
                        }
                    }
                }
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                if (e0 < k[p]) {
#pragma unroll
                    for (int h = 0; h < NQ; ++h) {
                        const float te[4] = {teq[p][h].x, teq[p][h].y, teq[p][h].z, teq[p][h].w};
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            r0v[p] += te[x] * zz[p][4 * h + x][0];
                            if constexpr (CPL == 2) r1v[p] += te[x] * zz[p][4 * h + x][1];
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            if (u[p] >= 0 && col_ok) {
                if constexpr (CPL == 2) *(float2 *)(R + u[p] * ldr + 2 * lane) = make_float2(r0v[p], r1v[p]);
                else R[u[p] * ldr + lane] = r0v[p];
            }
        }
    }
}

// LOOP = false: workgroup b takes step first_blk + b, if the list is that long (the launch for a list whose
// length the host knows from the previous call).  LOOP = true: grid-stride walk from first_blk to the end of
// the list, correct for any grid size (the length is only known on the device); the step inlined into a
// loop needs about twice the registers, so this form only serves what the first form did not cover.
template <int D, int M, bool ZB, bool LOOP>
__global__ __launch_bounds__(64) void dual_multi_kernel(const int64_t *__restrict__ indptr,
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
        if (blk * 4 < count) dual_multi_step<D, M, ZB>(indptr, indices, values, Z, R, ldr, r0, list, count, err_flag, blk, lds);
    } else {
        for (; blk * 4 < count; blk += gridDim.x) {
            dual_multi_step<D, M, ZB>(opaque(indptr), opaque(indices), opaque(values), opaque(Z), opaque(R), opaque(ldr),
                                  opaque(r0), opaque(list), opaque(count), opaque(err_flag), blk, opaque(lds));
            wave_sync();  // the next step reuses the LDS buffers
        }
    }
}

template <int D, bool ZB>
static void launch_multi_typed(const als_csr *Y, const void *Z, float *R, int64_t ldr, int64_t r0, const int32_t *list,
                               const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s) {
    using C = MultiCfg<D, MULTI_M>;
    constexpr size_t lds_bytes =
        (multi_resident<D, MULTI_M, ZB>() ? C::LDS_FLOATS_RESIDENT : C::LDS_FLOATS) * sizeof(float);
    if (g.known > 0)
        hipLaunchKernelGGL((dual_multi_kernel<D, MULTI_M, ZB, false>), dim3(g.known), dim3(64), lds_bytes, s,
                           Y->indptr, Y->indices, Y->values, Z, R, ldr, r0, list, count_dev, 0, err);
    if (g.rest > 0)
        hipLaunchKernelGGL((dual_multi_kernel<D, MULTI_M, ZB, true>), dim3(g.rest), dim3(64), lds_bytes, s,
                           Y->indptr, Y->indices, Y->values, Z, R, ldr, r0, list, count_dev, (int)g.known, err);
}

void launch_dual_multi2(int d, const als_csr *Y, const void *Z, bool zb16, float *R, int64_t ldr, int64_t r0,
                        const int32_t *list, const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s) {
#define ALS_MULTI_CASE(dd)                                                                       \
    case dd:                                                                                     \
        if (zb16) launch_multi_typed<dd, true>(Y, Z, R, ldr, r0, list, count_dev, g, err, s);    \
        else launch_multi_typed<dd, false>(Y, Z, R, ldr, r0, list, count_dev, g, err, s);        \
        break;
    switch (d) { ALS_MULTI_CASE(32) ALS_MULTI_CASE(64) ALS_MULTI_CASE(128) }  // the dual form stops at k = d
#undef ALS_MULTI_CASE
}

}  // namespace als
