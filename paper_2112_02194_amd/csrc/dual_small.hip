// Dual row update for rows with very few stored entries: k <= G with G = 8 or 4, compiled once per
// class with -DSMALL_G=8 / -DSMALL_G=4.  Several rows share one 16-entry MFMA tile (16/G rows per
// tile, four tiles per wavefront, so 8 or 16 rows per wavefront): the tile's 16x16 product then holds
// the rows' G x G systems S = I + Z_I Z_I^T as its diagonal blocks; the off-diagonal blocks are never
// read.  Lane i of a tile's 16-lane group owns row i of the tile, i.e. row i % G of sub-system i / G;
// every broadcast of the elimination stays inside the G lanes of a sub-system (DPP).  r = Z_I^T t is
// taken from an LDS copy of the tile's gathered entries.  The algebra is in the header comment of
// dual_prepare.hip.
#include "dual_common.h"

#ifndef SMALL_G
#error "compile with -DSMALL_G=8 or -DSMALL_G=4"
#endif

namespace als {

// Value of lane C of this lane's group of G consecutive lanes (G = 8 or 4, groups aligned inside a
// DPP row of 16 lanes).
template <int G, int C> __device__ __forceinline__ float sub_bcast(float x, bool upper_half) {
    if constexpr (G == 4) {
        constexpr int ctrl = C | (C << 2) | (C << 4) | (C << 6);  // quad_perm:[C,C,C,C]
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), ctrl, 0xf, 0xf, true));
    } else {
        const float lo = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + C, 0xf, 0xf, true));
        const float hi = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + 8 + C, 0xf, 0xf, true));
        return upper_half ? hi : lo;
    }
}

template <int D, int G> struct SmallCfg {
    static constexpr int SPT = 16 / G, NR = 4 * SPT;  // sub-systems per tile, rows per wavefront
    static constexpr int KP = 20, ZLD = D + 4;
    static constexpr int SB_FLOATS = 4 * 16 * KP, ZB_FLOATS = 16 * ZLD;
    static constexpr int MAIN = SB_FLOATS > ZB_FLOATS ? SB_FLOATS : ZB_FLOATS;  // S of the four tiles, later one tile's Z
    static constexpr int OFF_T = MAIN, OFF_META = OFF_T + 64;                    // t[64]; per row: u (2 ints), k
    static constexpr int LDS_FLOATS = OFF_META + 3 * NR + 1;
};

template <int D, int G, bool ZB>
__device__ __forceinline__ void dual_small_step(const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                                                const float *__restrict__ values, const void *__restrict__ Z,
                                                float *__restrict__ R, int64_t ldr, int64_t r0,
                                                const int32_t *__restrict__ list, int count,
                                                int32_t *__restrict__ err_flag, int blk, float *lds) {
    using C = SmallCfg<D, G>;
    constexpr int SPT = C::SPT, NR = C::NR, KP = C::KP, NJ = z_pieces<D, ZB>(), CPL = D >= 128 ? 2 : 1;
    constexpr int ZLDB = D * ZT<ZB>::ES + 16;  // row stride in bytes of the LDS copy of a tile's entries
    float *sb = lds, *tb = lds + C::OFF_T;
    char *zb = (char *)lds;
    int32_t *meta = (int32_t *)(lds + C::OFF_META);  // [NR][3]: u lo, u hi, k
    const int lane = opaque_tid(), a = lane & 15, q = lane >> 4;
    const int sub = a / G, e = a % G;  // MFMA view: sub-system of the tile and entry slot
    const bool upper = (a & 8) != 0;

    // ---- 1. gather: tile p holds rows p*SPT .. p*SPT + SPT-1 of this wavefront.  List entry, row
    // descriptor, column id and table row are four dependent loads; each stage is issued for all four
    // tiles before the next one starts (unconditional loads on clamped addresses, masked afterwards), so
    // that a wavefront waits for four memory round trips instead of sixteen.
    float4 z[4][NJ];
    float yl[4];  // label of this lane's entry in tile p
    int rel[4], kk[4];
    int64_t bb[4], b1[4], idx[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int item = blk * NR + p * SPT + sub;
        rel[p] = list[item < count ? item : count - 1];
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        bb[p] = indptr[r0 + rel[p]];
        b1[p] = indptr[r0 + rel[p] + 1];
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int rr = p * SPT + sub;
        const bool have = blk * NR + rr < count;
        const int64_t u = have ? r0 + rel[p] : -1;
        kk[p] = have ? (int)(b1[p] - bb[p]) : 0;
        if (q == 0 && e == 0) {
            meta[3 * rr + 0] = (int32_t)(u & 0xffffffff);
            meta[3 * rr + 1] = (int32_t)(u >> 32);
            meta[3 * rr + 2] = kk[p];
        }
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int64_t at = bb[p] + (e < kk[p] ? e : 0);  // a row of the list has k >= 1: always in range
        const int32_t id = indices[at];
        const float yv = values ? values[at] : 1.f;
        idx[p] = e < kk[p] ? (int64_t)id : -1;
        yl[p] = e < kk[p] ? yv : 0.f;
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) z[p][j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (idx[p] >= 0) {  // one masked region per tile, not one per load
#pragma unroll
            for (int j = 0; j < NJ; ++j) z[p][j] = load_piece<D, ZB>(Z, idx[p], j, q);
        }
    }
    // ---- 2. the tiles' products; tile p's 16 x 16 result to LDS (only its diagonal blocks are used)
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
        if constexpr (ZB) {  // bf16 rows are matrix-core operands as loaded
            acc = mfma_pieces_bf16<NJ>(z[p], z[p], acc);
        } else if constexpr (NJ >= 2) {  // split products on the bf16 matrix cores (dual_common.h)
#pragma unroll
            for (int h = 0; h < NJ / 2; ++h) {
                const SplitOperand zs = split_operand(z[p][2 * h], z[p][2 * h + 1]);
                acc = split_mfma(zs, zs, acc);
            }
        } else {
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][j].x, z[p][j].x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][j].y, z[p][j].y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][j].z, z[p][j].z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(z[p][j].w, z[p][j].w, acc, 0, 0, 0);
            }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = 4 * q + v;
            sb[(p * 16 + i) * KP + a] = acc[v] + (i == a ? 1.f : 0.f);
        }
    }
    wave_sync();

    // ---- 3. solver view: lane i of group g (= tile g) owns row i of the tile = row ei of sub-system si
    const int g = lane >> 4, i = lane & 15, si = i / G, ei = i % G;
    float s[G];
#pragma unroll
    for (int c = 0; c < G; ++c) s[c] = sb[(g * 16 + i) * KP + si * G + c];
    // this lane's label: the MFMA view of tile g had it in lane (a = i, any q); q == g holds a copy
    float y = 0.f;
#pragma unroll
    for (int p = 0; p < 4; ++p) y = g == p ? yl[p] : y;  // lane (a, q) of tile p == g: a == i because lane = 16 g + i
    float rpm = 1.f;
    bool bad = false;
    static_for<0, G>([&](auto cc) {
        constexpr int c = decltype(cc)::value;
        const float pivot = sub_bcast<G, c>(s[c], upper);
        const float uc = sub_bcast<G, c>(y, upper);
        bad |= !(pivot > 0.f);
        float rp = __builtin_amdgcn_rcpf(pivot);
        rp = rp * (2.f - pivot * rp);  // one Newton step on the hardware reciprocal
        rpm = ei == c ? rp : rpm;
        const float f = ei > c ? s[c] * rp : 0.f;  // M[ei][c]; rows above stay as they are
        y -= f * uc;
        static_for<c + 1, G>([&](auto jj) {
            constexpr int j = decltype(jj)::value;
            s[j] -= f * sub_bcast<G, j>(s[c], upper);
        });
    });
    if (bad) atomicOr(err_flag, 1);
    // factor back to LDS, read transposed: lt[c] = S'[c][ei] of the own sub-system
    wave_sync();
#pragma unroll
    for (int c = 0; c < G; ++c) sb[(g * 16 + i) * KP + si * G + c] = s[c];
    wave_sync();
#pragma unroll
    for (int c = 0; c < G; ++c) s[c] = sb[(g * 16 + si * G + c) * KP + si * G + ei];
    float t = 0.f;
    static_for<0, G>([&](auto cc) {
        constexpr int c = G - 1 - decltype(cc)::value;
        const float tc = sub_bcast<G, c>(y * rpm, upper);
        t = ei == c ? tc : t;
        y -= ei < c ? s[c] * tc : 0.f;
    });
    tb[lane] = t;  // lane 16 g + i holds t of entry slot i of tile g
    wave_sync();   // all reads of sb are done: its space becomes zb

    // ---- 4. r = Z_I^T t, tile by tile through an LDS copy of the tile's entries
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        if (p > 0) wave_sync();  // the previous tile's copy has been read
#pragma unroll
        for (int j = 0; j < NJ; ++j) *(float4 *)(zb + a * ZLDB + (4 * j + q) * 16) = z[p][j];
        wave_sync();
#pragma unroll
        for (int sidx = 0; sidx < SPT; ++sidx) {
            const int rr = p * SPT + sidx;
            const int k = meta[3 * rr + 2];
            const int64_t u = ((int64_t)meta[3 * rr + 1] << 32) | (uint32_t)meta[3 * rr + 0];
            if (u >= 0 && lane * CPL < D) {
                // four slots at a time (slots past the row's k hold t = 0 and zero entries): the LDS reads of a
                // group are issued together, one round trip per group instead of one per entry
                float r0v = 0.f, r1v = 0.f;
#pragma unroll
                for (int h = 0; h < G / 4; ++h) {
                    if (4 * h < k) {  // uniform
                        const float4 tq = *(const float4 *)(tb + p * 16 + sidx * G + 4 * h);
                        const float te[4] = {tq.x, tq.y, tq.z, tq.w};
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            const int e = sidx * G + 4 * h + x;
                            float zz[CPL];
                            row_cols<ZB, CPL>(zb + e * ZLDB, lane, zz);
                            r0v += te[x] * zz[0];
                            if constexpr (CPL == 2) r1v += te[x] * zz[1];
                        }
                    }
                }
                if constexpr (CPL == 2) *(float2 *)(R + u * ldr + 2 * lane) = make_float2(r0v, r1v);
                else R[u * ldr + lane] = r0v;
            }
        }
    }
}

// The two launch forms of a step kernel (see StepGrid): one step per workgroup, or a grid-stride walk from
// step first_blk to the end of the list.
template <int D, int G, bool ZB, bool LOOP>
__global__ __launch_bounds__(64) void dual_small_kernel(const int64_t *__restrict__ indptr,
                                                        const int32_t *__restrict__ indices,
                                                        const float *__restrict__ values,
                                                        const void *__restrict__ Z, float *__restrict__ R,
                                                        int64_t ldr, int64_t r0, const int32_t *__restrict__ list,
                                                        const int32_t *__restrict__ count_ptr, int first_blk,
                                                        int32_t *__restrict__ err_flag) {
    extern __shared__ float lds[];
    constexpr int NR = SmallCfg<D, G>::NR;
    const int count = *count_ptr;
    int blk = first_blk + blockIdx.x;
    if constexpr (!LOOP) {
        if (blk * NR < count) dual_small_step<D, G, ZB>(indptr, indices, values, Z, R, ldr, r0, list, count, err_flag, blk, lds);
    } else {
        for (; blk * NR < count; blk += gridDim.x) {
            dual_small_step<D, G, ZB>(opaque(indptr), opaque(indices), opaque(values), opaque(Z), opaque(R), opaque(ldr), opaque(r0),
                              opaque(list), opaque(count), opaque(err_flag), blk, opaque(lds));
            wave_sync();  // the next step reuses the LDS buffers
        }
    }
}

template <int D, bool ZB>
static void launch_small_typed(const als_csr *Y, const void *Z, float *R, int64_t ldr, int64_t r0, const int32_t *list,
                               const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s) {
    using C = SmallCfg<D, SMALL_G>;
    if (g.known > 0)
        hipLaunchKernelGGL((dual_small_kernel<D, SMALL_G, ZB, false>), dim3(g.known), dim3(64),
                           C::LDS_FLOATS * sizeof(float), s, Y->indptr, Y->indices, Y->values, Z, R, ldr, r0, list,
                           count_dev, 0, err);
    if (g.rest > 0)
        hipLaunchKernelGGL((dual_small_kernel<D, SMALL_G, ZB, true>), dim3(g.rest), dim3(64),
                           C::LDS_FLOATS * sizeof(float), s, Y->indptr, Y->indices, Y->values, Z, R, ldr, r0, list,
                           count_dev, (int)g.known, err);
}

#if SMALL_G == 8
void launch_dual_small8(int d, const als_csr *Y, const void *Z, bool zb16, float *R, int64_t ldr, int64_t r0,
                        const int32_t *list, const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s) {
#else
void launch_dual_small4(int d, const als_csr *Y, const void *Z, bool zb16, float *R, int64_t ldr, int64_t r0,
                        const int32_t *list, const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s) {
#endif
#define ALS_SMALL_CASE(dd)                                                                              \
    case dd:                                                                                            \
        if (zb16 && dd >= 32) launch_small_typed<dd, (dd >= 32)>(Y, Z, R, ldr, r0, list, count_dev, g, err, s); \
        else launch_small_typed<dd, false>(Y, Z, R, ldr, r0, list, count_dev, g, err, s);               \
        break;
    switch (d) { ALS_SMALL_CASE(16) ALS_SMALL_CASE(32) ALS_SMALL_CASE(64) ALS_SMALL_CASE(128) }
#undef ALS_SMALL_CASE
}

}  // namespace als
