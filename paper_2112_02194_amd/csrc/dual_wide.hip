// Dual row update for 32 < k <= 128 (d = 128; k <= 64 also at d = 64), compiled once per class with
// -DWIDE_KT=3..8 (k <= 16*WIDE_KT).  The algebra is in the header comment of dual_prepare.hip.
#include "dual_common.h"
#include "tri_cg.h"
#include "tri_solve.h"

#ifndef WIDE_KT
#error "compile with -DWIDE_KT=3 .. 8"
#endif

namespace als {

// One wavefront per row with k <= K = 16*KT entries (KT = 3..8).
//   1. S = I + Z_I Z_I^T tile by tile: the wavefront keeps the 16 entries of tile t1 in registers (B
//      operand) and streams the tiles t2 <= t1 past them (A operand, fetched again from the caches);
//      each finished 16x16 tile goes to LDS, where S is kept as a lower triangle.
//   2./3. Block elimination S = M P M^T and back-substitution by the wavefront (tri_solve.h).
//   4. r = Z_I^T t: with bf16 Z from the tiles still in registers, on the matrix cores (zt_times_t,
//      dual_common.h: bf16 entries are exact operands); with fp32 Z with D/64 adjacent output columns per lane,
//      gathering the entries a second time (the hi + lo operands kept for S carry z only to 2^-16, which is
//      enough for S = I + Z Z^T but would show in r).
template <int D, int KT, bool ZB> constexpr bool wide_resident() { return ZB; }

template <int D, int KT> struct WideCfg {
    static constexpr int K = 16 * KT;
    static constexpr int TRI = tri_row(K);           // lower triangle, rows padded (tri_solve.h)
    static constexpr int OFF_COL = TRI;              // solver's auxiliary buffer
    static constexpr int OFF_T = OFF_COL + TRI_AUX_FLOATS;  // tbuf[K]
    static constexpr int OFF_ID = OFF_T + K;         // ids[K]
    static constexpr int LDS_FLOATS = OFF_ID + K;
};

// CG: the k x k system is solved by conjugate gradients (tri_cg.h) instead of the panel elimination.
template <int D, int KT, bool ZB, bool CG>
__device__ __forceinline__ void dual_wide_step(const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                                               const float *__restrict__ values, const void *__restrict__ Z,
                                               float *__restrict__ R, int64_t ldr, int64_t r0,
                                               const int32_t *__restrict__ list, int32_t *__restrict__ err_flag,
                                               int item, float *lds, int cg_iters, float cg_tol) {
    using C = WideCfg<D, KT>;
    constexpr int K = C::K, NJ = z_pieces<D, ZB>();
    constexpr bool RES = wide_resident<D, KT, ZB>();
    float *tri = lds, *aux = lds + C::OFF_COL, *tbuf = lds + C::OFF_T;
    int32_t *ids = (int32_t *)(lds + C::OFF_ID);
    const int lane = opaque_tid(), a = lane & 15, q = lane >> 4;
    const int64_t u = r0 + list[item];
    const int64_t b = indptr[u];
    const int k = (int)(indptr[u + 1] - b);  // <= K by the list's class

    // ---- 1. S tiles
    int32_t myid[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t) {
        const int e = 16 * t + a;
        const int32_t id = indices[b + (e < k ? e : 0)];  // a slot past k: the row's first entry (meets t = 0 below)
        myid[t] = e < k ? id : (id | (int32_t)0x80000000);  // a padded slot: negative, and still a row of the table
        if (!RES && q == 0) ids[e] = id;
    }
    // the first RT tiles stay in registers for the whole phase (one round of loads, all in flight
    // together), already cut into the hi/lo bf16 operands of the split products (dual_common.h); later
    // tiles are fetched and cut when they are needed
    constexpr int RT = RES ? KT : (KT < 5 ? KT : (KT < 7 ? 5 : 4));
    typedef TileOperand<D, ZB> Op;
    auto fetch = [&](int t, float4 (&raw)[NJ]) {
        // with the direct solver the class holds rows with more than 16 (KT - 1) entries only: all tiles but the
        // last are full (under CG shorter rows come through the same kernel)
        if (!CG && t < KT - 1) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) raw[j] = load_piece<D, ZB>(Z, myid[t] & 0x7fffffff, j, q);
        } else {
#pragma unroll
            for (int j = 0; j < NJ; ++j) raw[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (myid[t] >= 0) {  // one masked region per tile, not one per load
#pragma unroll
                for (int j = 0; j < NJ; ++j) raw[j] = load_piece<D, ZB>(Z, myid[t], j, q);
            }
        }
    };
    Op zop[RT];
    {
        float4 raw[RT][NJ];
#pragma unroll
        for (int t = 0; t < RT; ++t) fetch(t, raw[t]);
#pragma unroll
        for (int t = 0; t < RT; ++t) zop[t].set(raw[t]);
    }
#pragma unroll
    for (int t1 = 0; t1 < KT; ++t1) {
        Op zb;
        if (t1 < RT) {
            zb = zop[t1 < RT ? t1 : 0];
        } else {
            float4 raw[NJ];
            fetch(t1, raw);
            zb.set(raw);
        }
#pragma unroll
        for (int t2 = 0; t2 <= t1; ++t2) {
            floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
            if (t2 == t1) {
                acc = tile_product<D, ZB>(zb, zb, acc);
            } else if (t2 < RT) {
                acc = tile_product<D, ZB>(zop[t2 < RT ? t2 : 0], zb, acc);
            } else {
                float4 raw[NJ];
                fetch(t2, raw);
                Op za;
                za.set(raw);
                acc = tile_product<D, ZB>(za, zb, acc);
            }
            // acc[v] = S[Rr][c], Rr = 16*t1 + a, c = 16*t2 + 4q + v (S is symmetric).  The triangle's rows are
            // padded to whole tiles, so a diagonal tile is stored whole: what lies beyond the diagonal lands in
            // the row's padding
            const int Rr = 16 * t1 + a, c0 = 16 * t2 + 4 * q;
            if (t2 == t1) {  // known after unrolling: the identity only meets diagonal tiles
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[v] += c0 + v == Rr ? 1.f : 0.f;
            }
            *(float4 *)(tri + tri_row(Rr) + c0) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        }
    }
    wave_sync();

    // ---- 2./3. elimination and back-substitution (tri_solve.h); lane i holds the labels of entries i, 64+i
    {
        float y0 = 0.f, y1 = 0.f;
        if (lane < k) y0 = values ? values[b + lane] : 1.f;
        if (64 + lane < k) y1 = values ? values[b + 64 + lane] : 1.f;
        if constexpr (CG) tri_cg<K>(tri, aux, tbuf, y0, y1, k, cg_iters, cg_tol);
        else tri_solve<K>(tri, aux, tbuf, y0, y1, k, err_flag);
    }

    // ---- 4. r = Z_I^T t
    if constexpr (RES) {
        // the triangle is free now: the remainders of the cut of t, a block of zeros and the finished row go there
        static_assert(tri_row(K) >= 3 * K + D, "the triangle area holds the parts of t and the row");
        float *p1 = tri, *p2 = tri + K, *zeros = tri + 2 * K, *rbuf = tri + 3 * K;
#pragma unroll
        for (int e0 = 0; e0 < K; e0 += 64) {
            const int e = e0 + lane;
            if (e < K) {
                float x1, x2;
                t_parts(tbuf[e], x1, x2);
                p1[e] = x1;
                p2[e] = x2;
                zeros[e] = 0.f;
            }
        }
        const SelOperands sel = make_sel(lane);
        wave_sync();
        const float *mine = (a == 0 ? tbuf : (a == 1 ? p1 : (a == 2 ? p2 : zeros))) + 4 * q;
        bf16x8 top[(KT + 1) / 2];
#pragma unroll
        for (int P = 0; P < (KT + 1) / 2; ++P) top[P] = t_operand(mine + 32 * P, 2 * P + 1 < KT);
        constexpr int NP = D / 32;
        floatx4 out[2 * NP];
#pragma unroll
        for (int x = 0; x < 2 * NP; ++x) out[x] = floatx4{0.f, 0.f, 0.f, 0.f};
        if constexpr (ZB)
            zt_times_t<KT, NP>([&](int t, int j) { return __builtin_bit_cast(bf16x8, zop[t].v[j]); }, top, sel, out);
        float *dump = aux + 128 + lane;  // the solver's per-lane dump slots
#pragma unroll
        for (int x = 0; x < 2 * NP; ++x)
            *(q == 0 ? rbuf + column_of_result(x >> 1, x & 1, a) : dump) = out[x][0] + out[x][1] + out[x][2];
        wave_sync();
        if constexpr (D >= 128) *(float2 *)(R + u * ldr + 2 * lane) = *(const float2 *)(rbuf + 2 * lane);
        else R[u * ldr + lane] = rbuf[lane];
    } else {
        constexpr int CPL = D / 64;
        float rv[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) rv[c] = 0.f;
        const int kp8 = (k + 7) & ~7;  // padded entries have t = 0 and the id of the row's first entry
        for (int e0 = 0; e0 < kp8; e0 += 8) {
            float zz[8][CPL];
            // ids and t of the round with 16-byte LDS reads, before the first load is issued
            const int4 ia = *(const int4 *)(ids + e0), ib = *(const int4 *)(ids + e0 + 4);
            const float4 ta = *(const float4 *)(tbuf + e0), tb = *(const float4 *)(tbuf + e0 + 4);
            const int idr[8] = {ia.x, ia.y, ia.z, ia.w, ib.x, ib.y, ib.z, ib.w};
            const float te[8] = {ta.x, ta.y, ta.z, ta.w, tb.x, tb.y, tb.z, tb.w};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int id = idr[i];
                row_cols<ZB, CPL>((const char *)Z + (int64_t)id * D * ZT<ZB>::ES, lane, zz[i]);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int c = 0; c < CPL; ++c) rv[c] += te[i] * zz[i][c];
        }
        if constexpr (CPL == 2) *(float2 *)(R + u * ldr + 2 * lane) = make_float2(rv[0], rv[1]);
        else R[u * ldr + lane] = rv[0];
    }
}

// The two launch forms of a step kernel (see StepGrid): one row per workgroup, or a grid-stride walk from
// row first_item to the end of the list.
template <int D, int KT, bool ZB, bool LOOP, bool CG>
__global__ __launch_bounds__(64, (LOOP || KT >= 7) ? 1 : (KT <= 4 ? 3 : 2)) void dual_wide_kernel(const int64_t *__restrict__ indptr,
                                                          const int32_t *__restrict__ indices,
                                                          const float *__restrict__ values,
                                                          const void *__restrict__ Z, float *__restrict__ R,
                                                          int64_t ldr, int64_t r0, const int32_t *__restrict__ list,
                                                          const int32_t *__restrict__ count_ptr, int first_item,
                                                          int32_t *__restrict__ err_flag, int cg_iters, float cg_tol) {
    extern __shared__ float lds[];
    const int count = *count_ptr;
    int item = first_item + blockIdx.x;
    if constexpr (!LOOP) {
        if (item < count)
            dual_wide_step<D, KT, ZB, CG>(indptr, indices, values, Z, R, ldr, r0, list, err_flag, item, lds, cg_iters, cg_tol);
    } else {
        for (; item < count; item += gridDim.x) {
            dual_wide_step<D, KT, ZB, CG>(opaque(indptr), opaque(indices), opaque(values), opaque(Z), opaque(R),
                                          opaque(ldr), opaque(r0), opaque(list), opaque(err_flag), item, opaque(lds),
                                          opaque(cg_iters), opaque(cg_tol));
            wave_sync();  // the next step reuses the LDS buffers
        }
    }
}

#define ALS_WIDE_NAME2(kt) launch_dual_wide##kt
#define ALS_WIDE_NAME(kt) ALS_WIDE_NAME2(kt)

template <int D, bool ZB>
static als_status wide_typed(als_ctx *ctx, const als_csr *Y, const void *Z, float *R, int64_t ldr, int64_t r0,
                             const int32_t *list, const int32_t *count_dev, StepGrid g, int32_t *err, const WideSolver &ws,
                             hipStream_t s) {
    using C = WideCfg<D, WIDE_KT>;
    constexpr int lds_bytes = (int)(C::LDS_FLOATS * sizeof(float));
    if (ws.cg) {  // only the grid-stride form exists with this solver: one launch covers the list
        auto kern_cg = dual_wide_kernel<D, WIDE_KT, ZB, true, true>;
        static const hipError_t attr_cg =
            hipFuncSetAttribute((const void *)kern_cg, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        ALS_HIP(ctx, attr_cg);
        hipLaunchKernelGGL(kern_cg, dim3(g.known + g.rest), dim3(64), lds_bytes, s, Y->indptr, Y->indices, Y->values, Z,
                           R, ldr, r0, list, count_dev, 0, err, ws.iters, ws.tol);
        return ALS_OK;
    }
    auto kern = dual_wide_kernel<D, WIDE_KT, ZB, false, false>;
    auto kern_loop = dual_wide_kernel<D, WIDE_KT, ZB, true, false>;
    static const hipError_t attr = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    static const hipError_t attr_loop =
        hipFuncSetAttribute((const void *)kern_loop, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);  // both once per process
    ALS_HIP(ctx, attr);
    ALS_HIP(ctx, attr_loop);
    if (g.known > 0)
        hipLaunchKernelGGL(kern, dim3(g.known), dim3(64), lds_bytes, s, Y->indptr, Y->indices, Y->values, Z, R, ldr, r0,
                           list, count_dev, 0, err, 0, 0.f);
    if (g.rest > 0)
        hipLaunchKernelGGL(kern_loop, dim3(g.rest), dim3(64), lds_bytes, s, Y->indptr, Y->indices, Y->values, Z, R, ldr,
                           r0, list, count_dev, (int)g.known, err, 0, 0.f);
    return ALS_OK;
}

als_status ALS_WIDE_NAME(WIDE_KT)(als_ctx *ctx, int d, const als_csr *Y, const void *Z, bool zb16, float *R, int64_t ldr,
                                  int64_t r0, const int32_t *list, const int32_t *count_dev, StepGrid g,
                                  int32_t *err, const WideSolver &ws, hipStream_t s) {
    if (g.known == 0 && g.rest == 0) return ALS_OK;
    if (d == 128)
        return zb16 ? wide_typed<128, true>(ctx, Y, Z, R, ldr, r0, list, count_dev, g, err, ws, s)
                    : wide_typed<128, false>(ctx, Y, Z, R, ldr, r0, list, count_dev, g, err, ws, s);
    if constexpr (WIDE_KT <= 4) {  // the dual form reaches k <= 64 at d = 64
        if (d == 64)
            return zb16 ? wide_typed<64, true>(ctx, Y, Z, R, ldr, r0, list, count_dev, g, err, ws, s)
                        : wide_typed<64, false>(ctx, Y, Z, R, ldr, r0, list, count_dev, g, err, ws, s);
    }
    return fail(ctx, ALS_EDTYPE, "wide dual kernel: unsupported d");
}

}  // namespace als
