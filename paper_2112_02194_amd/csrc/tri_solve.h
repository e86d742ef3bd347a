// One wavefront solves a symmetric positive definite K x K system (K <= 128, a multiple of 16) whose
// lower triangle sits in LDS, row r starting at tri_row(r).  Rows are padded to multiples of sixteen floats:
// a row at or below a panel of 16 columns then holds all 16 of them inside its own storage (beyond its
// diagonal: padding, never used), so a panel is read and written back with 16-byte accesses and no
// per-element test.
//
// Blocked elimination S = M P M^T (M unit lower triangular, P the pivots) with panels of 16 columns.
// Lane i owns rows i and 64+i.  Per panel:
//   1. every lane reads the panel's 16 entries of its rows into registers and the 16 columns are
//      eliminated there: pivot, column entries and right-hand-side entry of a step are read from the
//      owning lanes as wavefront-uniform values (no memory traffic, no synchronisation); the reciprocal
//      pivot of the next step is prepared right after that column's first update; u = M^{-1} y rides
//      along;
//   2. the eliminated entries S' go back to LDS and the trailing matrix is updated there on the matrix
//      cores: for 16 x 16 tiles (ti, tj <= ti) below the panel, S[ti][tj] -= (S' P^{-1})[ti] S'[tj]^T.
//      Lane (a, q) = (lane % 16, lane / 16) of v_mfma_f32_16x16x4f32 supplies A[a][q] and B[q][a] and
//      holds C[4q+v][a]; MFMA e of a tile contracts the panel columns 4q + e, so that every lane fetches
//      its operands of the four MFMAs with one 16-byte read; the tile is computed transposed (A from the
//      column tile's rows, B from the row tile's), so that C[4q+v][a] is row a, columns 4q+v of the tile.
// Then back-substitution t_c = (u_c - sum_{R>c} S'[R][c] t_R) / pivot_c along the rows of the factor in
// LDS, eight rows fetched ahead of the dependent chain; the value just found is read from its lane.
// Panels and steps at or beyond k are skipped: the caller guarantees that rows >= k are identity rows
// with zero right-hand side.  y0 / y1: right-hand-side entries of rows lane / 64+lane.  On exit
// tbuf[0..K) holds the solution.  A non-positive pivot sets bit 0 of *err_flag.
#pragma once

#include "dual_common.h"

namespace als {

// first float of row r in the padded triangle; tri_row(K) is the size of the whole triangle
__host__ __device__ constexpr int tri_row(int r) { return 16 * (r / 16 + 1) * (8 * (r / 16) + r % 16); }

constexpr int TRI_AUX_FLOATS = 192;  // reciprocal pivots [128]; the other 64 are the callers' per-lane dump slots

__device__ __forceinline__ float lane_value(float v, int src_lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src_lane));
}

// v with the wavefront-uniform value `uniform` put into lane DST (one instruction; the lane is a constant, so
// the instruction's wait states for a lane select computed just before do not apply)
template <int DST> __device__ __forceinline__ float lane_set(float v, float uniform) {
    asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(v) : "s"(uniform), "n"(DST));
    return v;
}

template <int K>
__device__ __forceinline__ void tri_solve(float *tri, float *aux /* [192] */, float *tbuf /* [K] */, float y0,
                                          float y1, int k, int32_t *err_flag) {
    static_assert(K % 16 == 0 && K >= 16 && K <= 128, "unsupported system size");
    constexpr bool TWO = K > 64;
    constexpr int NT = K / 16;
    const int lane = opaque_tid() & 63;
    const int ra = lane, rb = 64 + lane;
    const bool hasa = ra < K, hasb = TWO && rb < K;
    const int a = lane & 15, q = lane >> 4;
    float *rpbuf = aux;
    float *rowa = tri + tri_row(hasa ? ra : 0), *rowb = tri + tri_row(hasb ? rb : 0);
    float rp0 = 1.f, rp1 = 1.f;
    static_for<0, NT>([&](auto pp) {
        constexpr int p = decltype(pp)::value;
        constexpr int P0 = 16 * p;
        constexpr bool OB = P0 >= 64;  // the panel's pivot rows belong to the second set of rows
        if (P0 < k) {
            // Every lane reads 16 floats at the panel's columns of its rows.  What is not an entry of the matrix
            // there (beyond a row's diagonal; a row above the panel; a lane without a row) is never used: the
            // multipliers below are taken only for rows under the pivot, lane reads only go to lanes whose entry
            // exists, and only rows at or below the panel are written back.
            float xa[16], xb[16];
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                float4 va = make_float4(0.f, 0.f, 0.f, 0.f), vb = va;
                if constexpr (!OB) va = *(const float4 *)(rowa + P0 + 4 * c4);
                if constexpr (TWO) vb = *(const float4 *)(rowb + P0 + 4 * c4);
                xa[4 * c4] = va.x; xa[4 * c4 + 1] = va.y; xa[4 * c4 + 2] = va.z; xa[4 * c4 + 3] = va.w;
                xb[4 * c4] = vb.x; xb[4 * c4 + 1] = vb.y; xb[4 * c4 + 2] = vb.z; xb[4 * c4 + 3] = vb.w;
            }
            // reciprocal pivot and right-hand-side entry of a step are prepared during the step before
            // (right after its first update), off the critical path
            float rp, uc;
            auto prepare = [&](auto cc) {
                constexpr int c = decltype(cc)::value;
                constexpr int ol = (P0 + c) & 63;
                const float pivot = lane_value(OB ? xb[c] : xa[c], ol);
                rp = __builtin_amdgcn_rcpf(pivot);
                rp = rp * (2.f - pivot * rp);  // one Newton step on the hardware reciprocal
                if constexpr (OB) rp1 = lane == ol ? rp : rp1;
                else rp0 = lane == ol ? rp : rp0;
            };
            prepare(std::integral_constant<int, 0>{});
            static_for<0, 16>([&](auto cc) {
                constexpr int c = decltype(cc)::value;
                constexpr int col = P0 + c, ol = col & 63;
                if (col < k) {
                    const float own = OB ? xb[c] : xa[c];
                    float cv[16];
#pragma unroll
                    for (int j = c + 1; j < 16; ++j) cv[j] = lane_value(own, (P0 + j) & 63);
                    uc = lane_value(OB ? y1 : y0, ol);
                    float fa = 0.f, fb = 0.f;
                    if constexpr (!OB) {
                        fa = ra > col ? xa[c] * rp : 0.f;
                        y0 -= fa * uc;
                    }
                    if constexpr (TWO) {
                        fb = (!OB || rb > col) ? xb[c] * rp : 0.f;
                        y1 -= fb * uc;
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (c < 15) {
                        if constexpr (!OB) xa[c + 1] -= fa * cv[c + 1];
                        if constexpr (TWO) xb[c + 1] -= fb * cv[c + 1];
                        prepare(std::integral_constant<int, c + 1>{});
#pragma unroll
                        for (int j = c + 2; j < 16; ++j) {
                            if constexpr (!OB) xa[j] -= fa * cv[j];
                            if constexpr (TWO) xb[j] -= fb * cv[j];
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            });
            if constexpr (!OB) {
                if (hasa && ra >= P0) {
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4)
                        *(float4 *)(rowa + P0 + 4 * c4) = make_float4(xa[4 * c4], xa[4 * c4 + 1], xa[4 * c4 + 2], xa[4 * c4 + 3]);
                }
            }
            if constexpr (TWO) {
                if (hasb && rb >= P0) {
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4)
                        *(float4 *)(rowb + P0 + 4 * c4) = make_float4(xb[4 * c4], xb[4 * c4 + 1], xb[4 * c4 + 2], xb[4 * c4 + 3]);
                }
            }
            rpbuf[lane] = rp0;
            if constexpr (TWO) rpbuf[64 + lane] = rp1;
            wave_sync();
            if constexpr (p + 1 < NT) {
                constexpr int T = NT - p - 1;
                const float4 rpv = *(const float4 *)(rpbuf + P0 + 4 * q);
                float4 z[T];
#pragma unroll
                for (int t = 0; t < T; ++t) z[t] = *(const float4 *)(tri + tri_row(16 * (p + 1 + t) + a) + P0 + 4 * q);
                static_for<0, T>([&](auto tii) {
                    constexpr int ti = decltype(tii)::value;
                    const float4 za = make_float4(-z[ti].x * rpv.x, -z[ti].y * rpv.y, -z[ti].z * rpv.z, -z[ti].w * rpv.w);
                    // all tiles of the tile row are fetched before the first is stored back.  The operands are taken
                    // in the order that leaves a lane with four consecutive columns of ONE row of the tile (row
                    // 16 (p+1+ti) + a, columns 16 (p+1+tj) + 4q ..): one 16-byte access each way; in a diagonal tile
                    // the columns beyond the diagonal belong to the row's padding
                    floatx4 acc[ti + 1];
                    float4 *cell[ti + 1];
#pragma unroll
                    for (int tj = 0; tj <= ti; ++tj) {
                        cell[tj] = (float4 *)(tri + tri_row(16 * (p + 1 + ti) + a) + 16 * (p + 1 + tj) + 4 * q);
                        const float4 c4 = *cell[tj];
                        acc[tj] = floatx4{c4.x, c4.y, c4.z, c4.w};
                    }
#pragma unroll
                    for (int tj = 0; tj <= ti; ++tj) acc[tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[tj].x, za.x, acc[tj], 0, 0, 0);
#pragma unroll
                    for (int tj = 0; tj <= ti; ++tj) acc[tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[tj].y, za.y, acc[tj], 0, 0, 0);
#pragma unroll
                    for (int tj = 0; tj <= ti; ++tj) acc[tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[tj].z, za.z, acc[tj], 0, 0, 0);
#pragma unroll
                    for (int tj = 0; tj <= ti; ++tj) acc[tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[tj].w, za.w, acc[tj], 0, 0, 0);
#pragma unroll
                    for (int tj = 0; tj <= ti; ++tj) *cell[tj] = make_float4(acc[tj][0], acc[tj][1], acc[tj][2], acc[tj][3]);
                });
                wave_sync();
            }
        }
    });
    // A pivot that is not positive shows in its reciprocal, which the owning lane has kept: negative stays
    // negative, zero and NaN come out of the Newton step as NaN.
    if (__any(!(rp0 > 0.f) || !(rp1 > 0.f)) && lane == 0) atomicOr(err_flag, 1);

    // ---- back-substitution, eight rows of the factor fetched ahead of the dependent chain.  Every lane reads
    // row R at its own column: lanes at or beyond R have their unknown already and go on computing on
    // whatever lies there (the row's padding, later rows, at most the first 127 floats after the triangle,
    // which every caller's LDS layout has).  Groups of rows at or beyond k hold t = 0.
    float t0 = 0.f, t1v = 0.f;
    static_for<0, K / 8>([&](auto gg) {
        constexpr int Rt = K - 1 - 8 * decltype(gg)::value;  // the group's last row; rows Rt-7 .. Rt
        if (Rt - 7 < k) {
            float fa[8], fb[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int Rr = Rt - i;
                const float *row = tri + tri_row(Rr);
                fa[i] = row[lane];
                if (Rr >= 64) fb[i] = row[64 + lane];
            }
            static_for<0, 8>([&](auto ii) {
                constexpr int i = decltype(ii)::value, Rr = Rt - i;
                if constexpr (Rr >= 64) {
                    const float tR = lane_value(y1 * rp1, Rr - 64);
                    t1v = lane_set<Rr - 64>(t1v, tR);
                    y1 -= fb[i] * tR;
                    y0 -= fa[i] * tR;
                } else {
                    const float tR = lane_value(y0 * rp0, Rr);
                    t0 = lane_set<Rr>(t0, tR);
                    y0 -= fa[i] * tR;
                }
            });
        }
    });
    if (hasa) tbuf[ra] = t0;
    if (hasb) tbuf[rb] = t1v;
    wave_sync();
}
}  // namespace als
