// One wavefront solves a symmetric positive definite K x K system (K <= 128, a multiple of 4) whose
// lower triangle sits in LDS, row r starting at tri_row(r) (rows padded to multiples of four floats so
// that a row can be read with aligned 16-byte broadcast reads).
//
// Block elimination S = M P M^T (M unit lower triangular, P the pivots) with 64 x 64 blocks
//     S = | S11      |      rows 0..63  : lane i owns row i
//         | S21  S22 |      rows 64..K-1: lane i owns row 64+i
//   1. S11 is eliminated column by column with the rows in registers; every lane also carries its row
//      of S21 through the same column operations, which turns it into the matching row of M21 P1;
//      u = M^{-1} y rides along.  Pivot, column entries and right-hand-side entry of a step are read
//      from the owning lanes as wavefront-uniform values.
//   2. S22 -= M21 P1 M21^T as 16 x 16 tiles on the matrix cores, operands and tiles in LDS.
//   3. S22 is eliminated like S11.
//   4. Back-substitution t_c = (u_c - sum_{R>c} S'[R][c] t_R) / pivot_c along the rows of the factor,
//      which the lanes wrote back to LDS; the value just found is read from its lane.
// Steps at or beyond k are skipped: the caller guarantees that rows >= k are identity rows with zero
// right-hand side.  y0 / y1: right-hand-side entries of rows lane / 64+lane.  On exit tbuf[0..K) holds
// the solution.  A non-positive pivot sets bit 0 of *err_flag.
#pragma once

#include "dual_common.h"

namespace als {

// first float of row r in the padded triangle; tri_row(K) is the size of the whole triangle
__host__ __device__ constexpr int tri_row(int r) { return 4 * (r / 4 + 1) * (2 * (r / 4) + r % 4); }

__device__ __forceinline__ float lane_value(float v, int src_lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src_lane));
}

// Right-looking elimination of an N x N diagonal block held one row per lane (s[j] = entry (lane, j),
// j <= lane; lanes >= N hold zeros).  With ATTACHED, g[] holds a second row per lane that lies below
// the block (entries (64+lane, j)) and receives the same column operations.  Step c takes the pivot,
// the column entries (lane j's s[c]) and the right-hand-side entry straight from the owning lanes as
// wavefront-uniform values, so the steps need no memory traffic and no synchronisation (an exchange
// of the column through LDS with broadcast reads was measured slower).  nsteps <= N columns are
// eliminated; rp_own receives, in lane c, the reciprocal of pivot c; y / yg are the right-hand-side
// entries of the two rows.
template <int N, bool ATTACHED>
__device__ __forceinline__ void eliminate_block(float (&s)[N], float (&g)[ATTACHED ? N : 1], float &y, float &yg,
                                                float &rp_own, int nsteps, bool &bad) {
    const int lane = threadIdx.x & 63;
    static_for<0, N>([&](auto cc) {
        constexpr int c = decltype(cc)::value;
        if (c < nsteps) {
            const float pivot = lane_value(s[c], c), uc = lane_value(y, c);
            bad |= !(pivot > 0.f);
            float rp = __builtin_amdgcn_rcpf(pivot);
            rp = rp * (2.f - pivot * rp);  // one Newton step on the hardware reciprocal
            rp_own = lane == c ? rp : rp_own;
            const float f = lane > c ? s[c] * rp : 0.f;  // M[row][c]; rows above stay as they are
            y -= f * uc;
            float fg = 0.f;
            if constexpr (ATTACHED) {
                fg = g[c] * rp;
                yg -= fg * uc;
            }
            // column entries (j, c) eight at a time: the lane reads complete before the first use
            static_for<0, (N - c - 1 + 7) / 8>([&](auto bb) {
                constexpr int j0 = c + 1 + 8 * decltype(bb)::value;
                constexpr int nj = N - j0 < 8 ? N - j0 : 8;
                float col[nj];
#pragma unroll
                for (int i = 0; i < nj; ++i) col[i] = lane_value(s[c], j0 + i);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < nj; ++i) {
                    s[j0 + i] -= f * col[i];
                    if constexpr (ATTACHED) g[j0 + i] -= fg * col[i];
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    });
}

template <int K>
__device__ __forceinline__ void tri_solve(float *tri, float *aux /* [128] */, float *tbuf /* [K] */, float y0,
                                          float y1, int k, int32_t *err_flag) {
    static_assert(K <= 128 && (K <= 64 ? K % 8 == 0 && K >= 8 : K % 16 == 0), "unsupported system size");
    constexpr int N0 = K < 64 ? K : 64;      // rows of block 1
    constexpr int N1 = K > 64 ? K - 64 : 1;  // rows of block 2 (dummy size when there is none)
    constexpr bool TWO = K > 64;
    const int lane = threadIdx.x & 63;
    const int ra = lane, rb = 64 + lane;
    const bool hasa = ra < N0, hasb = TWO && rb < K;
    // lanes without a second row compute on zeros and store into tbuf, which is free until the end
    // (unconditional stores keep the unrolled code free of divergent branches)
    float *rowp = hasb ? tri + tri_row(rb) : tbuf;
    float rp0 = 1.f, rp1 = 1.f;
    bool bad = false;

    // ---- 1./2. block 1, with the S21 rows attached
    float g[TWO ? 64 : 1];
    {
        float s0[N0];
#pragma unroll
        for (int c = 0; c < N0; ++c) s0[c] = (hasa && c <= ra) ? tri[tri_row(ra) + c] : 0.f;
        if constexpr (TWO) {
#pragma unroll
            for (int c = 0; c < 64; ++c) g[c] = hasb ? rowp[c] : 0.f;
        }
        eliminate_block<N0, TWO>(s0, g, y0, y1, rp0, k < N0 ? k : N0, bad);
#pragma unroll
        for (int c = 0; c < N0; ++c)
            if (hasa && c <= ra) tri[tri_row(ra) + c] = s0[c];
    }

    if constexpr (TWO) {
        // ---- 2. S22 -= M21 P1 M21^T on the matrix cores, 16 x 16 tiles (ti, tj <= ti) updated in LDS.
        // Lane (a, q) = (lane % 16, lane / 16) of v_mfma_f32_16x16x4f32 supplies A[a][q] and B[q][a] and
        // holds C[4q+v][a]; step (s, e) of a tile contracts the columns c = 16s + 4q + e, so that every
        // lane fetches its operands of four steps with one 16-byte read:
        //     A = -M21[16ti + a][c] = -S'[64+16ti+a][c] * rp_c,   B = S'[64+16tj+a][c].
        constexpr int NT = N1 / 16;
        const int a = lane & 15, q = lane >> 4;
        float *rpbuf = aux, *dump = aux + 64;
#pragma unroll
        for (int c = 0; c < 64; ++c) rowp[c] = g[c];  // S' rows of block 2, also read by step 4
        rpbuf[lane] = rp0;
        wave_sync();
        float4 z[NT][4], rpv[4];
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            rpv[s4] = *(const float4 *)(rpbuf + 16 * s4 + 4 * q);
#pragma unroll
            for (int t = 0; t < NT; ++t) z[t][s4] = *(const float4 *)(tri + tri_row(64 + 16 * t + a) + 16 * s4 + 4 * q);
        }
        static_for<0, NT>([&](auto tii) {
            constexpr int ti = decltype(tii)::value;
            float4 za[4];
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4)
                za[s4] = make_float4(-z[ti][s4].x * rpv[s4].x, -z[ti][s4].y * rpv[s4].y, -z[ti][s4].z * rpv[s4].z,
                                     -z[ti][s4].w * rpv[s4].w);
            static_for<0, ti + 1>([&](auto tjj) {
                constexpr int tj = decltype(tjj)::value;
                floatx4 acc;
                float *cell[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = 16 * ti + 4 * q + v, col = 16 * tj + a;
                    // entries above the diagonal do not exist: they are computed on zeros and dumped
                    cell[v] = (tj < ti || col <= row) ? tri + tri_row(64 + row) + 64 + col : dump + lane;
                    acc[v] = *cell[v];
                }
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(za[s4].x, z[tj][s4].x, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(za[s4].y, z[tj][s4].y, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(za[s4].z, z[tj][s4].z, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(za[s4].w, z[tj][s4].w, acc, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) *cell[v] = acc[v];
            });
        });
        wave_sync();
        float s1[N1];
#pragma unroll
        for (int c = 0; c < N1; ++c) s1[c] = (hasb && 64 + c <= rb) ? rowp[64 + c] : 0.f;
        // ---- 3. block 2
        float none[1], ynone = 0.f;
        eliminate_block<N1, false>(s1, none, y1, ynone, rp1, k > 64 ? k - 64 : 0, bad);
#pragma unroll
        for (int c = 0; c < N1; ++c)
            if (hasb && 64 + c <= rb) rowp[64 + c] = s1[c];
    }
    wave_sync();
    if (bad && lane == 0) atomicOr(err_flag, 1);

    // ---- 4. back-substitution, eight rows of the factor fetched ahead of the dependent chain
    const int ktop = (k + 7) & ~7;  // rows k..ktop-1 are identity rows with zero right-hand side: t = 0
    float t0 = 0.f, t1v = 0.f;
    if constexpr (TWO) {
#pragma unroll 1
        for (int Rt = ktop - 1; Rt >= 64; Rt -= 8) {
            float fa[8], fb[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int base = tri_row(Rt - i);
                fa[i] = tri[base + ra];
                fb[i] = tri[base + (rb < Rt - i ? rb : 0)];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int Rr = Rt - i;
                const float tR = lane_value(y1 * rp1, Rr - 64);
                t1v = rb == Rr ? tR : t1v;
                y1 -= (rb < Rr ? fb[i] : 0.f) * tR;
                y0 -= fa[i] * tR;
            }
        }
    }
#pragma unroll 1
    for (int Rt = (ktop < N0 ? ktop : N0) - 1; Rt >= 0; Rt -= 8) {
        float fa[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) fa[i] = tri[tri_row(Rt - i) + (ra < Rt - i ? ra : 0)];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int Rr = Rt - i;
            const float tR = lane_value(y0 * rp0, Rr);
            t0 = ra == Rr ? tR : t0;
            y0 -= (ra < Rr ? fa[i] : 0.f) * tR;
        }
    }
    if (hasa) tbuf[ra] = t0;
    if (hasb) tbuf[rb] = t1v;
    wave_sync();
}

}  // namespace als
