// One wavefront solves a symmetric positive definite K x K system (K <= 128, a multiple of 16) by conjugate
// gradients (the solver Section 4.5 settles on), on the same LDS layout as tri_solve.h: lower triangle, row r
// starting at tri_row(r).  Lane i owns rows i and 64+i of every vector.  The product S p reads row i up to the
// diagonal and column i below it (S is symmetric), p from an LDS copy.  Starts from zero, stops when
// |residual| <= tol * |y| or after max_iters steps.  Rows at or beyond k are identity rows with zero
// right-hand side (the caller guarantees it): their unknowns are zero and they are left out of the products.
// y0 / y1: right-hand-side entries of rows lane / 64+lane.  pbuf: K floats of LDS.  On exit tbuf[0..K) holds
// the solution.
#pragma once

#include "tri_solve.h"

namespace als {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;  // the same bits in every lane
}

template <int K>
__device__ __forceinline__ void tri_cg(const float *tri, float *pbuf, float *tbuf, float y0, float y1, int k,
                                       int max_iters, float tol) {
    static_assert(K % 16 == 0 && K >= 16 && K <= 128, "unsupported system size");
    constexpr bool TWO = K > 64;
    const int lane = opaque_tid() & 63;
    const bool hasa = lane < k, hasb = TWO && 64 + lane < k;
    const int ra = hasa ? lane : 0, rb = hasb ? 64 + lane : 0;  // lanes without a row read row 0 and drop the result
    const int rowa = tri_row(ra), rowb = tri_row(rb);
    float x0 = 0.f, x1 = 0.f;
    float r0 = hasa ? y0 : 0.f, r1 = hasb ? y1 : 0.f;
    float p0 = r0, p1 = r1;
    float rs = wave_sum(r0 * r0 + r1 * r1);
    const float stop = fmaxf(tol * tol * rs, CG_RESIDUAL_FLOOR);
    for (int it = 0; it < max_iters && rs > stop; ++it) {
        if (lane < K) pbuf[lane] = p0;
        if (TWO && 64 + lane < K) pbuf[64 + lane] = p1;
        wave_sync();
        float a0 = 0.f, a1 = 0.f;
        for (int j = 0; j < k; ++j) {
            const float pj = pbuf[j];
            const int rj = tri_row(j);
            a0 += tri[j <= ra ? rowa + j : rj + ra] * pj;
            if constexpr (TWO) a1 += tri[j <= rb ? rowb + j : rj + rb] * pj;
        }
        a0 = hasa ? a0 : 0.f;
        a1 = hasb ? a1 : 0.f;
        const float pap = wave_sum(p0 * a0 + p1 * a1);
        if (!(pap > 0.f)) break;  // only when the numbers have left the fp32 range; the same in every lane
        const float alpha = rs / pap;
        x0 += alpha * p0;
        x1 += alpha * p1;
        r0 -= alpha * a0;
        r1 -= alpha * a1;
        const float rs_new = wave_sum(r0 * r0 + r1 * r1);
        const float beta = rs_new / rs;
        p0 = r0 + beta * p0;
        p1 = r1 + beta * p1;
        rs = rs_new;
        wave_sync();  // pbuf is rewritten by the next step
    }
    if (lane < K) tbuf[lane] = x0;
    if (TWO && 64 + lane < K) tbuf[64 + lane] = x1;
    wave_sync();
}
}  // namespace als
