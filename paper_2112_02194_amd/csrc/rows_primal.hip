// Primal row update: the d x d normal equations of the paper's Eq. 4, formed and solved per row
// exactly in the order of Algorithm 1 lines 4-10:
//     A = alpha*G + lambda*I ;  b = 0
//     for every stored (u, i, y):  A += v_i (x) v_i ;  b += y * v_i
//     x_u = A^{-1} b            (Cholesky, A is symmetric positive definite because lambda > 0)
//
// One workgroup owns one row (or one segment of a long row).  The gathered rows of the fixed
// table go straight from global memory into MFMA operand registers (no staging): lane (m, kk)
// loads the NC consecutive columns NC*m.. of the kk-th entry of the current step, wavefront I of
// the workgroup accumulates tile-row I of V_I^T V_I (see Geo<>).  The finished tiles are written
// to LDS together with alpha*G + lambda*I, factorised there, and the two triangular solves give
// the new row, which is rounded once to the table's element type.
//
// Rows longer than `split` are cut into segments (the counterpart of the paper's Section 4.3 row
// splitting): each segment's partial statistics go to a workspace and a second kernel sums them
// in a fixed order before the same factorisation.
#include <type_traits>

#include "dual_common.h"
#include "tri_solve.h"

namespace als {

template <int D> struct Team {
    static constexpr int WAVES = Geo<D>::NC;      // one wavefront per tile-row
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int LD = D + 1;              // LDS leading dimension (odd: conflict-free both ways)
    static constexpr size_t LDS_BYTES = (size_t)(D * LD + 6 * D + 8) * sizeof(float);
};

// ---------------------------------------------------------------------------------------------- accumulate
// Accumulates, for entries [begin, end) of the CSR arrays, tile-row `I` of sum v (x) v into acc[]
// and, in the wavefront of tile-row 0 only, this lane's share of sum y*v into bsum[] (lane (m,kk) holds
// columns NC*m.. of entries kk mod KS).
template <int D, bool BF16>
__device__ __forceinline__ void accumulate_entries(const void *__restrict__ V, int64_t ld,
                                                   const int32_t *__restrict__ indices,
                                                   const float *__restrict__ values, int64_t begin, int64_t end,
                                                   int I, typename AccT<Geo<D>::ACC>::type (&acc)[Geo<D>::NC],
                                                   float (&bsum)[Geo<D>::NC]) {
    using G = Geo<D>;
    constexpr int NC = G::NC, TM = G::TM, KS = G::KS, U = 8;
    const int lane = opaque_tid() & 63;
    const int m = lane % TM, kk = lane / TM;
    const uint32_t ld32 = (uint32_t)ld;  // the leading dimension fits 32 bits (checked on the host)
    const bool first_row = __builtin_amdgcn_readfirstlane(I) == 0;
    for (int64_t base = begin; base < end; base += 64) {
        const int64_t p = base + lane;
        const int myidx = p < end ? indices[p] : -1;
        const float myy = p < end ? (values ? values[p] : 1.f) : 0.f;
        const int cnt = (int)((end - base) < 64 ? (end - base) : 64);
        const int nsteps = (cnt + KS - 1) / KS;
        for (int s0 = 0; s0 < nsteps; s0 += U) {
            // all lane exchanges of the batch first, then all loads: one wait instead of one per load
            int idx[U];
            float x[U][NC], y[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int e = (s0 + u) * KS + kk;
                idx[u] = __shfl(myidx, e & 63);
                y[u] = __shfl(myy, e & 63);
            }
            if ((s0 + U) * KS <= cnt) {  // uniform: every slot of the batch holds an entry
#pragma unroll
                for (int u = 0; u < U; ++u)
                    load_vec<NC, BF16>(V, (int64_t)((uint64_t)(uint32_t)idx[u] * ld32) + NC * m, x[u]);
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool have = (s0 + u) * KS + kk < cnt;
                    y[u] = have ? y[u] : 0.f;
                    if (have) {
                        load_vec<NC, BF16>(V, (int64_t)((uint64_t)(uint32_t)idx[u] * ld32) + NC * m, x[u]);
                    } else {
#pragma unroll
                        for (int c = 0; c < NC; ++c) x[u][c] = 0.f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float a = x[u][0];
#pragma unroll
                for (int c = 1; c < NC; ++c) a = (I == c) ? x[u][c] : a;
#pragma unroll
                for (int j = 0; j < NC; ++j) acc[j] = mfma<D>(a, x[u][j], acc[j]);
            }
            if (first_row) {  // scalar branch: only the wavefront of tile-row 0 carries the right-hand side
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int j = 0; j < NC; ++j) bsum[j] += y[u] * x[u][j];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------- accumulate, bf16 tables
// The same statistics for bf16 tables with d = 64 or 128 on the bf16 matrix cores (16 times the fp32 rate;
// bf16 x bf16 products are exact in fp32, so nothing changes numerically except the order of the sums).  A
// step takes 32 entries: lane (m, kq) loads columns 16 c + 8 kq .. of entry m (16 bytes per piece); the
// matrix core transposes each 32-column block by a product with a constant 0/1 selection operand (see
// gramian_bf16_kernel: exact), the packed results are the K-contiguous operands (K = the step's entries) of
// the block products V_I^T V_I.  Every wavefront gathers and transposes all entries but owns only the block
// pairs p with p % 4 == wave of the upper block triangle (ten pairs at d = 128, three at d = 64), so that it
// carries at most three accumulator tiles.  b = sum y v is formed by wavefront 0 from the transposed fp32
// values.  On return acc[p / 4] holds pair p = (gi, gj): element v of lane (m, kq) is entry
// (32 gi + 8 (v / 4) + 4 kq + v % 4, 32 gj + m); lanes with kq == 0 of wavefront 0 hold b[32 g + m] in bsum[g].
template <int D> struct BlockPairs {
    static constexpr int NB = D / 32, COUNT = NB * (NB + 1) / 2;
    static constexpr int first(int p) {  // pairs in the order (0,0) (0,1) .. (0,NB-1) (1,1) ..
        int g = 0;
        while (p >= NB - g) {
            p -= NB - g;
            ++g;
        }
        return g;
    }
    static constexpr int second(int p) {
        int g = 0;
        while (p >= NB - g) {
            p -= NB - g;
            ++g;
        }
        return g + p;
    }
};

template <int D>
__device__ __forceinline__ void accumulate_entries_bf16(const uint16_t *__restrict__ V, int64_t ld,
                                                        const int32_t *__restrict__ indices,
                                                        const float *__restrict__ values, int64_t begin, int64_t end,
                                                        int wave, floatx16 (&acc)[3], float (&bsum)[4]) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    using BP = BlockPairs<D>;
    constexpr int NB = D / 32, NCH = D / 16;
    const int lane = opaque_tid() & 63, m = lane & 31, kq = lane >> 5;
    const uint32_t ld32 = (uint32_t)ld;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    bf16x8 sel[2];  // selection operands: sel[h] has a one at (k, 16 h + k)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        u32x4 w = {0u, 0u, 0u, 0u};
        const int k = m - 16 * h - 8 * kq;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (k == e) w[e / 2] = (e & 1) ? 0x3F800000u : 0x00003F80u;
        sel[h] = __builtin_bit_cast(bf16x8, w);
    }
    for (int64_t base = begin; base < end; base += 64) {
        const int64_t p = base + lane;
        const int myidx = p < end ? indices[p] : -1;
        const float myy = p < end ? (values ? values[p] : 1.f) : 0.f;
        const int cnt = (int)((end - base) < 64 ? (end - base) : 64);
        for (int s0 = 0; s0 < cnt; s0 += 32) {
            const int idx = __shfl(myidx, s0 + m);
            u32x4 raw[NCH];
#pragma unroll
            for (int c = 0; c < NCH; ++c) raw[c] = u32x4{0u, 0u, 0u, 0u};
            if (idx >= 0) {
                const uint16_t *row = V + (int64_t)((uint64_t)(uint32_t)idx * ld32) + 8 * kq;
#pragma unroll
                for (int c = 0; c < NCH; ++c) raw[c] = *(const u32x4 *)(row + 16 * c);
            }
            bf16x8 op[NB][2];
#pragma unroll
            for (int g = 0; g < NB; ++g) {
                floatx16 t;
#pragma unroll
                for (int v = 0; v < 16; ++v) t[v] = 0.f;
                t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw[2 * g]), sel[0], t, 0, 0, 0);
                t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw[2 * g + 1]), sel[1], t, 0, 0, 0);
                // t[v] = V[entry s0 + 8 (v / 4) + 4 kq + v % 4][32 g + m]
#pragma unroll
                for (int x = 0; x < 2; ++x) {
                    const u32x4 w = {__builtin_amdgcn_perm(__float_as_uint(t[8 * x + 1]), __float_as_uint(t[8 * x + 0]), 0x07060302u),
                                     __builtin_amdgcn_perm(__float_as_uint(t[8 * x + 3]), __float_as_uint(t[8 * x + 2]), 0x07060302u),
                                     __builtin_amdgcn_perm(__float_as_uint(t[8 * x + 5]), __float_as_uint(t[8 * x + 4]), 0x07060302u),
                                     __builtin_amdgcn_perm(__float_as_uint(t[8 * x + 7]), __float_as_uint(t[8 * x + 6]), 0x07060302u)};
                    op[g][x] = __builtin_bit_cast(bf16x8, w);
                }
                if (wave_s == 0) {  // scalar branch: the right-hand side rides in wavefront 0
                    if (values) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) bsum[g] += __shfl(myy, s0 + 8 * (v >> 2) + 4 * kq + (v & 3)) * t[v];
                    } else {  // y = 1; slots without an entry hold zeros
#pragma unroll
                        for (int v = 0; v < 16; ++v) bsum[g] += t[v];
                    }
                }
            }
            static_for<0, BP::COUNT>([&](auto pp) {
                constexpr int pr = decltype(pp)::value, gi = BP::first(pr), gj = BP::second(pr);
                if (wave_s == pr % 4) {
                    acc[pr / 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[gi][0], op[gj][0], acc[pr / 4], 0, 0, 0);
                    acc[pr / 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[gi][1], op[gj][1], acc[pr / 4], 0, 0, 0);
                }
            });
        }
    }
    if (wave_s == 0) {
#pragma unroll
        for (int g = 0; g < NB; ++g) bsum[g] += __shfl_xor(bsum[g], 32);
    }
}

// Sum bsum over the KS lanes that hold the same columns; afterwards lanes with kk == 0 hold b.
template <int D> __device__ __forceinline__ void fold_b(float (&bsum)[Geo<D>::NC]) {
    constexpr int TM = Geo<D>::TM, KS = Geo<D>::KS, NC = Geo<D>::NC;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
#pragma unroll
        for (int off = TM * KS / 2; off >= TM; off >>= 1) bsum[c] += __shfl_xor(bsum[c], off);
    }
}

// ---------------------------------------------------------------------------------------------- LDS solve
// a: [D][LD] with entry (r, c), r >= c, at a[c*LD + r]; on exit column c of L sits at a[c*LD + r]
// and its mirror copy at a[r*LD + c].  aux: dinv[D], z[D], xout[D], bvec[D].
template <int D>
__device__ __forceinline__ void cholesky_solve_lds(float *a, float *aux, int32_t *err_flag) {
    constexpr int LD = Team<D>::LD, T = Team<D>::THREADS, TY = T / 32;
    float *dinv = aux, *z = aux + D, *xout = aux + 2 * D, *bvec = aux + 3 * D;
    const int t = opaque_tid(), tx = t & 31, ty = t >> 5;
    for (int k = 0; k < D; ++k) {
        const float pivot = a[k * LD + k];
        if (t == 0 && !(pivot > 0.f)) atomicOr(err_flag, 1);
        const float rinv = 1.0f / sqrtf(pivot);
        for (int i = k + 1 + t; i < D; i += T) {
            const float l = a[k * LD + i] * rinv;
            a[k * LD + i] = l;
            a[i * LD + k] = l;
        }
        if (t == 0) dinv[k] = rinv;
        __syncthreads();
        for (int j = k + 1 + ty; j < D; j += TY) {
            const float cj = a[k * LD + j];
            for (int i = j + tx; i < D; i += 32) a[j * LD + i] -= a[k * LD + i] * cj;
        }
        __syncthreads();
    }
    // L z = b
    for (int j = 0; j < D; ++j) {
        const float zj = bvec[j] * dinv[j];  // final: only entries i > j change in step j
        for (int i = j + 1 + t; i < D; i += T) bvec[i] -= a[j * LD + i] * zj;
        if (t == 0) z[j] = zj;
        __syncthreads();
    }
    // L^T x = z
    for (int i = D - 1; i >= 0; --i) {
        const float xi = z[i] * dinv[i];
        for (int j = t; j < i; j += T) z[j] -= a[i * LD + j] * xi;
        if (t == 0) xout[i] = xi;
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------- one-wavefront solve
// LDS layout of the direct solver for D >= 64: lower triangle, the solver's auxiliary and result
// buffers (tri_solve.h), the right-hand side.
template <int D> struct Packed {
    static constexpr int TRI = tri_row(D);
    static constexpr int OFF_COL = TRI;                        // the solver's auxiliary buffer
    static constexpr int OFF_T = OFF_COL + TRI_AUX_FLOATS;     // tbuf[D]
    static constexpr int OFF_RHS = OFF_T + D;      // rhs[D]
    static constexpr size_t LDS_BYTES = (size_t)(OFF_RHS + D) * sizeof(float);
};

// Called by one wavefront after a workgroup barrier: solves the packed system and stores the row,
// rounded once to the table's element type.  The other wavefronts of the workgroup may have exited.
template <int D, bool BF16>
__device__ __forceinline__ void packed_solve_store(float *lds, void *X, int64_t xoff, int32_t *err_flag) {
    const int lane = opaque_tid() & 63;
    float *tbuf = lds + Packed<D>::OFF_T;
    const float *rhs = lds + Packed<D>::OFF_RHS;
    const float y0 = lane < D ? rhs[lane] : 0.f;
    const float y1 = (D > 64 && 64 + lane < D) ? rhs[64 + lane] : 0.f;
    int k = D;
    asm volatile("" : "+s"(k));  // opaque on purpose: with a compile-time step count the solver's steps merge
                                 // into one block, whose scheduling runs out of registers
    tri_solve<D>(lds, lds + Packed<D>::OFF_COL, tbuf, y0, y1, k, err_flag);
    for (int c = lane; c < D; c += 64) store_elem<BF16>(X, xoff + c, tbuf[c]);
}

// ---------------------------------------------------------------------------------------------- conjugate gradients
template <int D>
__device__ __forceinline__ float block_dot(float v, float *red /* [THREADS/64] */) {
    const int lane = opaque_tid() & 63, w = opaque_tid() >> 6;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();  // red is free again
    if (lane == 0) red[w] = v;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < Team<D>::THREADS / 64; ++i) s += red[i];
    return s;
}

template <int D>
__device__ __forceinline__ void cg_solve_lds(const float *a, float *aux, int max_iters, float tol) {
    constexpr int LD = Team<D>::LD;
    float *rvec = aux, *pvec = aux + D, *xvec = aux + 2 * D, *bvec = aux + 3 * D, *red = aux + 4 * D;
    const int i = opaque_tid();
    const bool mine = i < D;
    auto matvec = [&](const float *v) {  // row i of A times v (A symmetric: read column i, contiguous in LDS)
        float s = 0.f;
        if (mine) {
#pragma unroll 8
            for (int j = 0; j < D; ++j) s += a[j * LD + i] * v[j];
        }
        return s;
    };
    float x = mine ? xvec[i] : 0.f;
    const float b = mine ? bvec[i] : 0.f;
    float r = b - matvec(xvec);
    float pv = r;
    const float bb = block_dot<D>(b * b, red);
    float rs = block_dot<D>(r * r, red);
    const float stop = fmaxf(tol * tol * bb, CG_RESIDUAL_FLOOR);
    for (int it = 0; it < max_iters && rs > stop; ++it) {
        __syncthreads();
        if (mine) pvec[i] = pv;
        __syncthreads();
        const float ap = matvec(pvec);
        const float pap = block_dot<D>(pv * ap, red);
        if (!(pap > 0.f)) break;  // only when the numbers have left the fp32 range; the same in every thread
        const float alpha = rs / pap;
        x += alpha * pv;
        r -= alpha * ap;
        const float rs_new = block_dot<D>(r * r, red);
        pv = r + (rs_new / rs) * pv;
        rs = rs_new;
    }
    (void)rvec;
    __syncthreads();
    if (mine) xvec[i] = x;
    __syncthreads();
}

template <int D>
__device__ __forceinline__ void solve_spd_lds(float *a, float *aux, int32_t *err_flag, int solver, int cg_iters,
                                              float cg_tol) {
    if (solver == ALS_SOLVER_CG) {  // uniform for the launch
        cg_solve_lds<D>(a, aux, cg_iters, cg_tol);
        return;
    }
    if constexpr (D < 64) cholesky_solve_lds<D>(a, aux, err_flag);  // D >= 64: packed path of the callers
}

// ---------------------------------------------------------------------------------------------- kernels
enum PrimalMode { MODE_FUSED = 0, MODE_SEGMENT = 1 };

// One work item.  `last`: the workgroup has no further item, so the wavefronts that do not solve may retire
// as soon as their tiles are in LDS (their SIMD slots go to the next workgroup).  Returns false when the
// calling wavefront has retired.
template <int D, bool BF16, int MODE>
__device__ __forceinline__ bool primal_step(
    const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices, const float *__restrict__ values,
    const void *__restrict__ V, int64_t ldv, const float *__restrict__ G, float alpha, float lambda,
    void *__restrict__ X, int64_t ldx, int64_t row_begin, const int32_t *__restrict__ row_list,
    const Segment *__restrict__ segs, float *__restrict__ partials, int32_t *__restrict__ err_flag, int solver,
    int cg_iters, float cg_tol, int64_t item, bool last, float *lds) {
    using GE = Geo<D>;
    constexpr int NC = GE::NC, TM = GE::TM, ACC = GE::ACC, LD = Team<D>::LD;
    typedef typename AccT<ACC>::type acc_t;
    float *a = lds, *aux = lds + D * LD, *bvec = aux + 3 * D;

    const int lane = opaque_tid() & 63, wave = opaque_tid() >> 6;
    const int m = lane % TM, kk = lane / TM;
    int64_t u = 0, begin, end;
    if constexpr (MODE == MODE_FUSED) {
        u = row_begin + row_list[item];
        begin = indptr[u];
        end = indptr[u + 1];
    } else {
        begin = segs[item].begin;
        end = segs[item].end;
    }

    // The statistics are accumulated in one of two register layouts (fp32 matrix cores: tile-row `wave` of the
    // column-interleaved tiles; bf16 tables with d >= 64: block pairs of the upper block triangle, see
    // accumulate_entries_bf16) and handed, element by element, to whatever wants them: deliver(put, put_b)
    // calls put(r, c, value) for entries of V_I^T V_I - every (r, c) with c <= r at least once, possibly also
    // the mirror (c, r) - and put_b(c, value) for the entries of b.
    constexpr bool CORES16 = BF16 && D >= 64;
    acc_t acc[CORES16 ? 1 : NC];
    floatx16 acc16[CORES16 ? 3 : 1];
    float bsum[NC];
#pragma unroll
    for (int j = 0; j < NC; ++j) bsum[j] = 0.f;
    if constexpr (CORES16) {
#pragma unroll
        for (int j = 0; j < 3; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc16[j][v] = 0.f;
        accumulate_entries_bf16<D>((const uint16_t *)V, ldv, indices, values, begin, end, wave, acc16, bsum);
    } else {
#pragma unroll
        for (int j = 0; j < NC; ++j)
#pragma unroll
            for (int v = 0; v < ACC; ++v) acc[j][v] = 0.f;
        accumulate_entries<D, BF16>(V, ldv, indices, values, begin, end, wave, acc, bsum);
        fold_b<D>(bsum);
    }
    auto deliver = [&](auto &&put, auto &&put_b) {
        if constexpr (CORES16) {
            using BP = BlockPairs<D>;
            const int m32 = lane & 31, kq = lane >> 5;
            const int wave_s = __builtin_amdgcn_readfirstlane(wave);
            static_for<0, BP::COUNT>([&](auto pp) {
                constexpr int pr = decltype(pp)::value, gi = BP::first(pr), gj = BP::second(pr);
                if (wave_s == pr % 4) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int r = 32 * gi + 8 * (v >> 2) + 4 * kq + (v & 3), c = 32 * gj + m32;
                        put(r, c, acc16[pr / 4][v]);
                        if constexpr (gi != gj) put(c, r, acc16[pr / 4][v]);
                    }
                }
            });
            if (wave_s == 0 && kq == 0) {
#pragma unroll
                for (int g = 0; g < D / 32; ++g) put_b(32 * g + m32, bsum[g]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < NC; ++j)
#pragma unroll
                for (int v = 0; v < ACC; ++v) put(NC * acc_row<D>(v, lane) + wave, NC * m + j, acc[j][v]);
            if (wave == 0 && kk == 0) {
#pragma unroll
                for (int j = 0; j < NC; ++j) put_b(NC * m + j, bsum[j]);
            }
        }
    };

    if constexpr (MODE == MODE_SEGMENT) {
        float *out = partials + item * (int64_t)(D * D + D);
        deliver([&](int r, int c, float v) { out[r * D + c] = v; }, [&](int c, float v) { out[D * D + c] = v; });
        (void)last;
        return true;
    } else {
        if constexpr (D >= 64) {
            if (solver == ALS_SOLVER_DIRECT) {  // uniform for the launch
                // lower triangle of A = alpha*G + lambda*I + V_I^T V_I, packed, then one wavefront solves
                float *tri = lds, *rhs = lds + Packed<D>::OFF_RHS;
                deliver(
                    [&](int r, int c, float v) {
                        if (c <= r) tri[tri_row(r) + c] = v + alpha * G[r * D + c] + (r == c ? lambda : 0.f);
                    },
                    [&](int c, float v) { rhs[c] = v; });
                __syncthreads();
                // scalar test: the solver must not sit in (what looks like) divergent control flow
                if (__builtin_amdgcn_readfirstlane(wave) != 0) {
                    if (last) return false;
                } else {
                    packed_solve_store<D, BF16>(lds, X, u * ldx, err_flag);
                }
                if (!last) __syncthreads();  // the solver is done with the LDS before the next row's tiles arrive
                return true;
            }
        }
        // A = alpha*G + lambda*I + V_I^T V_I into LDS (entry (r,c) at a[c*LD + r])
        deliver([&](int r, int c, float v) { a[c * LD + r] = v + alpha * G[r * D + c] + (r == c ? lambda : 0.f); },
                [&](int c, float v) { bvec[c] = v; });
        if (solver == ALS_SOLVER_CG) {  // warm start from the row's current content
            for (int c = opaque_tid(); c < D; c += Team<D>::THREADS) aux[2 * D + c] = load_elem<BF16>(X, u * ldx + c);
        }
        __syncthreads();
        solve_spd_lds<D>(a, aux, err_flag, solver, cg_iters, cg_tol);
        const float *xout = aux + 2 * D;
        for (int c = opaque_tid(); c < D; c += Team<D>::THREADS) store_elem<BF16>(X, u * ldx + c, xout[c]);
        if (!last) __syncthreads();  // before the next row's tiles overwrite the LDS
        return true;
    }
}

// MODE_FUSED:   work item = the whole row u = row_begin + row_list[item].
// MODE_SEGMENT: work item = segment `item` of segs[]; raw partial statistics are written to
//               partials[item][D*D + D] (row-major D x D, then b).
// The two launch forms (see StepGrid): LOOP = false, workgroup b takes item first + b if there is one;
// LOOP = true, grid-stride walk from item `first` on.  *count_ptr is the number of items (device memory).
template <int D, bool BF16, int MODE, bool LOOP>
__global__ __launch_bounds__(Team<D>::THREADS, LOOP ? 1 : 2) void primal_kernel(
    const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices, const float *__restrict__ values,
    const void *__restrict__ V, int64_t ldv, const float *__restrict__ G, float alpha, float lambda,
    void *__restrict__ X, int64_t ldx, int64_t row_begin, const int32_t *__restrict__ row_list,
    const Segment *__restrict__ segs, float *__restrict__ partials, const int32_t *__restrict__ count_ptr, int first,
    int32_t *__restrict__ err_flag, int solver, int cg_iters, float cg_tol) {
    extern __shared__ float lds[];
    const int64_t nitems = *count_ptr;
    int64_t item = (int64_t)first + blockIdx.x;
    if constexpr (!LOOP) {
        if (item < nitems)
            primal_step<D, BF16, MODE>(indptr, indices, values, V, ldv, G, alpha, lambda, X, ldx, row_begin, row_list, segs,
                                       partials, err_flag, solver, cg_iters, cg_tol, item, true, lds);
    } else {
        for (; item < nitems; item += gridDim.x) {
            const bool last = item + gridDim.x >= nitems;
            if (!primal_step<D, BF16, MODE>(opaque(indptr), opaque(indices), opaque(values), opaque(V), opaque(ldv),
                                            opaque(G), opaque(alpha), opaque(lambda), opaque(X), opaque(ldx),
                                            opaque(row_begin), opaque(row_list), opaque(segs), opaque(partials),
                                            opaque(err_flag), opaque(solver), opaque(cg_iters), opaque(cg_tol), item, last,
                                            opaque(lds)))
                return;
        }
    }
}

// Adds the segment partials of every long row in a fixed order: workgroup (x, y) handles elements
// [256y, 256y+256) of long row x and overwrites the row's first partial with the sum.
template <int D>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const LongRow *__restrict__ long_rows,
                                                              float *__restrict__ partials,
                                                              const int32_t *__restrict__ n_long_ptr) {
    const int n_long = *n_long_ptr;
    for (int row = blockIdx.x; row < n_long; row += gridDim.x) {
    const LongRow lr = long_rows[row];
    const int e = blockIdx.y * 256 + opaque_tid();
    if (e >= D * D + D || lr.nseg <= 1) continue;
    float *p0 = partials + (int64_t)lr.seg_first * (D * D + D) + e;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int g = 0;
    for (; g + 4 <= lr.nseg; g += 4) {
        s0 += p0[(int64_t)(g + 0) * (D * D + D)];
        s1 += p0[(int64_t)(g + 1) * (D * D + D)];
        s2 += p0[(int64_t)(g + 2) * (D * D + D)];
        s3 += p0[(int64_t)(g + 3) * (D * D + D)];
    }
    for (; g < lr.nseg; ++g) s0 += p0[(int64_t)g * (D * D + D)];
    p0[0] = (s0 + s1) + (s2 + s3);
    }
}

// Loads the summed statistics of one long row, adds alpha*G + lambda*I, solves, stores.  `last` and the
// return value as in primal_step.
template <int D, bool BF16>
__device__ __forceinline__ bool reduce_solve_step(const LongRow lr, const float *__restrict__ partials,
                                                  const float *__restrict__ G, float alpha, float lambda,
                                                  void *__restrict__ X, int64_t ldx, int32_t *__restrict__ err_flag,
                                                  int solver, int cg_iters, float cg_tol, bool last, float *lds) {
    constexpr int LD = Team<D>::LD, T = Team<D>::THREADS;
    float *a = lds, *aux = lds + D * LD, *bvec = aux + 3 * D;
    const float *p0 = partials + (int64_t)lr.seg_first * (D * D + D);
    if constexpr (D >= 64) {
        if (solver == ALS_SOLVER_DIRECT) {
            float *tri = lds, *rhs = lds + Packed<D>::OFF_RHS;
            for (int e = opaque_tid(); e < D * D + D; e += T) {
                const float s = p0[e];
                if (e < D * D) {
                    const int r = e / D, c = e % D;
                    if (c <= r) tri[tri_row(r) + c] = s + alpha * G[e] + (r == c ? lambda : 0.f);
                } else {
                    rhs[e - D * D] = s;
                }
            }
            __syncthreads();
            if (__builtin_amdgcn_readfirstlane(opaque_tid() >> 6) != 0) {
                if (last) return false;
            } else {
                packed_solve_store<D, BF16>(lds, X, lr.row * ldx, err_flag);
            }
            if (!last) __syncthreads();
            return true;
        }
    }
    for (int e = opaque_tid(); e < D * D + D; e += T) {
        const float s = p0[e];
        if (e < D * D) {
            const int r = e / D, c = e % D;
            a[c * LD + r] = s + alpha * G[e] + (r == c ? lambda : 0.f);
        } else {
            bvec[e - D * D] = s;
        }
    }
    if (solver == ALS_SOLVER_CG) {
        for (int c = opaque_tid(); c < D; c += T) aux[2 * D + c] = load_elem<BF16>(X, lr.row * ldx + c);
    }
    __syncthreads();
    solve_spd_lds<D>(a, aux, err_flag, solver, cg_iters, cg_tol);
    const float *xout = aux + 2 * D;
    for (int c = opaque_tid(); c < D; c += T) store_elem<BF16>(X, lr.row * ldx + c, xout[c]);
    if (!last) __syncthreads();
    return true;
}

template <int D, bool BF16, bool LOOP>
__global__ __launch_bounds__(Team<D>::THREADS) void reduce_solve_kernel(
    const LongRow *__restrict__ long_rows, const float *__restrict__ partials, const float *__restrict__ G,
    float alpha, float lambda, void *__restrict__ X, int64_t ldx, const int32_t *__restrict__ n_long_ptr, int first,
    int32_t *__restrict__ err_flag, int solver, int cg_iters, float cg_tol) {
    extern __shared__ float lds[];
    const int n_long = *n_long_ptr;
    int row = first + (int)blockIdx.x;
    if constexpr (!LOOP) {
        if (row < n_long)
            reduce_solve_step<D, BF16>(long_rows[row], partials, G, alpha, lambda, X, ldx, err_flag, solver, cg_iters,
                                       cg_tol, true, lds);
    } else {
        for (; row < n_long; row += gridDim.x) {
            const bool last = row + (int)gridDim.x >= n_long;
            if (!reduce_solve_step<D, BF16>(long_rows[row], opaque(partials), opaque(G), opaque(alpha), opaque(lambda),
                                            opaque(X), opaque(ldx), opaque(err_flag), opaque(solver), opaque(cg_iters),
                                            opaque(cg_tol), last, opaque(lds)))
                return;
        }
    }
}

// ---------------------------------------------------------------------------------------------- launchers
template <int D> static size_t solve_lds_bytes(int solver) {
    if constexpr (D >= 64) {
        if (solver == ALS_SOLVER_DIRECT) return Packed<D>::LDS_BYTES;
    }
    return Team<D>::LDS_BYTES;
}

template <int D, bool BF16>
static als_status primal_typed(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                               const als_params *prm, als_table *X, int64_t r0, const int32_t *row_list,
                               const int32_t *count_dev, StepGrid g, hipStream_t s) {
    if (g.known == 0 && g.rest == 0) return ALS_OK;
    int32_t *err = (int32_t *)((char *)ctx->small.p + SM_COUNTERS) + 2;
    const int cg_iters = prm->cg_max_iters > 0 ? prm->cg_max_iters : 2 * D;
    const float cg_tol = prm->cg_tol > 0.f ? prm->cg_tol : 1e-6f;
    auto kern = primal_kernel<D, BF16, MODE_FUSED, false>;
    auto kern_loop = primal_kernel<D, BF16, MODE_FUSED, true>;
    static const hipError_t attr = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                       (int)Team<D>::LDS_BYTES);
    static const hipError_t attr_loop = hipFuncSetAttribute(
        (const void *)kern_loop, hipFuncAttributeMaxDynamicSharedMemorySize, (int)Team<D>::LDS_BYTES);  // both once per process
    ALS_HIP(ctx, attr);
    ALS_HIP(ctx, attr_loop);
    const size_t lds_bytes = solve_lds_bytes<D>(prm->solver);
    timer_begin(ctx, T_PRIMAL, s);
    if (g.known > 0)
        hipLaunchKernelGGL(kern, dim3(g.known), dim3(Team<D>::THREADS), lds_bytes, s, Y->indptr, Y->indices, Y->values,
                           V->data, V->ld, G, prm->alpha, prm->lambda, X->data, X->ld, r0, row_list,
                           (const Segment *)nullptr, (float *)nullptr, count_dev, 0, err, prm->solver, cg_iters, cg_tol);
    if (g.rest > 0)
        hipLaunchKernelGGL(kern_loop, dim3(g.rest), dim3(Team<D>::THREADS), lds_bytes, s, Y->indptr, Y->indices,
                           Y->values, V->data, V->ld, G, prm->alpha, prm->lambda, X->data, X->ld, r0, row_list,
                           (const Segment *)nullptr, (float *)nullptr, count_dev, (int)g.known, err, prm->solver,
                           cg_iters, cg_tol);
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

// counters[0] = number of long rows, counters[1] = number of their segments (device memory).
template <int D, bool BF16>
static als_status long_typed(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                             const als_params *prm, als_table *X, const LongRow *long_rows, const Segment *segs,
                             const int32_t *counters, int64_t seg_capacity, StepGrid g_long, StepGrid g_seg,
                             hipStream_t s) {
    if (g_seg.known == 0 && g_seg.rest == 0) return ALS_OK;
    als_status st = ensure(ctx, ctx->seg_partials, (size_t)seg_capacity * (D * D + D) * sizeof(float));
    if (st != ALS_OK) return st;
    int32_t *err = (int32_t *)((char *)ctx->small.p + SM_COUNTERS) + 2;
    const int cg_iters = prm->cg_max_iters > 0 ? prm->cg_max_iters : 2 * D;
    const float cg_tol = prm->cg_tol > 0.f ? prm->cg_tol : 1e-6f;
    auto kred = reduce_solve_kernel<D, BF16, false>;
    auto kred_loop = reduce_solve_kernel<D, BF16, true>;
    static const hipError_t attr = hipFuncSetAttribute((const void *)kred, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                       (int)Team<D>::LDS_BYTES);
    static const hipError_t attr_loop = hipFuncSetAttribute(
        (const void *)kred_loop, hipFuncAttributeMaxDynamicSharedMemorySize, (int)Team<D>::LDS_BYTES);  // both once per process
    ALS_HIP(ctx, attr);
    ALS_HIP(ctx, attr_loop);
    float *partials = (float *)ctx->seg_partials.p;
    timer_begin(ctx, T_SEGMENT, s);
    if (g_seg.known > 0)
        hipLaunchKernelGGL((primal_kernel<D, BF16, MODE_SEGMENT, false>), dim3(g_seg.known), dim3(Team<D>::THREADS), 0, s,
                           Y->indptr, Y->indices, Y->values, V->data, V->ld, G, prm->alpha, prm->lambda, X->data, X->ld,
                           (int64_t)0, (const int32_t *)nullptr, segs, partials, counters + 1, 0, err, 0, 0, 0.f);
    if (g_seg.rest > 0)
        hipLaunchKernelGGL((primal_kernel<D, BF16, MODE_SEGMENT, true>), dim3(g_seg.rest), dim3(Team<D>::THREADS), 0, s,
                           Y->indptr, Y->indices, Y->values, V->data, V->ld, G, prm->alpha, prm->lambda, X->data, X->ld,
                           (int64_t)0, (const int32_t *)nullptr, segs, partials, counters + 1, (int)g_seg.known, err, 0,
                           0, 0.f);
    timer_end(ctx, s);
    timer_begin(ctx, T_REDUCE, s);
    const unsigned red_blocks = std::max(1u, g_long.known + g_long.rest);  // grid-stride over the long rows
    hipLaunchKernelGGL(reduce_partials_kernel<D>, dim3(red_blocks, (D * D + D + 255) / 256), dim3(256), 0, s, long_rows,
                       partials, counters);
    const size_t lds_bytes = solve_lds_bytes<D>(prm->solver);
    if (g_long.known > 0)
        hipLaunchKernelGGL(kred, dim3(g_long.known), dim3(Team<D>::THREADS), lds_bytes, s, long_rows,
                           (const float *)partials, G, prm->alpha, prm->lambda, X->data, X->ld, counters, 0, err,
                           prm->solver, cg_iters, cg_tol);
    if (g_long.rest > 0)
        hipLaunchKernelGGL(kred_loop, dim3(g_long.rest), dim3(Team<D>::THREADS), lds_bytes, s, long_rows,
                           (const float *)partials, G, prm->alpha, prm->lambda, X->data, X->ld, counters,
                           (int)g_long.known, err, prm->solver, cg_iters, cg_tol);
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

#define ALS_DISPATCH(fn, d, bf, ...)                                                       \
    switch (d) {                                                                           \
        case 16: return bf ? fn<16, true>(__VA_ARGS__) : fn<16, false>(__VA_ARGS__);       \
        case 32: return bf ? fn<32, true>(__VA_ARGS__) : fn<32, false>(__VA_ARGS__);       \
        case 64: return bf ? fn<64, true>(__VA_ARGS__) : fn<64, false>(__VA_ARGS__);       \
        case 128: return bf ? fn<128, true>(__VA_ARGS__) : fn<128, false>(__VA_ARGS__);    \
    }                                                                                      \
    return fail(ctx, ALS_EDTYPE, "unsupported d")

als_status launch_primal_fused(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                               const als_params *prm, als_table *X, int64_t r0, const int32_t *row_list,
                               const int32_t *count_dev, StepGrid g, hipStream_t s) {
    const bool bf = V->dtype == ALS_BF16;
    ALS_DISPATCH(primal_typed, V->d, bf, ctx, Y, V, G, prm, X, r0, row_list, count_dev, g, s);
}

als_status launch_primal_long(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                              const als_params *prm, als_table *X, const LongRow *long_rows, const Segment *segs,
                              const int32_t *counters, int64_t seg_capacity, StepGrid g_long, StepGrid g_seg,
                              hipStream_t s) {
    const bool bf = V->dtype == ALS_BF16;
    ALS_DISPATCH(long_typed, V->d, bf, ctx, Y, V, G, prm, X, long_rows, segs, counters, seg_capacity, g_long, g_seg, s);
}

}  // namespace als
