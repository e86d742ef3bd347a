// Conjugate gradients on the d x d normal equations of Eq. 4 without ever forming a row's matrix
// (Section 4.5 names conjugate gradients as the solver of choice because it is made of matrix products):
//     A p = (alpha G + lambda I) p + V_I^T (V_I p),      b = V_I^T y,
// for sixteen rows per wavefront at a time.  The first term is the same matrix for every row, so the sixteen
// products are one 16 x d by d x d matrix product on the fp32 matrix cores, with alpha G + lambda I held in LDS by
// the workgroup; the second term is two passes over the row's gathered entries.  Nothing of size d x d exists per row.
//
// Lane (row, q) = (lane % 16, lane / 16) holds, of each of its row's vectors (x, r, p, A p), the columns
// 16 j + 4 q + v (j < d/16, v < 4) as float4 pieces: this is both what a lane supplies to v_mfma_f32_16x16x4f32 as
// the B operand of depth step (j, v) and what it receives of the product in the accumulator of column tile j, so
// the vectors never change layout.  Scalars of a row (step lengths, residual norms) are replicated in its
// four lanes.  Each row starts from its current content in X (warm start) and stops on its own when
// |residual| <= tol |b|; the wavefront goes on until all sixteen have stopped or max_iters is reached, then checks
// the true residuals once more.
#include "dual_common.h"

namespace als {

template <int D> struct FreeCfg {
    static constexpr int NT = D / 16;  // float4 pieces per lane and vector; column tiles of the product
    static constexpr int LDB = D + 4;  // row stride of alpha G + lambda I in LDS
    static constexpr size_t LDS_BYTES = (size_t)D * LDB * sizeof(float);
};

// four consecutive elements of a table row as fp32
template <bool BF16> __device__ __forceinline__ float4 load4(const void *T, int64_t elem) {
    if constexpr (!BF16) {
        return *(const float4 *)((const float *)T + elem);
    } else {
        const uint2 w = *(const uint2 *)((const uint16_t *)T + elem);
        return make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                           __uint_as_float(w.y & 0xffff0000u));
    }
}
template <bool BF16> __device__ __forceinline__ void store4(void *T, int64_t elem, const float4 &v) {
    if constexpr (!BF16) {
        *(float4 *)((float *)T + elem) = v;
    } else {  // round to nearest even
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float floatx2 __attribute__((ext_vector_type(2)));
        uint2 w;
        w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector((floatx2){v.x, v.y}, bf16x2));
        w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector((floatx2){v.z, v.w}, bf16x2));
        *(uint2 *)((uint16_t *)T + elem) = w;
    }
}

__device__ __forceinline__ float dot4(const float4 &a, const float4 &b) { return a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w; }
__device__ __forceinline__ void axpy4(float4 &y, float a, const float4 &x) {
    y.x += a * x.x;
    y.y += a * x.y;
    y.z += a * x.z;
    y.w += a * x.w;
}
// sum over the four lanes of a row
__device__ __forceinline__ float row_sum(float v) {
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

// Sixteen rows list[item0 .. item0 + 15] (item0 < count).  bl: alpha G + lambda I in LDS.
template <int D, bool BF16>
__device__ __forceinline__ void cg_free_step(const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                                             const float *__restrict__ values, const void *__restrict__ V, int64_t ldv,
                                             void *__restrict__ X, int64_t ldx, int64_t r0,
                                             const int32_t *__restrict__ list, int count, int item0, const float *bl,
                                             int max_iters, float tol) {
    constexpr int NT = FreeCfg<D>::NT, LDB = FreeCfg<D>::LDB;
    const int lane = opaque_tid() & 63, row = lane & 15, q = lane >> 4;
    const bool have = item0 + row < count;
    const int64_t u = r0 + list[have ? item0 + row : item0];
    const int64_t b = indptr[u];
    const int k = have ? (int)(indptr[u + 1] - b) : 0;  // >= 1 for listed rows; lanes past the list's end sit idle
    int kmax = k;
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) kmax = max(kmax, __shfl_xor(kmax, off));

    // out += V_I^T w with w_e = <v_e, p> (p given) or w_e = y_e (p == nullptr)
    auto gather = [&](const float4 *p, float4 (&out)[NT]) {
        for (int e = 0; e < kmax; ++e) {
            const bool valid = e < k;
            const int32_t id = indices[b + (valid ? e : 0)];  // the row has a first entry also where k was set to 0
            float4 v[NT];
#pragma unroll
            for (int j = 0; j < NT; ++j) v[j] = load4<BF16>(V, (int64_t)id * ldv + 16 * j + 4 * q);
            float w;
            if (p) {
                w = 0.f;
#pragma unroll
                for (int j = 0; j < NT; ++j) w += dot4(v[j], p[j]);
                w = row_sum(w);
            } else {
                w = values ? values[b + (valid ? e : 0)] : 1.f;
            }
            w = valid ? w : 0.f;
#pragma unroll
            for (int j = 0; j < NT; ++j) axpy4(out[j], w, v[j]);
        }
    };
    // out = A p
    auto apply = [&](const float4 (&p)[NT], float4 (&out)[NT]) {
        floatx4 acc[NT];
#pragma unroll
        for (int jo = 0; jo < NT; ++jo) acc[jo] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NT; ++j) {
#pragma unroll
            for (int jo = 0; jo < NT; ++jo) {
                // A operand: lane (mm, kq) = (row, q) supplies (alpha G + lambda I)[16 jo + mm][16 j + 4 kq + v]
                const float4 a = *(const float4 *)(bl + (16 * jo + row) * LDB + 16 * j + 4 * q);
                acc[jo] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, p[j].x, acc[jo], 0, 0, 0);
                acc[jo] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, p[j].y, acc[jo], 0, 0, 0);
                acc[jo] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, p[j].z, acc[jo], 0, 0, 0);
                acc[jo] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, p[j].w, acc[jo], 0, 0, 0);
            }
        }
#pragma unroll
        for (int jo = 0; jo < NT; ++jo) out[jo] = make_float4(acc[jo][0], acc[jo][1], acc[jo][2], acc[jo][3]);
        gather(p, out);
    };

    float4 x[NT], r[NT], p[NT], ap[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) x[j] = load4<BF16>(X, u * ldx + 16 * j + 4 * q);
    // The residual carried along by the recurrence drifts away from b - A x when the start is far from the
    // solution (rounding errors scale with the first residual, not with b): when every row has stopped, the
    // residuals are formed afresh and the iteration goes on from there if one of them is still too large.
    float stop = 0.f;
    int it = 0;
    for (int pass = 0; pass < 4; ++pass) {
#pragma unroll
        for (int j = 0; j < NT; ++j) r[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        gather(nullptr, r);  // b
        if (pass == 0) {
            float bb = 0.f;
#pragma unroll
            for (int j = 0; j < NT; ++j) bb += dot4(r[j], r[j]);
            stop = fmaxf(tol * tol * row_sum(bb), CG_RESIDUAL_FLOOR);
        }
        apply(x, ap);
        float rs = 0.f;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            r[j].x -= ap[j].x;
            r[j].y -= ap[j].y;
            r[j].z -= ap[j].z;
            r[j].w -= ap[j].w;
            p[j] = r[j];
            rs += dot4(r[j], r[j]);
        }
        rs = row_sum(rs);
        if (!__any(have && rs > stop) || it >= max_iters) break;
        for (; it < max_iters; ++it) {
            const bool act = have && rs > stop;
            if (!__any(act)) break;
            apply(p, ap);
            float pap = 0.f;
#pragma unroll
            for (int j = 0; j < NT; ++j) pap += dot4(p[j], ap[j]);
            pap = row_sum(pap);
            // p^T A p > 0 unless the numbers have left the fp32 range: such a row stops where it is
            const bool go = act && pap > 0.f;
            const float alpha = go ? rs / pap : 0.f;
            float rs_new = 0.f;
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                axpy4(x[j], alpha, p[j]);
                axpy4(r[j], -alpha, ap[j]);
                rs_new += dot4(r[j], r[j]);
            }
            rs_new = row_sum(rs_new);
            const float beta = go ? rs_new / rs : 0.f;
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                p[j].x = r[j].x + beta * p[j].x;
                p[j].y = r[j].y + beta * p[j].y;
                p[j].z = r[j].z + beta * p[j].z;
                p[j].w = r[j].w + beta * p[j].w;
            }
            rs = go ? rs_new : (act ? 0.f : rs);
        }
    }
    if (have) {
#pragma unroll
        for (int j = 0; j < NT; ++j) store4<BF16>(X, u * ldx + 16 * j + 4 * q, x[j]);
    }
}

// Grid-stride over chunks of 64 list entries (16 per wavefront); the list's length is read on the device.
template <int D, bool BF16>
__global__ __launch_bounds__(256, D >= 128 ? 1 : 2) void cg_free_kernel(const int64_t *__restrict__ indptr,
                                                         const int32_t *__restrict__ indices,
                                                         const float *__restrict__ values, const void *__restrict__ V,
                                                         int64_t ldv, const float *__restrict__ G, float alpha,
                                                         float lambda, void *__restrict__ X, int64_t ldx, int64_t r0,
                                                         const int32_t *__restrict__ list,
                                                         const int32_t *__restrict__ count_ptr, int max_iters, float tol) {
    constexpr int LDB = FreeCfg<D>::LDB;
    extern __shared__ float bl[];
    const int count = *count_ptr;
    if ((int64_t)blockIdx.x * 64 >= count) return;  // uniform for the workgroup
    for (int e = threadIdx.x; e < D * D; e += 256) {
        const int rr = e / D, c = e % D;
        bl[rr * LDB + c] = alpha * G[e] + (rr == c ? lambda : 0.f);
    }
    __syncthreads();
    const int wave = threadIdx.x >> 6;
    for (int64_t chunk = blockIdx.x; chunk * 64 < count; chunk += gridDim.x) {
        const int item0 = (int)(chunk * 64) + 16 * wave;
        if (item0 < count)
            cg_free_step<D, BF16>(opaque(indptr), opaque(indices), opaque(values), opaque(V), opaque(ldv), opaque(X),
                                  opaque(ldx), opaque(r0), opaque(list), count, item0, bl, max_iters, tol);
    }
}

template <int D, bool BF16>
static als_status cg_free_typed(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G, const als_params *prm,
                                als_table *X, int64_t r0, const int32_t *list, const int32_t *count_dev, int64_t cap,
                                int hint, hipStream_t s) {
    auto kern = cg_free_kernel<D, BF16>;
    static const hipError_t attr = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                       (int)FreeCfg<D>::LDS_BYTES);  // once per process
    ALS_HIP(ctx, attr);
    const int64_t rows = hint >= 0 ? std::min<int64_t>(hint, cap) : cap;
    const int64_t chunks = std::max<int64_t>(1, (rows + 63) / 64);
    const unsigned blocks = (unsigned)std::min<int64_t>(chunks, (int64_t)ctx->num_cu * 2);
    const int iters = prm->cg_max_iters > 0 ? prm->cg_max_iters : 2 * D;
    const float tol = prm->cg_tol > 0.f ? prm->cg_tol : 1e-6f;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), FreeCfg<D>::LDS_BYTES, s, Y->indptr, Y->indices, Y->values,
                       (const void *)V->data, V->ld, G, prm->alpha, prm->lambda, X->data, X->ld, r0, list, count_dev, iters,
                       tol);
    return ALS_OK;
}

// One launch per class list (rows of similar length share a wavefront).  `caps` bounds the lists, `hints` holds
// the lengths the previous call on the same matrix saw, or -1: they only size the grids.
als_status launch_cg_free(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G, const als_params *prm,
                          als_table *X, int64_t r0, const int32_t *const lists[10], const int32_t *const counts_dev[10],
                          const int64_t caps[10], const int hints[10], hipStream_t s) {
    static const int slot_of[10] = {T_DUAL_CLASS0,     T_DUAL_CLASS0 + 1, T_DUAL_CLASS0 + 2, T_DUAL_CLASS0 + 3,
                                    T_DUAL_CLASS0 + 4, T_DUAL_CLASS0 + 5, T_DUAL_CLASS0 + 6, T_DUAL_CLASS0 + 7,
                                    T_SMALL4,          T_SMALL8};
    const bool bf = V->dtype == ALS_BF16;
    for (int c = 0; c < 10; ++c) {
        if (caps[c] <= 0) continue;
        timer_begin(ctx, slot_of[c], s);
        als_status st = ALS_EDTYPE;
#define ALS_FREE_CASE(dd)                                                                                              \
    case dd:                                                                                                           \
        st = bf ? cg_free_typed<dd, true>(ctx, Y, V, G, prm, X, r0, lists[c], counts_dev[c], caps[c], hints[c], s)     \
                : cg_free_typed<dd, false>(ctx, Y, V, G, prm, X, r0, lists[c], counts_dev[c], caps[c], hints[c], s);   \
        break;
        switch (V->d) { ALS_FREE_CASE(16) ALS_FREE_CASE(32) ALS_FREE_CASE(64) ALS_FREE_CASE(128) }
#undef ALS_FREE_CASE
        timer_end(ctx, s);
        if (st != ALS_OK) return st == ALS_EDTYPE ? fail(ctx, ALS_EDTYPE, "unsupported d") : st;
    }
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

}  // namespace als
