// Exact top-k retrieval by inner product: for every query row, the k rows of an item table with the largest
// <query, item>.  The paper names top-K retrieval as the step after training (Section 4.6) and evaluates with
// Recall@20 / Recall@50 on test rows whose embedding is folded in with Eq. 4 from part of their links
// (Section 5); the folded-in rows come from als_solve_rows, this file supplies the retrieval.
//
// scan kernel   a wavefront owns 16 queries (their operand registers stay loaded) and walks the item tiles of
//               its slice of the table, 16 items at a time: one 16 x 16 tile of scores on the fp32 matrix
//               cores per tile.  A score at least as large as the query's current k-th best is appended to the
//               query's candidate buffer in LDS (after a look at the query's exclusion list); a buffer that
//               fills up is sorted by the wavefront and cut back to its best k, which also raises the bar.  The
//               four wavefronts of a workgroup walk the same tiles for 64 different queries, so a tile comes
//               from HBM once per 64 queries.  Each slice leaves its best k per query in a workspace.
// merge kernel  one wavefront per query sorts the slices' candidates and writes the best k.
// Order everywhere: descending score, equal scores by ascending item id, so the result is unique.
#include <cmath>

#include "dual_common.h"

namespace als {

constexpr int TOPK_CAP = 128;       // candidate slots per query in LDS
constexpr int TOPK_MERGE = 1024;    // candidates the merge sorts per query (slices * padded k)
constexpr int TOPK_QPW = 16, TOPK_WAVES = 4;
constexpr int TOPK_TILES = 2;       // tiles of 16 items a wavefront scores per round

__device__ __forceinline__ bool ranks_before(float sa, int32_t ia, float sb, int32_t ib) {
    return sa > sb || (sa == sb && ia < ib);
}

// Bitonic sort of N (a power of two) candidates in LDS by one wavefront, best first.
template <int N> __device__ __forceinline__ void wave_sort(float *sc, int32_t *id, int lane) {
    for (int k2 = 2; k2 <= N; k2 <<= 1) {
        for (int j = k2 >> 1; j > 0; j >>= 1) {
            for (int t = lane; t < N / 2; t += 64) {
                const int i = (t / j) * 2 * j + (t % j), l = i + j;
                const float sa = sc[i], sb = sc[l];
                const int32_t ia = id[i], ib = id[l];
                const bool first_i = (i & k2) == 0;  // this block is sorted best-first / best-last
                if (ranks_before(sb, ib, sa, ia) == first_i) {
                    sc[i] = sb; sc[l] = sa;
                    id[i] = ib; id[l] = ia;
                }
            }
            wave_sync();
        }
    }
}

template <int D, bool BF16>
__global__ __launch_bounds__(64 * TOPK_WAVES) void topk_scan_kernel(
    const void *__restrict__ Q, int64_t ldq, int64_t nq, const void *__restrict__ H, int64_t ldh, int64_t n,
    const int64_t *__restrict__ ex_indptr, const int32_t *__restrict__ ex_indices, int k, int kpad,
    int64_t slice_items, float *__restrict__ part_sc, int32_t *__restrict__ part_id) {
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, a = lane & 15, q = lane >> 4;
    // per wavefront: scores [16][CAP], ids [16][CAP], count [16], bar [16]
    float *sc = lds + wave * (2 * TOPK_QPW * TOPK_CAP + 2 * TOPK_QPW);
    int32_t *id = (int32_t *)(sc + TOPK_QPW * TOPK_CAP);
    int32_t *cnt = id + TOPK_QPW * TOPK_CAP;
    float *bar = (float *)(cnt + TOPK_QPW);
    const int64_t q0 = ((int64_t)blockIdx.x * TOPK_WAVES + wave) * TOPK_QPW;
    if (q0 >= nq) return;  // wavefronts are independent of each other: no workgroup barrier below
    if (lane < TOPK_QPW) {
        cnt[lane] = 0;
        bar[lane] = -INFINITY;
    }
    // Operands: lane (a, q) holds, of query q0 + a and of item t0 + a, the 16-byte pieces j = 0 .. NP - 1 of the row
    // (piece j, lane group q: elements (4j + q) * EPP ..).  bf16 tables with d >= 32 are multiplied as they are
    // stored on the bf16 matrix cores (eight bf16 entries are one operand of v_mfma_f32_16x16x32_bf16; the
    // products are exact, the sums fp32); everything else as fp32 on v_mfma_f32_16x16x4f32.
    constexpr bool NATIVE = BF16 && D >= 32;
    constexpr int EPP = NATIVE ? 8 : 4, NP = D / (4 * EPP);
    auto load_row = [&](const void *T, int64_t elem0, bool ok, float4 (&z)[NP]) {
#pragma unroll
        for (int j = 0; j < NP; ++j) z[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ok) {
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                if constexpr (NATIVE) {
                    z[j] = *(const float4 *)((const uint16_t *)T + elem0 + (4 * j + q) * 8);
                } else {
                    float x[4];
                    load_vec<4, BF16>(T, elem0 + (4 * j + q) * 4, x);
                    z[j] = make_float4(x[0], x[1], x[2], x[3]);
                }
            }
        }
    };
    float4 zq[NP];
    load_row(Q, (q0 + a) * ldq, q0 + a < nq, zq);
    wave_sync();
    const int64_t i0 = (int64_t)blockIdx.y * slice_items, i1 = i0 + slice_items < n ? i0 + slice_items : n;

    auto compact = [&](int qy) {  // sort query qy's buffer, keep its best k, raise its bar
        float *s = sc + qy * TOPK_CAP;
        int32_t *d = id + qy * TOPK_CAP;
        const int c = cnt[qy];
        for (int t = c + lane; t < TOPK_CAP; t += 64) {
            s[t] = -INFINITY;
            d[t] = 0x7fffffff;
        }
        wave_sync();
        wave_sort<TOPK_CAP>(s, d, lane);
        if (lane == 0) {
            const int keep = c < k ? c : k;
            cnt[qy] = keep;
            bar[qy] = keep == k ? s[k - 1] : -INFINITY;
        }
        wave_sync();
    };

    // TOPK_TILES tiles of 16 items per round; the next round's rows are requested before this round's products
    float4 zh[TOPK_TILES][NP], zn[TOPK_TILES][NP];
#pragma unroll
    for (int u = 0; u < TOPK_TILES; ++u) load_row(H, (i0 + 16 * u + a) * ldh, i0 + 16 * u + a < i1, zh[u]);
    for (int64_t t0 = i0; t0 < i1; t0 += 16 * TOPK_TILES) {
#pragma unroll
        for (int u = 0; u < TOPK_TILES; ++u) {
            const int64_t nxt = t0 + 16 * (TOPK_TILES + u) + a;
            load_row(H, nxt * ldh, nxt < i1, zn[u]);
        }
        floatx4 acc[TOPK_TILES];
#pragma unroll
        for (int u = 0; u < TOPK_TILES; ++u) {
            acc[u] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                if constexpr (NATIVE) {
                    acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, zq[j]),
                                                                     __builtin_bit_cast(bf16x8, zh[u][j]), acc[u], 0, 0, 0);
                } else {
                    acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(zq[j].x, zh[u][j].x, acc[u], 0, 0, 0);
                    acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(zq[j].y, zh[u][j].y, acc[u], 0, 0, 0);
                    acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(zq[j].z, zh[u][j].z, acc[u], 0, 0, 0);
                    acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(zq[j].w, zh[u][j].w, acc[u], 0, 0, 0);
                }
            }
        }
        // acc[u][v] = <query q0 + 4q + v, item t0 + 16 u + a>
        const float4 b4 = *(const float4 *)(bar + 4 * q);
        const float bq[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
        for (int u = 0; u < TOPK_TILES; ++u) {
            const int64_t item = t0 + 16 * u + a;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int qy = 4 * q + v;
                if (item < i1 && q0 + qy < nq && acc[u][v] >= bq[v]) {
                    bool skip = false;
                    if (ex_indptr) {
                        const int64_t eb = ex_indptr[q0 + qy], ee = ex_indptr[q0 + qy + 1];
                        for (int64_t p = eb; p < ee; ++p) skip |= ex_indices[p] == (int32_t)item;
                    }
                    if (!skip) {
                        const int pos = atomicAdd(&cnt[qy], 1);  // at most 16 per tile and query: never beyond CAP
                        sc[qy * TOPK_CAP + pos] = acc[u][v];
                        id[qy * TOPK_CAP + pos] = (int32_t)item;
                    }
                }
            }
        }
        wave_sync();
        const int mine = lane < TOPK_QPW ? cnt[lane] : 0;
        unsigned long long full = __ballot(mine > TOPK_CAP - 16 * TOPK_TILES);
        while (full) {
            const int qy = __ffsll((long long)full) - 1;
            full &= full - 1;
            compact(qy);
        }
#pragma unroll
        for (int u = 0; u < TOPK_TILES; ++u)
#pragma unroll
            for (int j = 0; j < NP; ++j) zh[u][j] = zn[u][j];
    }
    for (int qy = 0; qy < TOPK_QPW; ++qy) {
        compact(qy);
        if (q0 + qy < nq && lane < kpad) {
            const int64_t o = ((int64_t)blockIdx.y * nq + q0 + qy) * kpad + lane;
            const bool have = lane < cnt[qy];
            part_sc[o] = have ? sc[qy * TOPK_CAP + lane] : -INFINITY;
            part_id[o] = have ? id[qy * TOPK_CAP + lane] : 0x7fffffff;
        }
    }
}

// One wavefront per query: the slices' candidates, sorted, best k written (ids -1 and scores -inf where the
// table has fewer than k admissible rows).
__global__ __launch_bounds__(64) void topk_merge_kernel(const float *__restrict__ part_sc,
                                                        const int32_t *__restrict__ part_id, int64_t nq, int slices,
                                                        int kpad, int k, int32_t *__restrict__ ids,
                                                        float *__restrict__ scores) {
    __shared__ float sc[TOPK_MERGE];
    __shared__ int32_t id[TOPK_MERGE];
    const int lane = threadIdx.x;
    const int64_t qy = blockIdx.x;
    const int total = slices * kpad;
    for (int t = lane; t < TOPK_MERGE; t += 64) {
        float s = -INFINITY;
        int32_t d = 0x7fffffff;
        if (t < total) {
            const int64_t o = ((int64_t)(t / kpad) * nq + qy) * kpad + t % kpad;
            s = part_sc[o];
            d = part_id[o];
        }
        sc[t] = s;
        id[t] = d;
    }
    wave_sync();
    wave_sort<TOPK_MERGE>(sc, id, lane);
    if (lane < k) {
        const bool have = id[lane] != 0x7fffffff;
        ids[qy * k + lane] = have ? id[lane] : -1;
        scores[qy * k + lane] = have ? sc[lane] : -INFINITY;
    }
}

template <int D, bool BF16>
static als_status topk_typed(als_ctx *ctx, const als_table *Q, const als_table *H, const als_csr *ex, int k,
                             int32_t *ids, float *scores, hipStream_t s) {
    int kpad = 1;
    while (kpad < k) kpad <<= 1;
    const int max_slices = TOPK_MERGE / kpad;
    int slices = (int)std::min<int64_t>(max_slices, std::max<int64_t>(1, (H->rows + 8191) / 8192));
    int64_t slice_items = (H->rows + slices - 1) / slices;
    slice_items = (slice_items + 15) / 16 * 16;
    slices = (int)std::max<int64_t>(1, (H->rows + slice_items - 1) / slice_items);
    const size_t part = (size_t)slices * Q->rows * kpad;
    als_status st = ensure(ctx, ctx->topk_partials, part * (sizeof(float) + sizeof(int32_t)));
    if (st != ALS_OK) return st;
    float *part_sc = (float *)ctx->topk_partials.p;
    int32_t *part_id = (int32_t *)(part_sc + part);
    constexpr int lds_bytes = TOPK_WAVES * (2 * TOPK_QPW * TOPK_CAP + 2 * TOPK_QPW) * 4;
    static const hipError_t attr = hipFuncSetAttribute((const void *)topk_scan_kernel<D, BF16>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);  // once
    ALS_HIP(ctx, attr);
    const unsigned qblocks = (unsigned)((Q->rows + TOPK_QPW * TOPK_WAVES - 1) / (TOPK_QPW * TOPK_WAVES));
    hipLaunchKernelGGL((topk_scan_kernel<D, BF16>), dim3(qblocks, slices), dim3(64 * TOPK_WAVES), lds_bytes, s, Q->data,
                       Q->ld, Q->rows, H->data, H->ld, H->rows, ex ? ex->indptr : nullptr, ex ? ex->indices : nullptr, k,
                       kpad, slice_items, part_sc, part_id);
    hipLaunchKernelGGL(topk_merge_kernel, dim3((unsigned)Q->rows), dim3(64), 0, s, (const float *)part_sc,
                       (const int32_t *)part_id, Q->rows, slices, kpad, k, ids, scores);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

als_status launch_topk(als_ctx *ctx, const als_table *Q, const als_table *H, const als_csr *ex, int k, int32_t *ids,
                       float *scores, hipStream_t s) {
    const bool bf = H->dtype == ALS_BF16;
    switch (H->d) {
        case 16: return bf ? topk_typed<16, true>(ctx, Q, H, ex, k, ids, scores, s) : topk_typed<16, false>(ctx, Q, H, ex, k, ids, scores, s);
        case 32: return bf ? topk_typed<32, true>(ctx, Q, H, ex, k, ids, scores, s) : topk_typed<32, false>(ctx, Q, H, ex, k, ids, scores, s);
        case 64: return bf ? topk_typed<64, true>(ctx, Q, H, ex, k, ids, scores, s) : topk_typed<64, false>(ctx, Q, H, ex, k, ids, scores, s);
        case 128: return bf ? topk_typed<128, true>(ctx, Q, H, ex, k, ids, scores, s) : topk_typed<128, false>(ctx, Q, H, ex, k, ids, scores, s);
    }
    return fail(ctx, ALS_EDTYPE, "unsupported d");
}

}  // namespace als
