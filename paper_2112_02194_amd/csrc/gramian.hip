// Gramian G = V^T V of an embedding table (paper Section 3, the remark after Eq. 4; Algorithm 1
// line 2): a tall-skinny contraction over the table's rows on the fp32 matrix cores.
//
// Each wavefront walks a strided set of row groups; a lane fetches NC consecutive columns of one
// row with a single vector load and feeds them as both MFMA operands (see Geo<> for the column
// interleave), accumulating all (d/TM)^2 output tiles in registers.  The four wavefronts of a
// workgroup are summed through LDS in a fixed order, every workgroup writes one fp32 partial
// Gramian, and two further kernels add the partials in fp64 in a fixed order, so the result is
// reproducible bit for bit.  The grid grows with the table so that no fp32 summation chain inside
// the matrix core is longer than GRAM_CHAIN steps: on a 1e8-row table chains of 12 000 steps showed a
// relative error of 1.3e-5 on the diagonal (sums of squares), all of one sign.
#include <mutex>

#include "dual_common.h"

namespace als {

constexpr int GRAM_THREADS = 256;
constexpr int GRAM_CHAIN = 256;         // MFMA steps a wavefront accumulates in fp32
constexpr int GRAM_MAX_BLOCKS = 65536;  // beyond rows = 65536 * 4 * KS * GRAM_CHAIN the chains grow
constexpr int GRAM_SLICES = 64;         // fp64 partial sums of the second stage

template <int D, bool BF16>
__global__ __launch_bounds__(GRAM_THREADS, 2) void gramian_partial_kernel(const void *__restrict__ V, int64_t rows,
                                                                       int64_t ld, float *__restrict__ partials) {
    using G = Geo<D>;
    constexpr int NC = G::NC, TM = G::TM, KS = G::KS, ACC = G::ACC;
    typedef typename AccT<ACC>::type acc_t;
    __shared__ float red[D * D];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane % TM, kk = lane / TM;
    const int64_t wave_id = (int64_t)blockIdx.x * (GRAM_THREADS / 64) + wave;
    const int64_t nwaves = (int64_t)gridDim.x * (GRAM_THREADS / 64);

    acc_t acc[NC][NC];
#pragma unroll
    for (int i = 0; i < NC; ++i)
#pragma unroll
        for (int j = 0; j < NC; ++j)
#pragma unroll
            for (int v = 0; v < ACC; ++v) acc[i][j][v] = 0.f;

    // Rows r0 + kk, r0 advancing by nwaves*KS per MFMA step, in batches of U steps.  The loads of the next
    // batch are issued before the MFMAs of the current one (two register sets used alternately), so that
    // a wavefront always has a batch of rows in flight while the matrix core works.
    constexpr int U = 4;
    const int64_t step = nwaves * KS, batch = step * U;
    auto issue = [&](int64_t r0, float (&x)[U][NC]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t r = r0 + u * step + kk;
            if (r < rows) {
                load_vec<NC, BF16>(V, r * ld + NC * m, x[u]);
            } else {
#pragma unroll
                for (int c = 0; c < NC; ++c) x[u][c] = 0.f;
            }
        }
    };
    auto consume = [&](float (&x)[U][NC]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < NC; ++i)
#pragma unroll
                for (int j = i; j < NC; ++j)  // upper tiles only; the result is symmetric
                    acc[i][j] = mfma<D>(x[u][i], x[u][j], acc[i][j]);
    };
    float xa[U][NC], xb[U][NC];
    int64_t r0 = wave_id * KS;
    issue(r0, xa);
    for (; r0 < rows; r0 += 2 * batch) {
        issue(r0 + batch, xb);  // past the end: zeros, no loads
        consume(xa);
        issue(r0 + 2 * batch, xa);
        if (r0 + batch < rows) consume(xb);
    }

    // fixed-order sum of the four wavefronts through LDS
    for (int w = 0; w < GRAM_THREADS / 64; ++w) {
        if (wave == w) {
#pragma unroll
            for (int i = 0; i < NC; ++i)
#pragma unroll
                for (int j = i; j < NC; ++j)
#pragma unroll
                    for (int v = 0; v < ACC; ++v) {
                        const int r = NC * acc_row<D>(v, lane) + i, c = NC * m + j;
                        if (w == 0) red[r * D + c] = acc[i][j][v];
                        else red[r * D + c] += acc[i][j][v];
                    }
        }
        __syncthreads();
    }
    float *out = partials + (int64_t)blockIdx.x * D * D;
    for (int e = threadIdx.x; e < D * D; e += GRAM_THREADS) {
        const int r = e / D, c = e % D;
        // tile (i,j) with i<=j was computed, where i = r % NC, j = c % NC; otherwise mirror
        const bool have = (r % NC) <= (c % NC);
        out[e] = have ? red[r * D + c] : red[c * D + r];
    }
}

// ---------------------------------------------------------------------------------------------- bf16 tables
// The same contraction for bf16 tables (d = 64, 128) on the bf16 matrix cores, where a table pass is bound
// by HBM instead of by the fp32 matrix-core rate.  v_mfma_f32_32x32x16_bf16 wants, per lane, eight
// consecutive entries along the contraction index, which here is the table row - but a lane loads eight
// consecutive COLUMNS of one row (16 bytes).  The matrix core does the transposition itself: multiplying the
// 32 rows x 16 columns piece as loaded (rows = M, columns = K) by a constant 0/1 selection matrix leaves
// the piece in the accumulator layout, where a lane holds 16 rows of ONE column; products with 1 and sums
// with 0 are exact, so cutting the fp32 results back to bf16 loses nothing, and the packed registers are
// the K-contiguous operands of the Gramian products (both operands come from the same registers, so the
// order in which rows sit in the K slots does not matter).  Per 32 table rows and d = 128: 8 selection
// products + 20 Gramian products (upper block triangle) of 32 clocks each.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int D>
__global__ __launch_bounds__(GRAM_THREADS, 1) void gramian_bf16_kernel(const uint16_t *__restrict__ V, int64_t rows,
                                                                       int64_t ld, float *__restrict__ partials) {
    constexpr int NB = D / 32, NCH = D / 16;  // column blocks of 32, loaded pieces of 16 columns
    __shared__ float red[D * D];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, kq = lane >> 5;
    const int64_t wave_id = (int64_t)blockIdx.x * (GRAM_THREADS / 64) + wave;
    const int64_t nwaves = (int64_t)gridDim.x * (GRAM_THREADS / 64);

    // selection operands: sel[h] (K = 16 piece columns, N = 32 block columns) has a one at (k, 16 h + k)
    bf16x8 sel[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        u32x4 w = {0u, 0u, 0u, 0u};
        const int k = m - 16 * h - 8 * kq;  // the K slot of this lane (8 kq + e) that equals column m - 16 h
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (k == e) w[e / 2] = (e & 1) ? 0x3F800000u : 0x00003F80u;  // bf16 1.0 in the upper / lower half
        sel[h] = __builtin_bit_cast(bf16x8, w);
    }
    floatx16 acc[NB][NB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // 32 rows per step (lane (m, kq) loads columns 16 c + 8 kq .. of row r0 + m); the loads of the next step are
    // issued before the products of the current one
    auto issue = [&](int64_t r0, u32x4 (&raw)[NCH]) {
        const int64_t r = r0 + m;
#pragma unroll
        for (int c = 0; c < NCH; ++c) raw[c] = u32x4{0u, 0u, 0u, 0u};
        if (r < rows) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) raw[c] = *(const u32x4 *)(V + r * ld + 16 * c + 8 * kq);
        }
    };
    auto consume = [&](u32x4 (&raw)[NCH]) {
        bf16x8 op[NB][2];  // per column block: rows 0..15 and 16..31 of the step in the K slots
#pragma unroll
        for (int g = 0; g < NB; ++g) {
            floatx16 t;
#pragma unroll
            for (int v = 0; v < 16; ++v) t[v] = 0.f;
            t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw[2 * g]), sel[0], t, 0, 0, 0);
            t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw[2 * g + 1]), sel[1], t, 0, 0, 0);
            // t[v] = V[r0 + 8 (v / 4) + 4 kq + v % 4][32 g + m], exactly a bf16 value
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const u32x4 w = {__builtin_amdgcn_perm(__float_as_uint(t[8 * x + 1]), __float_as_uint(t[8 * x + 0]), 0x07060302u),
                                 __builtin_amdgcn_perm(__float_as_uint(t[8 * x + 3]), __float_as_uint(t[8 * x + 2]), 0x07060302u),
                                 __builtin_amdgcn_perm(__float_as_uint(t[8 * x + 5]), __float_as_uint(t[8 * x + 4]), 0x07060302u),
                                 __builtin_amdgcn_perm(__float_as_uint(t[8 * x + 7]), __float_as_uint(t[8 * x + 6]), 0x07060302u)};
                op[g][x] = __builtin_bit_cast(bf16x8, w);
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int j = i; j < NB; ++j) {  // upper block triangle; the result is symmetric
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[i][0], op[j][0], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[i][1], op[j][1], acc[i][j], 0, 0, 0);
            }
    };
    u32x4 ra[NCH], rb[NCH];
    const int64_t step = nwaves * 32;
    int64_t r0 = wave_id * 32;
    issue(r0, ra);
    for (; r0 < rows; r0 += 2 * step) {
        issue(r0 + step, rb);  // past the end: zeros, no loads
        consume(ra);
        issue(r0 + 2 * step, ra);
        if (r0 + step < rows) consume(rb);
    }

    // fixed-order sum of the four wavefronts through LDS: acc[i][j][v] = G[32 i + row(v)][32 j + m]
    for (int w = 0; w < GRAM_THREADS / 64; ++w) {
        if (wave == w) {
#pragma unroll
            for (int i = 0; i < NB; ++i)
#pragma unroll
                for (int j = i; j < NB; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int r = 32 * i + 8 * (v >> 2) + 4 * kq + (v & 3), c = 32 * j + m;
                        if (w == 0) red[r * D + c] = acc[i][j][v];
                        else red[r * D + c] += acc[i][j][v];
                    }
        }
        __syncthreads();
    }
    float *out = partials + (int64_t)blockIdx.x * D * D;
    for (int e = threadIdx.x; e < D * D; e += GRAM_THREADS) {
        const int r = e / D, c = e % D;
        out[e] = (r / 32) <= (c / 32) ? red[r * D + c] : red[c * D + r];
    }
}

// ---------------------------------------------------------------------------------------------- fp32 tables, d >= 64
// fp32 tables on the same bf16 matrix cores: every entry is cut into three bf16 parts, x = h + m + l exactly
// (8 + 8 + 8 significant bits: h = upper 16 bits of x, m = upper 16 bits of x - h, l = the rest), each part
// is transposed by the matrix core as above, and a product x y is taken as hh' + hm' + mh' + hl' + lh' + mm'
// (what is dropped - ml', lm', ll' - is below 2^-23 |x y|, the rounding of an fp32 product).  Per 32 table rows
// and d = 128: 24 selection products + 120 Gramian products of 32 clocks, 4 600 clocks against the 10 240 that
// the same ten blocks take on the fp32 matrix instruction: 2.2 times less matrix-core time, which leaves the
// pass bound by the table read.  The two cross terms of a pair of parts enter a diagonal block in
// different order at (r, c) and (c, r), so the output takes the lower triangle from the upper one element by
// element (symmetric to the bit).  The raw registers of a column block are refilled with the next step's rows
// as soon as that block has been cut, so that loads are in flight during the products.
constexpr int GRAM_SPLIT_STEPS = 64;  // 32-row steps a wavefront sums before its workgroup writes a partial

template <int D>
__global__ __launch_bounds__(GRAM_THREADS, 1) void gramian_split_kernel(const float *__restrict__ V, int64_t rows,
                                                                        int64_t ld, float *__restrict__ partials) {
    constexpr int NB = D / 32;  // column blocks of 32 = two loaded pieces of 16 columns
    __shared__ float red[D * D];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, kq = lane >> 5;
    const int64_t wave_id = (int64_t)blockIdx.x * (GRAM_THREADS / 64) + wave;
    const int64_t nwaves = (int64_t)gridDim.x * (GRAM_THREADS / 64);
    bf16x8 sel[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        u32x4 w = {0u, 0u, 0u, 0u};
        const int k = m - 16 * h - 8 * kq;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (k == e) w[e / 2] = (e & 1) ? 0x3F800000u : 0x00003F80u;
        sel[h] = __builtin_bit_cast(bf16x8, w);
    }
    floatx16 acc[NB][NB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // raw[g][c][0..1]: columns 32 g + 16 c + 8 kq .. + 7 of row r0 + m
    float4 raw[NB][2][2];
    auto issue = [&](int64_t r0, int g) {
        const int64_t r = r0 + m;
#pragma unroll
        for (int c = 0; c < 2; ++c) raw[g][c][0] = raw[g][c][1] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < rows) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const float *src = V + r * ld + 32 * g + 16 * c + 8 * kq;
                raw[g][c][0] = *(const float4 *)src;
                raw[g][c][1] = *(const float4 *)(src + 4);
            }
        }
    };
    auto upper = [](float x, float y) { return __builtin_amdgcn_perm(__float_as_uint(y), __float_as_uint(x), 0x07060302u); };
    auto rest = [](float x) { return x - __uint_as_float(__float_as_uint(x) & 0xffff0000u); };
    // the three parts of eight consecutive entries as matrix-core operands
    auto cut = [&](const float4 &a, const float4 &b, u32x4 (&part)[3]) {
        float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int t = 0; t < 3; ++t) {
#pragma unroll
            for (int e = 0; e < 4; ++e) part[t][e] = upper(x[2 * e], x[2 * e + 1]);
            if (t < 2) {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = rest(x[e]);
            }
        }
    };
    const int64_t step = nwaves * 32;
    int64_t r0 = wave_id * 32;
#pragma unroll
    for (int g = 0; g < NB; ++g) issue(r0, g);
    for (; r0 < rows; r0 += step) {
        bf16x8 op[3][NB][2];  // per part and column block: rows 0..15 and 16..31 of the step in the K slots
#pragma unroll
        for (int g = 0; g < NB; ++g) {
            u32x4 p0[3], p1[3];
            cut(raw[g][0][0], raw[g][0][1], p0);
            cut(raw[g][1][0], raw[g][1][1], p1);
            if (g < NB / 2) issue(r0 + step, g);  // past the end: zeros, no loads
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                floatx16 tr;
#pragma unroll
                for (int v = 0; v < 16; ++v) tr[v] = 0.f;
                tr = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, p0[t]), sel[0], tr, 0, 0, 0);
                tr = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, p1[t]), sel[1], tr, 0, 0, 0);
#pragma unroll
                for (int x = 0; x < 2; ++x) {
                    const u32x4 w = {upper(tr[8 * x + 0], tr[8 * x + 1]), upper(tr[8 * x + 2], tr[8 * x + 3]),
                                     upper(tr[8 * x + 4], tr[8 * x + 5]), upper(tr[8 * x + 6], tr[8 * x + 7])};
                    op[t][g][x] = __builtin_bit_cast(bf16x8, w);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int j = i; j < NB; ++j) {
                if (i == 1 && j == 1) {  // the other half of the next step's loads: their registers are free only now
#pragma unroll
                    for (int g = NB / 2; g < NB; ++g) issue(r0 + step, g);
                }
                // the step's twelve products are summed inside the matrix core from zero (small terms first), and the
                // step's sum joins the running sum by a vector addition, which rounds to nearest: no long chain
                // of the matrix core's one-sided additions builds up
                constexpr int PA[6] = {1, 2, 0, 1, 0, 0}, PB[6] = {1, 0, 2, 0, 1, 0};  // mm lh hl mh hm hh
                floatx16 t16;
#pragma unroll
                for (int v = 0; v < 16; ++v) t16[v] = 0.f;
#pragma unroll
                for (int t = 0; t < 6; ++t) {
                    t16 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[PA[t]][i][0], op[PB[t]][j][0], t16, 0, 0, 0);
                    t16 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[PA[t]][i][1], op[PB[t]][j][1], t16, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] += t16[v];
            }
    }
    for (int w = 0; w < GRAM_THREADS / 64; ++w) {
        if (wave == w) {
#pragma unroll
            for (int i = 0; i < NB; ++i)
#pragma unroll
                for (int j = i; j < NB; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int r = 32 * i + 8 * (v >> 2) + 4 * kq + (v & 3), c = 32 * j + m;
                        if (w == 0) red[r * D + c] = acc[i][j][v];
                        else red[r * D + c] += acc[i][j][v];
                    }
        }
        __syncthreads();
    }
    float *out = partials + (int64_t)blockIdx.x * D * D;
    for (int e = threadIdx.x; e < D * D; e += GRAM_THREADS) {
        const int r = e / D, c = e % D;
        out[e] = r <= c ? red[r * D + c] : red[c * D + r];
    }
}

// Stage 2: slice y of gridDim.y adds the partials b = y, y + gridDim.y, ... in fp64.
template <int D>
__global__ __launch_bounds__(256) void gramian_slice_kernel(const float *__restrict__ partials, int nblocks,
                                                            double *__restrict__ slices) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= D * D) return;
    double s = 0.0;
#pragma unroll 4
    for (int b = blockIdx.y; b < nblocks; b += gridDim.y) s += (double)partials[(int64_t)b * D * D + e];
    slices[(int64_t)blockIdx.y * D * D + e] = s;
}

// Stage 3: the slices in order.
template <int D>
__global__ __launch_bounds__(256) void gramian_reduce_kernel(const double *__restrict__ slices, int nslices,
                                                             float *__restrict__ G) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= D * D) return;
    double s = 0.0;
    for (int b = 0; b < nslices; ++b) s += slices[(int64_t)b * D * D + e];
    G[e] = (float)s;
}

template <int D, bool BF16> constexpr bool gram_bf16_cores() { return BF16 && D >= 64; }
template <int D, bool BF16> constexpr bool gram_split_cores() { return !BF16 && D >= 64; }

template <int D, bool BF16 = false> static int gramian_blocks(int64_t rows) {
    // rows a workgroup may take so that no accumulator sees more than GRAM_CHAIN matrix-core additions
    // (the bf16 kernel adds twice per 32-row step; the split kernel sums the steps on the vector units)
    int64_t per_block = gram_bf16_cores<D, BF16>() ? (int64_t)(GRAM_THREADS / 64) * 32 * (GRAM_CHAIN / 2)
                                                   : (int64_t)(GRAM_THREADS / 64) * Geo<D>::KS * GRAM_CHAIN;
    if constexpr (gram_split_cores<D, BF16>()) {
        // at most GRAM_SPLIT_STEPS steps per wavefront, down to 16 for smaller tables so that more workgroups exist
        constexpr int64_t unit = (int64_t)(GRAM_THREADS / 64) * 32;
        per_block = std::min<int64_t>(unit * GRAM_SPLIT_STEPS, std::max<int64_t>(16 * unit, (rows / 1024 + unit - 1) / unit * unit));
    }
    return (int)std::min<int64_t>(GRAM_MAX_BLOCKS, std::max<int64_t>(1, (rows + per_block - 1) / per_block));
}

// The three launches; `work` holds nblocks fp32 partials followed by nslices fp64 slices.
template <int D, bool BF16>
static void gramian_enqueue(const als_table *V, float *G, void *work, int nblocks, int nslices, hipStream_t s) {
    float *partials = (float *)work;
    double *slices = (double *)((char *)work + (size_t)nblocks * D * D * sizeof(float));
    if constexpr (gram_bf16_cores<D, BF16>())
        hipLaunchKernelGGL((gramian_bf16_kernel<D>), dim3(nblocks), dim3(GRAM_THREADS), 0, s, (const uint16_t *)V->data,
                           V->rows, V->ld, partials);
    else if constexpr (gram_split_cores<D, BF16>())
        hipLaunchKernelGGL((gramian_split_kernel<D>), dim3(nblocks), dim3(GRAM_THREADS), 0, s, (const float *)V->data,
                           V->rows, V->ld, partials);
    else
        hipLaunchKernelGGL((gramian_partial_kernel<D, BF16>), dim3(nblocks), dim3(GRAM_THREADS), 0, s, V->data, V->rows,
                           V->ld, partials);
    hipLaunchKernelGGL((gramian_slice_kernel<D>), dim3((D * D + 255) / 256, nslices), dim3(256), 0, s,
                       (const float *)partials, nblocks, slices);
    hipLaunchKernelGGL((gramian_reduce_kernel<D>), dim3((D * D + 255) / 256), dim3(256), 0, s,
                       (const double *)slices, nslices, G);
}

template <int D, bool BF16>
static als_status gramian_typed(als_ctx *ctx, const als_table *V, float *G, hipStream_t s) {
    const int nblocks = gramian_blocks<D, BF16>(V->rows);
    const int nslices = std::min(nblocks, GRAM_SLICES);
    als_status st = ensure(ctx, ctx->gram_partials, (size_t)nblocks * D * D * sizeof(float) +
                                                        (size_t)nslices * D * D * sizeof(double));
    if (st != ALS_OK) return st;
    timer_begin(ctx, T_GRAMIAN, s);
    gramian_enqueue<D, BF16>(V, G, ctx->gram_partials.p, nblocks, nslices, s);
    timer_end(ctx, s);
    ALS_HIP(ctx, hipGetLastError());
    return ALS_OK;
}

als_status launch_gramian(als_ctx *ctx, const als_table *V, float *G, hipStream_t s) {
    const bool bf = V->dtype == ALS_BF16;
    switch (V->d) {
        case 16: return bf ? gramian_typed<16, true>(ctx, V, G, s) : gramian_typed<16, false>(ctx, V, G, s);
        case 32: return bf ? gramian_typed<32, true>(ctx, V, G, s) : gramian_typed<32, false>(ctx, V, G, s);
        case 64: return bf ? gramian_typed<64, true>(ctx, V, G, s) : gramian_typed<64, false>(ctx, V, G, s);
        case 128: return bf ? gramian_typed<128, true>(ctx, V, G, s) : gramian_typed<128, false>(ctx, V, G, s);
    }
    return fail(ctx, ALS_EDTYPE, "unsupported d");
}

// ---------------------------------------------------------------------------------------------- no allocation
// als_gramian_static: the same kernels with their partial sums in a file-scope device array instead of
// the context's workspace, for callers that cannot allocate.  Every GPU holds its own copy of the array
// at its own address; the address is looked up once per device (with that device current) and kept.
// Nothing in the array has to start at zero: every partial and slice that is read has been written by
// the same call.  Calls that overlap on one GPU share the array and race.
constexpr int STATIC_BLOCKS = 128;   // 262 144 rows at d = 128 (2048 rows per workgroup)
constexpr int STATIC_SLICES = 16;
constexpr size_t STATIC_BYTES = (size_t)STATIC_BLOCKS * 128 * 128 * sizeof(float) +
                                (size_t)STATIC_SLICES * 128 * 128 * sizeof(double);
static __device__ __align__(256) unsigned char scratch[STATIC_BYTES];

constexpr int STATIC_MAX_DEVICES = 64;
static void *scratch_ptr[STATIC_MAX_DEVICES];  // per device, null until looked up
static std::mutex scratch_mutex;

// Device address of this GPU's copy of the array; `device` must be current.
hipError_t gramian_static_setup(int device) {
    if (device < 0 || device >= STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_ptr[device]) return hipSuccess;
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    scratch_ptr[device] = p;
    return hipSuccess;
}

template <int D, bool BF16>
static als_status gramian_static_typed(const als_table *V, float *G, void *work, hipStream_t s) {
    // the caller has checked the row count: with STATIC_BLOCKS workgroups no wavefront exceeds its step limit
    // (the kernels stride over the table, so fewer workgroups only means more steps each)
    const int nblocks = std::min(gramian_blocks<D, BF16>(V->rows), STATIC_BLOCKS);
    gramian_enqueue<D, BF16>(V, G, work, nblocks, std::min(nblocks, STATIC_SLICES), s);
    return hipGetLastError() == hipSuccess ? ALS_OK : ALS_EHIP;
}

als_status launch_gramian_static(int device, const als_table *V, float *G, hipStream_t s) {
    if (gramian_static_setup(device) != hipSuccess) return ALS_EHIP;
    void *work = scratch_ptr[device];
    const bool bf = V->dtype == ALS_BF16;
    switch (V->d) {
        case 16: return bf ? gramian_static_typed<16, true>(V, G, work, s) : gramian_static_typed<16, false>(V, G, work, s);
        case 32: return bf ? gramian_static_typed<32, true>(V, G, work, s) : gramian_static_typed<32, false>(V, G, work, s);
        case 64: return bf ? gramian_static_typed<64, true>(V, G, work, s) : gramian_static_typed<64, false>(V, G, work, s);
        case 128: return bf ? gramian_static_typed<128, true>(V, G, work, s) : gramian_static_typed<128, false>(V, G, work, s);
    }
    return ALS_EDTYPE;
}

}  // namespace als
