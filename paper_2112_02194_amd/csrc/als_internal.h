// Internal declarations shared by the libals translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "als.h"

namespace als {

// ----------------------------------------------------------------------------------------------
// Operand geometry of the fp32 MFMA contractions X^T X (X = rows of a table, d columns).
//
// A lane owns NC consecutive columns [NC*m, NC*m+NC) of one table row and feeds component I
// as the A operand of output tile-row I and component J as the B operand of tile-column J, so
// tile (I,J) element (m,n) is entry (NC*m+I, NC*n+J) of X^T X.  This column interleave lets a
// lane fetch its operands with one vector load of NC elements, and a group of TM lanes fetch
// one whole table row as a single contiguous segment.
//   d=128: v_mfma_f32_32x32x2  TM=32 NC=4 KS=2 (two table rows per MFMA step)
//   d= 64: v_mfma_f32_16x16x4  TM=16 NC=4 KS=4
//   d= 32: v_mfma_f32_16x16x4  TM=16 NC=2 KS=4
//   d= 16: v_mfma_f32_16x16x4  TM=16 NC=1 KS=4
// ----------------------------------------------------------------------------------------------
template <int D> struct Geo;
template <> struct Geo<128> { static constexpr int TM = 32, NC = 4, KS = 2, ACC = 16; };
template <> struct Geo<64>  { static constexpr int TM = 16, NC = 4, KS = 4, ACC = 4; };
template <> struct Geo<32>  { static constexpr int TM = 16, NC = 2, KS = 4, ACC = 4; };
template <> struct Geo<16>  { static constexpr int TM = 16, NC = 1, KS = 4, ACC = 4; };

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int ACC> struct AccT;
template <> struct AccT<16> { typedef floatx16 type; };
template <> struct AccT<4>  { typedef floatx4 type; };

template <int D>
__device__ __forceinline__ typename AccT<Geo<D>::ACC>::type mfma(float a, float b,
                                                                typename AccT<Geo<D>::ACC>::type c) {
    if constexpr (Geo<D>::TM == 32) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
}

// Row index inside a TM x TM output tile of accumulator register v on `lane`; the column is lane % TM.
template <int D> __device__ __forceinline__ int acc_row(int v, int lane) {
    if constexpr (Geo<D>::TM == 32) {
        return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    } else {
        return 4 * (lane >> 4) + v;
    }
}

// ---------------------------------------------------------------------------------------------- element access
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) {  // inf / nan: keep the class, quiet the nan
        return (uint16_t)((u >> 16) | ((u & 0xffffu) ? 0x40u : 0u));
    }
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Load NC consecutive elements starting at element offset `off` (a multiple of NC) of a table.
template <int NC, bool BF16>
__device__ __forceinline__ void load_vec(const void *base, int64_t off, float (&x)[NC]) {
    if constexpr (!BF16) {
        const float *p = (const float *)base + off;
        if constexpr (NC == 4) {
            float4 t = *(const float4 *)p;
            x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
        } else if constexpr (NC == 2) {
            float2 t = *(const float2 *)p;
            x[0] = t.x; x[1] = t.y;
        } else {
            x[0] = *p;
        }
    } else {
        const uint16_t *p = (const uint16_t *)base + off;
        if constexpr (NC == 4) {
            uint2 t = *(const uint2 *)p;
            x[0] = __uint_as_float(t.x << 16); x[1] = __uint_as_float(t.x & 0xffff0000u);
            x[2] = __uint_as_float(t.y << 16); x[3] = __uint_as_float(t.y & 0xffff0000u);
        } else if constexpr (NC == 2) {
            uint32_t t = *(const uint32_t *)p;
            x[0] = __uint_as_float(t << 16); x[1] = __uint_as_float(t & 0xffff0000u);
        } else {
            x[0] = bf16_to_f32(*p);
        }
    }
}

template <bool BF16> __device__ __forceinline__ void store_elem(void *base, int64_t off, float v) {
    if constexpr (!BF16) {
        ((float *)base)[off] = v;
    } else {
        ((uint16_t *)base)[off] = f32_to_bf16_rne(v);
    }
}

template <bool BF16> __device__ __forceinline__ float load_elem(const void *base, int64_t off) {
    if constexpr (!BF16) {
        return ((const float *)base)[off];
    } else {
        return bf16_to_f32(((const uint16_t *)base)[off]);
    }
}

// ---------------------------------------------------------------------------------------------- context
struct DevBuf {
    void *p = nullptr;
    size_t bytes = 0;
};

// One slot per kernel (or pair of kernels timed together); T_DUAL_CLASS0 + c: dual row kernel of the class
// 16c < k <= 16(c+1) (c = 0: 8 < k <= 16).
enum TimingSlot { T_GRAMIAN = 0, T_CLASSIFY, T_TRANSFORM, T_TRANSFORM_X, T_PRIMAL, T_SEGMENT, T_REDUCE, T_SMALL4,
                  T_SMALL8, T_DUAL_CLASS0 = 9, T_COUNT = ALS_TIMING_SLOTS };

struct Timer {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int slot = 0;
};

constexpr int N_HINTS = 8, HINT_INTS = 32;  // per slot: [0..15] the counters, [16] the sequence number (written last)
struct HintSlot {
    const void *indptr = nullptr;  // key: the matrix (by address and size), the row range and what shapes the classes
    int64_t rows = 0, nnz = 0, r0 = 0, r1 = 0;
    int32_t split = 0, dual_max = 0, d = 0;
    uint32_t seq = 0;              // sequence number of the call that last enqueued a write of this slot; 0 = unused
    uint32_t first_seq = 0;        // sequence number of the first call with this key: counts stamped >= it belong to the key
};

}  // namespace als

struct als_ctx {
    int device = 0;
    std::string last_error;
    als::DevBuf gram_partials;  // fp32 [nblocks][d*d] per-workgroup Gramians
    als::DevBuf lists;          // long-row and segment descriptors
    als::DevBuf seg_partials;   // fp32 [nseg][d*d + d] partial statistics of long-row segments
    als::DevBuf ztable;         // fp32 [rows][d] transformed fixed table of the dual form
    als::DevBuf rtable;         // fp32 [rows][d] untransformed dual solutions when the output table is bf16
    als::DevBuf small;          // counters, flags, factor matrices, scalars
    als::DevBuf loss_partials;  // fp64 per-workgroup sums
    als::DevBuf topk_partials;  // per slice and query: best k scores and ids
    als::DevBuf gram_w, gram_h; // fp32 [d*d] Gramians used by als_epoch / als_loss
    int32_t *host_counters = nullptr;  // pinned, 16 ints
    double *host_scalar = nullptr;     // pinned, 2 doubles
    int num_cu = 256;                  // compute units of the device (sizes the default grids)
    // Launch-size hints.  als_solve_rows never waits for the row-class counts: its kernels read them
    // from device memory and walk their lists with grid-stride loops, so any grid is correct.  The counts
    // of a call are also stored (by the GPU, into host-visible memory) in one of these slots, and the next
    // call on the same matrix and range sizes its grids from them, so that every workgroup gets one item.
    als::HintSlot hints[als::N_HINTS];
    int32_t *hint_counts = nullptr;    // pinned, device-visible: [N_HINTS][HINT_INTS], written by the GPU
    int32_t *hint_counts_dev = nullptr;  // the same memory as the device addresses it
    uint32_t hint_seq = 0;
    bool timing = false;
    std::vector<als::Timer> timers;
    std::vector<als::Timer> free_timers;
    double timing_ms[2 * als::T_COUNT] = {0};  // ms per slot, then launches per slot
};

namespace als {

// Layout of ctx->small (byte offsets).
constexpr size_t SM_COUNTERS = 0;       // int32[16]: [0] n_long [1] n_seg [2] error flag [3] n_mid [4] csr check [5] k<=4 [6] 5<=k<=8 [7] split in use [8..15] dual classes
constexpr size_t SM_LONGSTAT = 128;     // int64[2]: entries and rows beyond the requested split (sizes the segments)
constexpr size_t SM_LOSS = 64;          // double[2]
constexpr size_t SM_FACTOR = 256;       // fp32 [2][128*128]: L^{-1} and scratch for the dual form
constexpr size_t SM_BYTES = SM_FACTOR + 2 * 128 * 128 * sizeof(float) + 128 * 128 * sizeof(double);

struct LongRow {   // a row whose statistics are accumulated by several segments
    int64_t row;
    int32_t seg_first, nseg;
};
struct Segment {   // entries [begin, end) of CSR arrays belonging to long row `slot`
    int64_t begin, end;
};

als_status fail(als_ctx *ctx, als_status st, const std::string &msg);
als_status ensure(als_ctx *ctx, DevBuf &b, size_t bytes);
void timer_begin(als_ctx *ctx, int slot, hipStream_t s);
void timer_end(als_ctx *ctx, hipStream_t s);
// How a list of `capacity` steps at most is launched when its length is only known on the device.  The
// row kernels come in two forms: one step per workgroup (launched with `known` workgroups, the length the
// previous call on the same matrix saw; steps beyond the true length return at once), and a grid-stride walk
// over everything from step `known` on (launched with `rest` workgroups; finds nothing to do when the hint
// was right).  Together they cover the list whatever the hint was.
struct StepGrid {
    unsigned known, rest;
};
StepGrid step_grid(const als_ctx *ctx, int64_t capacity, int64_t hint, int per_cu);

#define ALS_HIP(ctx, expr)                                                                      \
    do {                                                                                        \
        hipError_t e__ = (expr);                                                                \
        if (e__ != hipSuccess)                                                                  \
            return als::fail(ctx, ALS_EHIP, std::string(#expr) + ": " + hipGetErrorString(e__)); \
    } while (0)

// kernels' host launchers (each validates nothing: the API layer has done so)
als_status launch_gramian(als_ctx *ctx, const als_table *V, float *G, hipStream_t s);
hipError_t gramian_static_setup(int device);
als_status launch_gramian_static(int device, const als_table *V, float *G, hipStream_t s);
als_status launch_solve_rows(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                             const als_params *prm, als_table *X, int64_t r0, int64_t r1, hipStream_t s);
als_status launch_loss(als_ctx *ctx, const als_csr *Y, const als_table *W, const als_table *H,
                       const float *GW, const float *GH, const als_params *prm, double *out_dev, hipStream_t s);
als_status launch_check_csr(als_ctx *ctx, const als_csr *Y, int32_t *flag_dev, hipStream_t s);
als_status launch_topk(als_ctx *ctx, const als_table *Q, const als_table *H, const als_csr *ex, int k, int32_t *ids,
                       float *scores, hipStream_t s);
als_status launch_copy_probe(als_ctx *ctx, const void *src, void *dst, int64_t bytes, hipStream_t s);

}  // namespace als
