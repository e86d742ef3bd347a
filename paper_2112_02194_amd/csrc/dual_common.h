// Helpers shared by the translation units of the dual (k x k) row update.
#pragma once

#include <cstdlib>
#include <type_traits>

#include "als_internal.h"

namespace als {

__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Makes a wavefront-uniform value opaque to the optimiser.  The grid-stride forms of the row kernels pass their
// arguments through this at the top of every iteration: with nothing loop-invariant left in sight, the
// compiler cannot hoist the step's address arithmetic out of the loop, which otherwise costs the step about
// twice its registers (and scratch memory for the larger steps).
template <class T> __device__ __forceinline__ T opaque(T v) {
    asm volatile("" : "+s"(v));
    return v;
}
__device__ __forceinline__ int opaque_tid() {
    int lane = threadIdx.x;
    asm volatile("" : "+v"(lane));
    return lane;
}

// Four consecutive entries of a row list, read with one load.  The lists start at arbitrary 4-byte offsets of
// the workspace (which is padded so that reading up to three entries past a list's end stays inside it).
struct __attribute__((packed, aligned(4))) ListQuad { int32_t x, y, z, w; };

template <int B, int E, class F> __device__ __forceinline__ void static_for(F &&f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// Value of lane C of this lane's group of GW consecutive lanes (GW = 16: DPP row broadcast,
// GW = 32: LDS-crossbar swizzle, GW = 64: scalar read of the lane).
template <int GW, int C> __device__ __forceinline__ float group_bcast(float x) {
    if constexpr (GW == 16) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + C, 0xf, 0xf, true));
    } else if constexpr (GW == 32) {
        return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), C << 5));
    } else {
        return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), C));
    }
}

// ---------------------------------------------------------------------------------------------- fused broadcasts
// acc += (src as held by lane C of this lane's row of 16 lanes) * mul in ONE vector instruction: the row
// broadcast is a DPP modifier of the multiply-add (the compiler emits a separate broadcast move and a
// three-operand multiply-add instead).  The hardware needs two idle issue slots between a vector
// instruction that writes a register and a DPP read of it, and does not interlock: dpp_settle() must be
// applied to every register that one of these instructions (or a plain vector instruction right before)
// has written and that is read through DPP next; the dependence it creates also keeps the compiler from
// moving such a read in front of it.
template <int C> __device__ __forceinline__ void fmac_bcast16(float &acc, float src, float mul) {
    asm volatile("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                 : "+v"(acc)
                 : "v"(src), "v"(mul), "n"(C));
}
__device__ __forceinline__ void dpp_settle(float &a) { asm volatile("s_nop 1" : "+v"(a)); }
__device__ __forceinline__ void dpp_settle(float &a, float &b) { asm volatile("s_nop 1" : "+v"(a), "+v"(b)); }

// ---------------------------------------------------------------------------------------------- split products
// S = I + Z_I Z_I^T on the bf16 matrix cores at fp32-like accuracy: every fp32 entry z is cut into
// hi = its upper 16 bits (a bf16 number) and lo = the upper 16 bits of z - hi (z - hi is exact), so that
// z = hi + lo up to 2^-16 |z|, and a product z z' is taken as hi hi' + hi lo' + lo hi' (the dropped
// lo lo' is below 2^-16 |z z'|).  Three v_mfma_f32_16x16x32_bf16 (16 clocks each, 32 columns deep) replace
// eight v_mfma_f32_16x16x4_f32 (32 clocks each): a fifth of the matrix-core time for three vector
// instructions per entry.  Accumulation is fp32 as before.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
struct SplitOperand { bf16x8 hi, lo; };  // eight columns of one table row

// Upper halves of x (low 16 bits of the result) and y (high 16 bits).
__device__ __forceinline__ uint32_t pack_upper(float x, float y) {
    return __builtin_amdgcn_perm(__float_as_uint(y), __float_as_uint(x), 0x07060302u);
}
__device__ __forceinline__ float lower_part(float x) { return x - __uint_as_float(__float_as_uint(x) & 0xffff0000u); }

// Operand of one 32-column step from two 16-byte pieces of a row (the column order inside the step is the
// same for both operands of a product, so it does not matter).
__device__ __forceinline__ SplitOperand split_operand(const float4 &p, const float4 &r) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 h = {pack_upper(p.x, p.y), pack_upper(p.z, p.w), pack_upper(r.x, r.y), pack_upper(r.z, r.w)};
    const u32x4 l = {pack_upper(lower_part(p.x), lower_part(p.y)), pack_upper(lower_part(p.z), lower_part(p.w)),
                     pack_upper(lower_part(r.x), lower_part(r.y)), pack_upper(lower_part(r.z), lower_part(r.w))};
    SplitOperand o;
    o.hi = __builtin_bit_cast(bf16x8, h);
    o.lo = __builtin_bit_cast(bf16x8, l);
    return o;
}

// acc += A B^T over the step's 32 columns (A supplies the tile's rows 4q+v, B its column a, as with the
// fp32 instruction).
__device__ __forceinline__ floatx4 split_mfma(const SplitOperand &a, const SplitOperand &b, floatx4 acc) {
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.hi, b.hi, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.hi, b.lo, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.lo, b.hi, acc, 0, 0, 0);
    return acc;
}

// Selection operands of v_mfma_f32_16x16x32_bf16: h[x] (depth 32, 16 columns) has a one at (16 x + n, n).  A
// 16 x 32 operand times h[x] is its columns 16 x .. 16 x + 15 in the accumulator layout, exactly: the matrix
// core used as a transposer.
struct SelOperands { bf16x8 h[2]; };
__device__ __forceinline__ SelOperands make_sel(int lane) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int n = lane & 15, kq = lane >> 4;
    SelOperands s;
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        // this lane holds depth slots 8 kq .. 8 kq + 7 of column n; the one sits at slot 16 x + n
        const int w = 16 * x + n - 8 * kq;  // 0 .. 7 if it is one of them
        u32x4 v;
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = w == 2 * c ? 0x00003f80u : (w == 2 * c + 1 ? 0x3f800000u : 0u);
        s.h[x] = __builtin_bit_cast(bf16x8, v);
    }
    return s;
}

// ---------------------------------------------------------------------------------------------- the table Z
// The row kernels read the transformed table Z = V L^-T either as fp32 (fp32 tables) or as bf16 (ZB: bf16
// tables with d >= 32, where Z is rounded once to the tables' own element type).  A lane (a, q) of a
// 16-entry tile holds an entry's row as 16-byte pieces: piece j covers columns (4 j + q) * EPP .. with EPP = 4
// (fp32) or 8 (bf16) elements, so that a bf16 piece is, as loaded, one operand of v_mfma_f32_16x16x32_bf16.
template <bool ZB> struct ZT {
    static constexpr int ES = ZB ? 2 : 4, EPP = 16 / ES;
};
template <int D, bool ZB> constexpr int z_pieces() { return D * ZT<ZB>::ES / 64; }

template <int D, bool ZB> __device__ __forceinline__ float4 load_piece(const void *Z, int64_t id, int j, int q) {
    return *(const float4 *)((const char *)Z + (id * D + (4 * j + q) * ZT<ZB>::EPP) * ZT<ZB>::ES);
}

// CPL adjacent columns starting at column CPL * lane of the row stored at `row` (global memory or LDS), as fp32
template <bool ZB, int CPL> __device__ __forceinline__ void row_cols(const void *row, int lane, float (&c)[CPL]) {
    if constexpr (!ZB) {
        if constexpr (CPL == 2) {
            const float2 v = *(const float2 *)((const float *)row + 2 * lane);
            c[0] = v.x;
            c[1] = v.y;
        } else {
            c[0] = ((const float *)row)[lane];
        }
    } else {
        if constexpr (CPL == 2) {
            const uint32_t v = ((const uint32_t *)row)[lane];
            c[0] = __uint_as_float(v << 16);
            c[1] = __uint_as_float(v & 0xffff0000u);
        } else {
            c[0] = __uint_as_float((uint32_t)((const uint16_t *)row)[lane] << 16);
        }
    }
}

// acc += A B^T over all columns of two entries' bf16 rows held as NP pieces each
template <int NP> __device__ __forceinline__ floatx4 mfma_pieces_bf16(const float4 (&A)[NP], const float4 (&B)[NP], floatx4 acc) {
#pragma unroll
    for (int j = 0; j < NP; ++j)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A[j]), __builtin_bit_cast(bf16x8, B[j]), acc, 0, 0, 0);
    return acc;
}

// A lane's share of a 16-entry tile (d >= 32) ready for the S products: the bf16 pieces as loaded, or the hi/lo
// operands cut from fp32 pieces.
template <int D, bool ZB> struct TileOperand {
    static constexpr int N = D / 32;
    typename std::conditional<ZB, float4, SplitOperand>::type v[N];
    __device__ __forceinline__ void set(const float4 (&raw)[z_pieces<D, ZB>()]) {
#pragma unroll
        for (int h = 0; h < N; ++h) {
            if constexpr (ZB) v[h] = raw[h];
            else v[h] = split_operand(raw[2 * h], raw[2 * h + 1]);
        }
    }
};
template <int D, bool ZB>
__device__ __forceinline__ floatx4 tile_product(const TileOperand<D, ZB> &A, const TileOperand<D, ZB> &B, floatx4 acc) {
#pragma unroll
    for (int h = 0; h < D / 32; ++h) {
        if constexpr (ZB)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A.v[h]), __builtin_bit_cast(bf16x8, B.v[h]), acc, 0, 0, 0);
        else
            acc = split_mfma(A.v[h], B.v[h], acc);
    }
    return acc;
}

// ---------------------------------------------------------------------------------------------- r = Z_I^T t on chip
// r = Z_I^T t from tiles that are still in registers as S operands, on the matrix cores.  The product contracts
// over the entries, so the tiles are needed with the entries along the operand's depth: a tile operand times
// a selection operand is the same numbers in the accumulator layout (one column, entries 4q .. 4q+3 per lane),
// exactly, and two tiles packed that way are the depth-32 operand of 16 columns.  The other operand (`top`,
// one per pair of tiles) holds t cut into three bf16 parts, t = p0 + p1 + p2 exactly, in its rows 0 .. 2 and
// zeros below; rows 0 .. 2 of the product, summed, are r on those 16 columns with fp32 accuracy.  out[2 j + x]
// accumulates the product for operand piece j, half x; column_of_result() names the column a lane holds there.
//
// t_operand(): `mine` points at this lane's part of t (p0, p1, p2 or a block of zeros by its row a = lane % 16)
// plus 4 q; the parts are fp32 numbers of which the operand takes the upper 16 bits.
__device__ __forceinline__ bf16x8 t_operand(const float *mine, bool second_tile) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const float4 ta = *(const float4 *)mine;
    float4 tb = make_float4(0.f, 0.f, 0.f, 0.f);
    if (second_tile) tb = *(const float4 *)(mine + 16);
    const u32x4 w = {pack_upper(ta.x, ta.y), pack_upper(ta.z, ta.w), pack_upper(tb.x, tb.y), pack_upper(tb.z, tb.w)};
    return __builtin_bit_cast(bf16x8, w);
}
// the two remainders of the cut: x - upper16(x) is exact
__device__ __forceinline__ void t_parts(float x0, float &x1, float &x2) {
    x1 = lower_part(x0);
    x2 = lower_part(x1);
}

template <int NT, int NP, class Tile>  // Tile(t, j): operand piece j (32 columns) of tile t as bf16x8
__device__ __forceinline__ void zt_times_t(Tile &&tile, const bf16x8 (&top)[(NT + 1) / 2], const SelOperands &sel,
                                           floatx4 (&out)[2 * NP]) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const floatx4 zero = floatx4{0.f, 0.f, 0.f, 0.f};
    static_for<0, NP>([&](auto jj) {
        constexpr int j = decltype(jj)::value;
        static_for<0, 2>([&](auto xx) {
            constexpr int x = decltype(xx)::value;
            static_for<0, (NT + 1) / 2>([&](auto pp) {
                constexpr int P = decltype(pp)::value;
                const floatx4 d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tile(2 * P, j), sel.h[x], zero, 0, 0, 0);
                floatx4 d1 = zero;
                if constexpr (2 * P + 1 < NT) d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tile(2 * P + 1, j), sel.h[x], zero, 0, 0, 0);
                const u32x4 zw = {pack_upper(d0[0], d0[1]), pack_upper(d0[2], d0[3]), pack_upper(d1[0], d1[1]), pack_upper(d1[2], d1[3])};
                out[2 * j + x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(top[P], __builtin_bit_cast(bf16x8, zw), out[2 * j + x], 0, 0, 0);
            });
        });
    });
}
// Column of r that lanes (n, q = 0) hold in out[2 j + x]: depth slot 16 x + n of operand piece j, and a bf16
// piece is 32 consecutive columns.  (Only bf16 tiles are exact operands; the hi + lo operands cut from fp32
// tiles carry an entry to 2^-16 only, which is enough for S but would show in r.)
__device__ __forceinline__ int column_of_result(int j, int x, int n) { return 32 * j + 16 * x + n; }

// The conjugate-gradient solvers work with squared residual norms: below this the squares lose their bits to
// the bottom of the fp32 range and step lengths formed from them are noise, so a residual with |r|^2 at or
// below it (|r| <= 1e-15) counts as converged whatever the right-hand side's size.
constexpr float CG_RESIDUAL_FLOOR = 1e-30f;

// How the one-row-per-wavefront kernels solve their k x k system: the panel elimination, or conjugate gradients
// with these limits.
struct WideSolver {
    bool cg;
    int iters;
    float tol;
};

// per-class launchers, one translation unit each (they compile in parallel)
// (`count_dev`: device address of the list's length; `g`: see StepGrid)
// `zb16`: Z is stored as bf16
void launch_dual_k16(int d, const als_csr *Y, const void *Z, bool zb16, float *R, int64_t ldr, int64_t r0,
                     const int32_t *list, const int32_t *count_dev, StepGrid g, int32_t *err, hipStream_t s);

}  // namespace als
