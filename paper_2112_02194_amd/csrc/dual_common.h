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

// per-class launchers, one translation unit each (they compile in parallel)
void launch_dual_k16(int d, const als_csr *Y, const float *Z, float *R, int64_t ldr, int64_t r0, const int32_t *list,
                     int count, int32_t *err, hipStream_t s);

}  // namespace als
