// Wavefront-wide reductions for the 64-lane wavefronts of gfx950, shared by the gate and the
// routing bookkeeping kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace emoe {

// Wavefront reductions on the DPP network (no LDS round trips): row_shr 1,2,4,8 leave each row's
// result in its lane 15, row_bcast15 / row_bcast31 carry it across rows, lane 63 ends up with the
// whole wavefront's result, which is then read back as a scalar.  Lanes without a source take the
// operation's identity.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i32(int identity, int v)
{
    return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xf, false);
}
#define EMOE_DPP_REDUCE(STEP)                                                             \
    STEP(0x111, 0xf) STEP(0x112, 0xf) STEP(0x114, 0xf) STEP(0x118, 0xf) /* row_shr 1,2,4,8 */ \
    STEP(0x142, 0xa) STEP(0x143, 0xc)                                   /* row_bcast15, 31 */

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v)
{
    unsigned hi = (unsigned)(v >> 32), lo = (unsigned)v;
#define STEP(CTRL, MASK)                                                                   \
    {                                                                                      \
        const unsigned ohi = (unsigned)dpp_i32<CTRL, MASK>(0, (int)hi);                    \
        const unsigned olo = (unsigned)dpp_i32<CTRL, MASK>(0, (int)lo);                    \
        const bool take = ohi > hi || (ohi == hi && olo > lo);                             \
        hi = take ? ohi : hi;                                                              \
        lo = take ? olo : lo;                                                              \
    }
    EMOE_DPP_REDUCE(STEP)
#undef STEP
    hi = (unsigned)__builtin_amdgcn_readlane((int)hi, 63);
    lo = (unsigned)__builtin_amdgcn_readlane((int)lo, 63);
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#define STEP(CTRL, MASK) { const uint32_t o = (uint32_t)dpp_i32<CTRL, MASK>(0, (int)v); v = o > v ? o : v; }
    EMOE_DPP_REDUCE(STEP)
#undef STEP
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ int wave_min_i32(int v)
{
#define STEP(CTRL, MASK) { const int o = dpp_i32<CTRL, MASK>(0x7fffffff, v); v = o < v ? o : v; }
    EMOE_DPP_REDUCE(STEP)
#undef STEP
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int wave_sum_i32(int v)
{
#define STEP(CTRL, MASK) v += dpp_i32<CTRL, MASK>(0, v);
    EMOE_DPP_REDUCE(STEP)
#undef STEP
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ float wave_max_f32(float v)
{
    const int ninf = (int)0xff800000u;
#define STEP(CTRL, MASK) v = fmaxf(v, __int_as_float(dpp_i32<CTRL, MASK>(ninf, __float_as_int(v))));
    EMOE_DPP_REDUCE(STEP)
#undef STEP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
// Orders this wavefront's LDS traffic: writes before it are visible to every lane after it.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ float wave_sum_f32(float v)
{
#define STEP(CTRL, MASK) v += __int_as_float(dpp_i32<CTRL, MASK>(0, __float_as_int(v)));
    EMOE_DPP_REDUCE(STEP)
#undef STEP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}


}  // namespace emoe
