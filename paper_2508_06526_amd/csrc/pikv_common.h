// Internal helpers shared by the gfx950 kernels of libpikv (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "pikv.h"

namespace pikv {

constexpr int kWave = 64;

// Storage element tags.  bfloat16 is handled as its 16-bit pattern: widening to fp32 is a
// shift, and the kernels never round back to bf16.
struct bf16 {
    uint16_t bits;
};

template <typename T>
struct Pack16;  // how many elements one 16-byte lane load carries, and how to widen them

template <>
struct Pack16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void widen(const uint4 &r, float *f) {
        f[0] = __uint_as_float(r.x);
        f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z);
        f[3] = __uint_as_float(r.w);
    }
};

template <>
struct Pack16<bf16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void widen(const uint4 &r, float *f) {
        f[0] = __uint_as_float(r.x << 16);
        f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16);
        f[3] = __uint_as_float(r.y & 0xffff0000u);
        f[4] = __uint_as_float(r.z << 16);
        f[5] = __uint_as_float(r.z & 0xffff0000u);
        f[6] = __uint_as_float(r.w << 16);
        f[7] = __uint_as_float(r.w & 0xffff0000u);
    }
};

template <typename T>
__device__ __forceinline__ float load_scalar(const T *p, int64_t i);
template <>
__device__ __forceinline__ float load_scalar<float>(const float *p, int64_t i) {
    return p[i];
}
template <>
__device__ __forceinline__ float load_scalar<bf16>(const bf16 *p, int64_t i) {
    return __uint_as_float(static_cast<uint32_t>(p[i].bits) << 16);
}

// Exchange across one lane-index bit of the wavefront.  Bits 0..3 stay inside a DPP row of
// 16 lanes (no LDS traffic); bits 2 and 3 use the mirror patterns, which pair lane i with
// the lane whose lower bits are complemented as well - callers only use them on values
// that are already uniform across the lower bits (a bottom-up butterfly guarantees it).
template <int BIT>
__device__ __forceinline__ float lane_xchg(float x) {
    static_assert(BIT >= 0 && BIT < 6, "wave64");
    if constexpr (BIT == 0) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, true));
    } else if constexpr (BIT == 1) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, true));
    } else if constexpr (BIT == 2) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, true));
    } else if constexpr (BIT == 3) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xf, 0xf, true));
    } else {
        return __shfl_xor(x, 1 << BIT, kWave);
    }
}

// Exact exchange: lane i receives the value of lane i ^ (1 << BIT), whatever the lanes hold.
// Inside a row of 16 lanes two DPP moves compose the xor patterns the hardware lacks: the half
// mirror (i -> i ^ 7) followed by the reversed quad (i -> i ^ 3) is i ^ 4; the row mirror
// (i -> i ^ 15) followed by the half mirror is i ^ 8.
template <int BIT>
__device__ __forceinline__ float lane_xor(float x) {
    static_assert(BIT >= 0 && BIT < 6, "wave64");
    auto dpp = [](float v, auto ctrl) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xf, 0xf, true));
    };
    if constexpr (BIT == 0) {
        return dpp(x, std::integral_constant<int, 0xB1>{});
    } else if constexpr (BIT == 1) {
        return dpp(x, std::integral_constant<int, 0x4E>{});
    } else if constexpr (BIT == 2) {
        return dpp(dpp(x, std::integral_constant<int, 0x141>{}), std::integral_constant<int, 0x1B>{});
    } else if constexpr (BIT == 3) {
        return dpp(dpp(x, std::integral_constant<int, 0x140>{}), std::integral_constant<int, 0x141>{});
    } else {
        return __shfl_xor(x, 1 << BIT, kWave);
    }
}

// Sum / max over the lane bits [LO, HI): every participating lane ends with the result.
template <int LO, int HI>
__device__ __forceinline__ float bits_sum(float x) {
    if constexpr (LO < HI) {
        x += lane_xchg<LO>(x);
        return bits_sum<LO + 1, HI>(x);
    } else {
        return x;
    }
}
template <int LO, int HI>
__device__ __forceinline__ float bits_max(float x) {
    if constexpr (LO < HI) {
        x = fmaxf(x, lane_xchg<LO>(x));
        return bits_max<LO + 1, HI>(x);
    } else {
        return x;
    }
}

constexpr __host__ __device__ int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v >> 1); }

__device__ __forceinline__ uint4 load16(const void *p) {
    return *reinterpret_cast<const uint4 *>(p);
}

// 16-byte load of data that is read exactly once (the K/V stream): the non-temporal hint
// keeps it from displacing reusable lines in L2 / Infinity Cache.
// The pointer is known to be device (global) memory, which lets the compiler emit
// global_load instead of a flat load.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef const u32x4_t __attribute__((address_space(1))) *global_u32x4_ptr;
__device__ __forceinline__ uint4 load16_stream(const void *p) {
    const u32x4_t v = __builtin_nontemporal_load((global_u32x4_ptr)(uintptr_t)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
// 16-byte store of data nobody reads back soon (written once, consumed by a later kernel):
// the non-temporal hint sends it on its way instead of parking a dirty line in L2.
typedef u32x4_t __attribute__((address_space(1))) *global_u32x4_wptr;
__device__ __forceinline__ void store16_stream(void *p, uint4 v) {
    const u32x4_t x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, (global_u32x4_wptr)(uintptr_t)p);
}

// fp32 -> uint32 whose unsigned order is the float order (-0 folded onto +0).
__device__ __forceinline__ uint32_t order_key(float u) {
    uint32_t bits = __float_as_uint(u);
    if (bits == 0x80000000u) bits = 0u;
    return (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
}

// Eviction order in one integer: smaller composite = lower utility, then HIGHER slot (among
// equal utilities the lower slot is the one that is kept).
__device__ __forceinline__ uint64_t evict_composite(float u, int slot) {
    return ((uint64_t)order_key(u) << 32) | (uint32_t)(0x7fffffff - slot);
}
__device__ __forceinline__ int evict_composite_slot(uint64_t c) {
    return 0x7fffffff - (int)(uint32_t)(c & 0xffffffffu);
}

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline int launch_status() { return hipGetLastError() == hipSuccess ? PIKV_OK : PIKV_ERR_HIP; }

// Host-side descriptor checks common to every call that takes a pikv_desc.
int check_desc(const pikv_desc *d);
inline int desc_width(const pikv_desc *d) { return d->rank ? d->rank : d->D; }
inline int elem_bytes(int dtype) { return dtype == PIKV_F32 ? 4 : 2; }

// Split geometry of the attention pass (also defines the workspace size).
struct AttnPlan {
    bool gqa_mfma;        // matrix-core grouped-query kernel (bf16, D = 128, 2..64 query rows per kv head)
    int heads_per_block;  // query heads sharing one K/V stream
    int row_tiles;        // matrix-core kernel: 16-row tiles the query group occupies (1, 2 or 4)
    int head_blocks;      // Hq / heads_per_block
    int tile_rows;        // rows one wave consumes per iteration
    int chunk;            // rows per split (multiple of tile_rows)
    int nsplit;
    int resident_blocks;  // blocks of the split pass the GPU holds at once
    size_t score_stage_bytes;  // LDS per block for the raw scores (0: written straight to memory)
    size_t acc_floats;    // B*Hq*k*nsplit*width
    size_t ml_floats;     // B*Hq*k*nsplit*2
};
int make_attn_plan(const pikv_desc *d, int k, AttnPlan *plan);
void g_split_override_set(int v);
void g_profile_events_set(void *start, void *stop);

}  // namespace pikv
