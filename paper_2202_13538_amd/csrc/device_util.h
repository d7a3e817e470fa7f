// Device-side helpers shared by the HIP kernels of libsurel (gfx950, wave64 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace surel {

constexpr int kWave = 64;

// Bits of the sticky device error word (same values as SUREL_DEV_* in the public header).
constexpr uint32_t kDevBadSeed = 0x01u;
constexpr uint32_t kDevBadGraph = 0x02u;
constexpr uint32_t kDevBadWalk = 0x04u;
constexpr uint32_t kDevBadQuery = 0x08u;
constexpr uint32_t kDevSetTooLarge = 0x10u;
constexpr uint32_t kDevCapacity = 0x20u;
constexpr uint32_t kDevBadTable = 0x40u;
constexpr uint32_t kDevBadSizes = 0x80u;
constexpr uint32_t kDevStall = 0x100u;

__device__ __forceinline__ int lane_id() {
    return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Orders LDS traffic between the lanes of ONE wavefront.  LDS instructions of a wave execute
// in issue order, so no hardware barrier is needed; the fence keeps the compiler from moving
// LDS accesses across this point.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Raise bits of the error word: one atomic per wave at most, none in the common case.
__device__ __forceinline__ void raise_error(uint32_t* err, bool cond, uint32_t bit) {
    if (__ballot(cond) != 0ull) {
        if (lane_id() == 0) atomicOr(err, bit);
    }
}

// Value of `x` held by lane (lane ^ MASK), MASK a compile-time constant in 1..63.  Uses the
// cheapest exchange the pattern allows: DPP quad permutes and row mirrors (folded into the
// consuming VALU instruction), the LDS crossbar's swizzle for other masks below 32, and a
// general ds_bpermute otherwise.  None of them touches LDS memory.
template <int MASK>
__device__ __forceinline__ uint32_t lane_xor(uint32_t x, int lane) {
    static_assert(MASK >= 1 && MASK < kWave, "mask out of range");
    if constexpr (MASK == 1) {
        return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, false);  // quad_perm [1,0,3,2]
    } else if constexpr (MASK == 2) {
        return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, false);  // quad_perm [2,3,0,1]
    } else if constexpr (MASK == 3) {
        return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x1B, 0xF, 0xF, false);  // quad_perm [3,2,1,0]
    } else if constexpr (MASK == 7) {
        return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xF, 0xF, false);  // row_half_mirror
    } else if constexpr (MASK == 15) {
        return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x140, 0xF, 0xF, false);  // row_mirror
    } else if constexpr (MASK < 32) {
        // swizzle, bit mode: new lane = ((lane & and) | or) ^ xor inside each group of 32
        return (uint32_t)__builtin_amdgcn_ds_swizzle((int)x, (MASK << 10) | 0x1F);
    } else {
        return (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ MASK) << 2, (int)x);
    }
}

__device__ __forceinline__ uint32_t wave_bcast_u32(uint32_t v, int src_lane) {
    return (uint32_t)__shfl((int)v, src_lane, kWave);
}

// Inclusive prefix sum over the 64 lanes.
__device__ __forceinline__ uint32_t wave_incl_sum(uint32_t v) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t t = (uint32_t)__shfl_up((int)v, d, kWave);
        if (lane >= d) v += t;
    }
    return v;
}

// Inclusive prefix maximum (signed) over the 64 lanes.
__device__ __forceinline__ int32_t wave_incl_max(int32_t v) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int32_t t = __shfl_up(v, d, kWave);
        if (lane >= d) v = max(v, t);
    }
    return v;
}

// Copies n 32-bit words from global memory to LDS with the whole wave.  Loads are issued U
// at a time before any of them is waited for, so a copy costs ceil(n / (64*U)) memory round
// trips instead of one per 64 words.
template <int U>
__device__ __forceinline__ void stage_words(uint32_t* dst, const uint32_t* __restrict__ src, int n,
                                            int lane) {
    for (int t0 = 0; t0 < n; t0 += kWave * U) {
        uint32_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * kWave + lane;
            v[u] = t < n ? src[t] : 0u;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * kWave + lane;
            if (t < n) dst[t] = v[u];
        }
    }
}

// Philox-4x32 with 10 rounds (Salmon et al., SC'11): counter c[0..3], key (k0, k1).
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0);
        const uint32_t lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2);
        const uint32_t lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0;
        c1 = lo1;
        c2 = n2;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}

// floor(x / d) for 0 <= x < 4096 and 1 <= d <= 16 with magic = 65536 / d + 1.
// Exact because x * (magic * d - 65536) <= x * d < 65536.
__device__ __forceinline__ uint32_t small_div(uint32_t x, uint32_t magic) {
    return (x * magic) >> 16;
}

// floor(x / d) for x * d < 2^32 with magic = 2^32 / d + 1 (d >= 2; the host passes it in).
__device__ __forceinline__ uint32_t div_magic32(uint32_t x, uint32_t magic) {
    return __umulhi(x, magic);
}

}  // namespace surel
