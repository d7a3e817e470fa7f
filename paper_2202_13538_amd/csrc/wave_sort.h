// Bitonic sort of 64*E 32-bit keys held in the registers of one wavefront (gfx950, wave64).
#pragma once

#include "device_util.h"

namespace surel {

// Compare-exchange with the lane `lane ^ MASK`: the lower lane of a pair keeps the smaller
// key.  `y < x` decides for a lower lane, its negation for an upper one (equal keys need
// no exchange, so either answer is right for them).
template <int MASK>
__device__ __forceinline__ uint32_t exchange(uint32_t x, uint32_t y, bool upper) {
    const bool take = (y < x) != upper;
    return take ? y : x;
}

// Sorts the 64*E keys of a wave ascending.  Sort position p = lane*E + r (lane-blocked).
// Bitonic merge sort written with ascending comparators only: a merge of two sorted runs
// starts with a mirror step (p against p ^ (k-1)) and continues with half-cleaners
// (p against p ^ j, j = k/4 .. 1).  Strides below E stay inside a lane (register to
// register); the others exchange registers between lanes.
template <int E, int K>
__device__ __forceinline__ void sort_merge_level(uint32_t (&x)[E], int lane) {
    if constexpr (K <= E) {
#pragma unroll
        for (int r = 0; r < E; ++r) {
            const int q = r ^ (K - 1);
            if (q > r) {
                const uint32_t a = min(x[r], x[q]);
                const uint32_t b = max(x[r], x[q]);
                x[r] = a;
                x[q] = b;
            }
        }
    } else {
        constexpr int kLaneMask = K / E - 1;
        const bool upper = (lane & (K / (2 * E))) != 0;
        uint32_t y[E];
#pragma unroll
        for (int r = 0; r < E; ++r) y[r] = lane_xor<kLaneMask>(x[E - 1 - r], lane);
#pragma unroll
        for (int r = 0; r < E; ++r) x[r] = exchange<kLaneMask>(x[r], y[r], upper);
    }
}

template <int E, int J>
__device__ __forceinline__ void sort_half_cleaner(uint32_t (&x)[E], int lane) {
    if constexpr (J >= 1) {
        if constexpr (J < E) {
#pragma unroll
            for (int r = 0; r < E; ++r) {
                if ((r & J) == 0) {
                    const uint32_t a = min(x[r], x[r | J]);
                    const uint32_t b = max(x[r], x[r | J]);
                    x[r] = a;
                    x[r | J] = b;
                }
            }
        } else {
            constexpr int kLaneMask = J / E;
            const bool upper = (lane & kLaneMask) != 0;
#pragma unroll
            for (int r = 0; r < E; ++r) {
                const uint32_t y = lane_xor<kLaneMask>(x[r], lane);
                x[r] = exchange<kLaneMask>(x[r], y, upper);
            }
        }
        sort_half_cleaner<E, J / 2>(x, lane);
    }
}

template <int E, int K>
__device__ __forceinline__ void sort_levels(uint32_t (&x)[E], int lane) {
    if constexpr (K <= kWave * E) {
        sort_merge_level<E, K>(x, lane);
        sort_half_cleaner<E, K / 4>(x, lane);
        sort_levels<E, K * 2>(x, lane);
    }
}

template <int E>
__device__ __forceinline__ void wave_sort(uint32_t (&x)[E], int lane) {
    sort_levels<E, 2>(x, lane);
}

}  // namespace surel
