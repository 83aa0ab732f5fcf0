// Device helpers shared by the streaming kernels: vector loads of a matrix row's elements and index arithmetic.
#pragma once

#include "atk_common.h"

namespace atk {

#ifdef __HIPCC__

template <int ELT, int V>
struct RowVec {
    static constexpr int kBytes = V * ((ELT == ATK_F32) ? 4 : 2);
    static constexpr int kWords = (kBytes + 3) / 4;
    uint32_t w[kWords];
};

// One load of V adjacent elements (16, 8, 4 or 2 bytes).  The data is read exactly once,
// so the loads are marked non-temporal.
template <int ELT, int V>
__device__ __forceinline__ RowVec<ELT, V> load_vec(const unsigned char *p) {
    RowVec<ELT, V> r;
    constexpr int B = RowVec<ELT, V>::kBytes;
    if constexpr (B == 16) {
        typedef uint32_t v4u __attribute__((ext_vector_type(4)));
        v4u q = __builtin_nontemporal_load((const v4u *)p);
        r.w[0] = q.x;
        r.w[1] = q.y;
        r.w[2] = q.z;
        r.w[3] = q.w;
    } else if constexpr (B == 8) {
        typedef uint32_t v2u __attribute__((ext_vector_type(2)));
        v2u q = __builtin_nontemporal_load((const v2u *)p);
        r.w[0] = q.x;
        r.w[1] = q.y;
    } else if constexpr (B == 4) {
        r.w[0] = __builtin_nontemporal_load((const uint32_t *)p);
    } else {
        r.w[0] = (uint32_t)__builtin_nontemporal_load((const uint16_t *)p);
    }
    return r;
}

// element e of the vector as float bits (bf16 widened exactly)
template <int ELT, int V>
__device__ __forceinline__ uint32_t elem_bits(const RowVec<ELT, V> &r, int e) {
    if constexpr (ELT == ATK_F32) {
        return r.w[e];
    } else {
        uint32_t w = r.w[e >> 1];
        return (e & 1) ? (w & 0xffff0000u) : (w << 16);
    }
}

// q = x / d, rem = x % d; shift = log2(d) when d is a power of two, else -1
__device__ __forceinline__ void divmod(int x, int d, int shift, int &q, int &rem) {
    if (shift >= 0) {
        q = x >> shift;
        rem = x & (d - 1);
    } else {
        q = x / d;
        rem = x - q * d;
    }
}

#endif  // __HIPCC__

}  // namespace atk
