// Workgroup-level exact selection in LDS: radix select on composite words, then an
// ordered write-out.  This is Stage 2 of the method (Section 2: "if b*k_b > k, use an
// exact top-k to select the k largest values") and the body of the small-row exact_topk.
// The radix descent follows the RadixSelect scheme of Appendix D.2 (most significant
// digit first, keep the digit bucket that contains the k-th element), with 8-bit digits
// and an LDS histogram; because composites are distinct the descent ends as soon as the
// chosen digit bucket holds exactly the number of elements still needed.
#pragma once

#include "atk_common.h"

namespace atk {

#ifdef __HIPCC__

constexpr int kHistWords = 256 + 8;  // 256 bins + [256]=digit, [257]=need, [258]=bucket count, [259]=write cursor

__device__ __forceinline__ int pow2_ceil_dev(int v) {
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

// Decode a composite and store it as output element `pos` (absolute element offset).
template <int ELT>
__device__ __forceinline__ void write_composite(u64 c, void *out_vals, int32_t *out_idx, int64_t pos) {
    store_val<ELT>(out_vals, pos, composite_bits(c));
    out_idx[pos] = composite_index(c);
}

template <int ELT>
__device__ void select_sort_write(u64 *cand, int count, int k, u64 *sel, uint32_t *hist, void *out_vals,
                                  int32_t *out_idx, int64_t row_out) {
    const int tid = threadIdx.x, T = blockDim.x;

    // ---- radix descent: find thr such that exactly k composites are >= thr
    u64 prefix = 0;
    int need = k;
    int shift = 56;
    while (true) {
        for (int i = tid; i < kHistWords; i += T) hist[i] = 0;
        __syncthreads();
        const u64 hi_mask = (shift == 56) ? 0ull : (~0ull << (shift + 8));
        for (int i = tid; i < count; i += T) {
            u64 c = cand[i];
            if ((c & hi_mask) == prefix) atomicAdd(&hist[(uint32_t)(c >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < kWave) {
            // lane l owns bins 4l..4l+3; suffix sums from the top bin down
            uint32_t h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3];
            uint32_t lane_sum = h0 + h1 + h2 + h3;
            uint32_t incl = lane_sum;  // sum over lanes >= tid
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                uint32_t other = __shfl_down(incl, off, kWave);
                if (tid + off < kWave) incl += other;
            }
            uint32_t above = incl - lane_sum;  // elements in bins of higher lanes
            // walk own bins from high to low
            uint32_t hb[4] = {h0, h1, h2, h3};
#pragma unroll
            for (int q = 3; q >= 0; --q) {
                uint32_t with = above + hb[q];
                if (above < (uint32_t)need && with >= (uint32_t)need) {
                    hist[256] = 4 * tid + q;
                    hist[257] = (uint32_t)need - above;
                    hist[258] = hb[q];
                }
                above = with;
            }
        }
        __syncthreads();
        const uint32_t digit = hist[256];
        const int bucket_count = (int)hist[258];
        need = (int)hist[257];
        prefix |= (u64)digit << shift;
        __syncthreads();  // everyone has read hist before it is cleared again
        if (bucket_count == need || shift == 0) break;
        shift -= 8;
    }
    // every composite whose bits above `shift` are >= prefix is selected
    const u64 thr = prefix;

    // ---- compaction (arbitrary order)
    if (tid == 0) hist[259] = 0;
    __syncthreads();
    for (int i = tid; i < count; i += T) {
        u64 c = cand[i];
        if (c >= thr) {
            uint32_t pos = atomicAdd(&hist[259], 1u);
            sel[pos] = c;
        }
    }
    __syncthreads();

    // ---- order the k survivors, largest first
    if (k <= 256) {
        // rank sort: position = number of larger survivors
        for (int i = tid; i < k; i += T) {
            u64 c = sel[i];
            int rank = 0;
            for (int j = 0; j < k; ++j) rank += (sel[j] > c) ? 1 : 0;
            write_composite<ELT>(c, out_vals, out_idx, row_out * k + rank);
        }
    } else {
        const int kp = pow2_ceil_dev(k);
        for (int i = k + tid; i < kp; i += T) sel[i] = 0;  // empties sort to the end
        __syncthreads();
        for (int size = 2; size <= kp; size <<= 1) {
            for (int stride = size >> 1; stride >= 1; stride >>= 1) {
                for (int i = tid; i < (kp >> 1); i += T) {
                    int lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));
                    int hi = lo + stride;
                    bool desc = (lo & size) == 0;
                    u64 a = sel[lo], c = sel[hi];
                    bool sw = desc ? (c > a) : (c < a);
                    if (sw) {
                        sel[lo] = c;
                        sel[hi] = a;
                    }
                }
                __syncthreads();
            }
        }
        for (int i = tid; i < k; i += T) write_composite<ELT>(sel[i], out_vals, out_idx, row_out * k + i);
    }
}

#endif  // __HIPCC__

}  // namespace atk
