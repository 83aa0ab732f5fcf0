// Workgroup-level exact selection in LDS: radix select on composite words, then an
// ordered write-out.  This is Stage 2 of the method (Section 2: "if b*k_b > k, use an
// exact top-k to select the k largest values") and the body of the small-row exact_topk.
// The radix descent follows the RadixSelect scheme of Appendix D.2 (most significant
// digit first, keep the digit bucket that contains the k-th element), with 8-bit digits
// and an LDS histogram.  Two departures: the descent starts at the highest bit in which
// the candidates differ at all (their common leading bits cannot separate anything), and,
// because composites are distinct, it stops as soon as the chosen digit bucket holds
// exactly the number of elements still needed.  When few candidates per lane remain and they
// spread well over their range, a single histogram pass plus exact in-bin ranking replaces
// the descent, the compaction and the ordering altogether (select_write).
#pragma once

#include "atk_common.h"

namespace atk {

#ifdef __HIPCC__

__host__ __device__ constexpr int pow2_ceil_c(int v) {
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}
__device__ __forceinline__ int pow2_ceil_dev(int v) { return pow2_ceil_c(v); }

// ---- LDS layout behind the `count` candidates -------------------------------------------------
constexpr int kRankMax = 256;                 // largest k ordered by all-pairs ranking (else bitonic sort)
constexpr int kSelWredWords = 32;             // u64: per-wavefront OR / AND
constexpr int kSelU32Words = 512 + 8 + 8 + kRankMax;  // two histograms, scan result, cursor, ranks
constexpr int kBkBins = 2048;                 // bucket-rank path: bins over the candidates' range
constexpr int kBkBinMax = 32;                 // fullest bin it accepts
constexpr int kBkSlots = 4;                   // candidates per lane it holds in registers
constexpr int kBkU32Words = kBkBins + (kBkBins + 8) + 32;  // counts, offsets (+sentinel), flag and wavefront totals
__host__ __device__ constexpr int64_t select_lds_bytes(int64_t count, int kp) {
    const int64_t radix = (int64_t)(kp + kSelWredWords) * 8 + kSelU32Words * 4;
    const int64_t bucket = 16 + (int64_t)kBkU32Words * 4;
    return count * 8 + (radix > bucket ? radix : bucket);
}

// Phase timestamps of the measurement build of the fused kernel (atk_trace_approx): lane 0 of every wavefront
// stores the 100 MHz wall clock into its own row of `tr`.  TR = false (every product launch) compiles to nothing.
constexpr int kTracePhases = 16;   // words per wavefront: 12 phase stamps, [12] HW_ID, [13] XCC_ID of the wavefront
constexpr int kTraceWaves = 16;    // wavefronts per workgroup the buffer has rows for
template <bool TR>
__device__ __forceinline__ void trace_mark(u64 *tr, int phase) {
    if constexpr (TR) {
        if ((threadIdx.x & (kWave - 1)) == 0) {
            u64 *row = tr + ((int64_t)blockIdx.x * kTraceWaves + (threadIdx.x >> 6)) * kTracePhases;
            row[phase] = wall_clock64();
            if (phase == 0) {  // where the wavefront runs: hardware registers HW_ID (4) and XCC_ID (20), all 32 bits
                row[12] = (u64)__builtin_amdgcn_s_getreg((31 << 11) | 4);
                row[13] = (u64)__builtin_amdgcn_s_getreg((31 << 11) | 20);
            }
        }
    }
}

// Decode a composite and store it as output element `pos` (absolute element offset).
template <int ELT>
__device__ __forceinline__ void write_composite(u64 c, void *out_vals, int32_t *out_idx, int64_t pos) {
    store_val<ELT>(out_vals, pos, composite_bits(c));
    out_idx[pos] = composite_index(c);
}

// Number of entries of list[j0..j1) that are larger than c; eight LDS reads in flight at a time.
__device__ __forceinline__ int count_larger(const u64 *list, int j0, int j1, u64 c) {
    int rank = 0;
    int j = j0;
    for (; j + 8 <= j1; j += 8) {
        u64 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = list[j + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) rank += (v[u] > c) ? 1 : 0;
    }
    for (; j < j1; ++j) rank += (list[j] > c) ? 1 : 0;
    return rank;
}

// ---- wavefront helpers (DPP: register-to-register, no LDS traffic) -----------------------------
// dpp_ctrl codes: quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E, row_shr:n = 0x110+n,
// row_mirror = 0x140, row_half_mirror = 0x141, row_bcast:15 = 0x142, row_bcast:31 = 0x143.
template <int CTRL>
__device__ __forceinline__ u64 dpp_u64(u64 v) {
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    lo = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, 0xf, 0xf, false);
    hi = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)hi, CTRL, 0xf, 0xf, false);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 readlane_u64(u64 v, int lane) {
    uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, lane);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
    return ((u64)hi << 32) | lo;
}
// OR and AND over the 64 lanes of a fully active wavefront (result in every lane).  The two
// quad permutations and the two mirrors fold a row of 16 lanes; the four rows are read out.
__device__ __forceinline__ void wave_or_and_u64(u64 &o, u64 &a) {
    o |= dpp_u64<0xB1>(o);
    a &= dpp_u64<0xB1>(a);
    o |= dpp_u64<0x4E>(o);
    a &= dpp_u64<0x4E>(a);
    o |= dpp_u64<0x141>(o);
    a &= dpp_u64<0x141>(a);
    o |= dpp_u64<0x140>(o);
    a &= dpp_u64<0x140>(a);
    o = readlane_u64(o, 0) | readlane_u64(o, 16) | readlane_u64(o, 32) | readlane_u64(o, 48);
    a = readlane_u64(a, 0) & readlane_u64(a, 16) & readlane_u64(a, 32) & readlane_u64(a, 48);
}
// Minimum and maximum over the 64 lanes of a fully active wavefront (result in every lane).
__device__ __forceinline__ void wave_min_max_u64(u64 &lo, u64 &hi) {
    u64 t;
    t = dpp_u64<0xB1>(lo);  lo = t < lo ? t : lo;
    t = dpp_u64<0xB1>(hi);  hi = t > hi ? t : hi;
    t = dpp_u64<0x4E>(lo);  lo = t < lo ? t : lo;
    t = dpp_u64<0x4E>(hi);  hi = t > hi ? t : hi;
    t = dpp_u64<0x141>(lo); lo = t < lo ? t : lo;
    t = dpp_u64<0x141>(hi); hi = t > hi ? t : hi;
    t = dpp_u64<0x140>(lo); lo = t < lo ? t : lo;
    t = dpp_u64<0x140>(hi); hi = t > hi ? t : hi;
    u64 a = readlane_u64(lo, 0), b = readlane_u64(lo, 16), c = readlane_u64(lo, 32), d = readlane_u64(lo, 48);
    a = a < b ? a : b;
    c = c < d ? c : d;
    lo = a < c ? a : c;
    a = readlane_u64(hi, 0), b = readlane_u64(hi, 16), c = readlane_u64(hi, 32), d = readlane_u64(hi, 48);
    a = a > b ? a : b;
    c = c > d ? c : d;
    hi = a > c ? a : c;
}

// Minimum / maximum of a 32-bit value over the 64 lanes of a fully active wavefront.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    v = min(v, dpp_u32<0xB1>(v));
    v = min(v, dpp_u32<0x4E>(v));
    v = min(v, dpp_u32<0x141>(v));
    v = min(v, dpp_u32<0x140>(v));
    const uint32_t a = min((uint32_t)__builtin_amdgcn_readlane((int)v, 0), (uint32_t)__builtin_amdgcn_readlane((int)v, 16));
    const uint32_t b = min((uint32_t)__builtin_amdgcn_readlane((int)v, 32), (uint32_t)__builtin_amdgcn_readlane((int)v, 48));
    return min(a, b);
}
__device__ __forceinline__ uint32_t wave_or_u32(uint32_t v) {
    v |= dpp_u32<0xB1>(v);
    v |= dpp_u32<0x4E>(v);
    v |= dpp_u32<0x141>(v);
    v |= dpp_u32<0x140>(v);
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) | (uint32_t)__builtin_amdgcn_readlane((int)v, 16) |
           (uint32_t)__builtin_amdgcn_readlane((int)v, 32) | (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = max(v, dpp_u32<0xB1>(v));
    v = max(v, dpp_u32<0x4E>(v));
    v = max(v, dpp_u32<0x141>(v));
    v = max(v, dpp_u32<0x140>(v));
    const uint32_t a = max((uint32_t)__builtin_amdgcn_readlane((int)v, 0), (uint32_t)__builtin_amdgcn_readlane((int)v, 16));
    const uint32_t b = max((uint32_t)__builtin_amdgcn_readlane((int)v, 32), (uint32_t)__builtin_amdgcn_readlane((int)v, 48));
    return max(a, b);
}

// Lanes without a source (row edge) or outside ROW_MASK receive 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_zero_fill(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, true);
}
// Inclusive prefix sum over the lanes of a fully active wavefront.
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
    v += dpp_zero_fill<0x111, 0xf>(v);  // row_shr:1
    v += dpp_zero_fill<0x112, 0xf>(v);  // row_shr:2
    v += dpp_zero_fill<0x114, 0xf>(v);  // row_shr:4
    v += dpp_zero_fill<0x118, 0xf>(v);  // row_shr:8  -> inclusive scan inside each row of 16
    v += dpp_zero_fill<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
    v += dpp_zero_fill<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
    return v;
}

// Writes the k distinct composites sel[0..k) (LDS, any order) to row `row_out`, largest first.
// sel has room for pow2_ceil(k) words; rk: LDS, kRankMax zeroed words (used when k <= kRankMax).
// All threads of the workgroup call it, after a barrier that made sel (and the zeroed rk) visible.
template <int ELT>
__device__ __forceinline__ void order_write(u64 *sel, int k, uint32_t *rk, void *out_vals, int32_t *out_idx, int64_t row_out) {
    const int tid = threadIdx.x, T = blockDim.x;
    const int kp = pow2_ceil_dev(k);
    if (k <= kRankMax) {
        // rank = number of larger survivors; iw lanes side by side take one survivor each and
        // the T/iw groups of lanes split the range of partners
        int iw = kWave, iw_shift = 6;
        while (iw < k && iw * 2 <= T) {  // iw divides into T, also when T is not a power of two
            iw <<= 1;
            ++iw_shift;
        }
        const int parts = T >> iw_shift;
        if (parts == 1) {
            for (int i = tid; i < k; i += iw)
                write_composite<ELT>(sel[i], out_vals, out_idx, row_out * k + count_larger(sel, 0, k, sel[i]));
            return;
        }
        const int chunk = (k + parts - 1) / parts;
        const int part = tid >> iw_shift;
        const int j0 = part * chunk, j1 = min(k, j0 + chunk);
        const int i = tid & (iw - 1);
        if (i < k && j0 < j1) {
            const int r = count_larger(sel, j0, j1, sel[i]);
            if (r) atomicAdd(&rk[i], (uint32_t)r);
        }
        __syncthreads();
        for (int q = tid; q < k; q += T) write_composite<ELT>(sel[q], out_vals, out_idx, row_out * k + (int)rk[q]);
    } else {
        for (int i = k + tid; i < kp; i += T) sel[i] = 0;  // empties sort to the end
        __syncthreads();
        for (int size = 2; size <= kp; size <<= 1) {
            for (int stride = size >> 1; stride >= 1; stride >>= 1) {
                for (int i = tid; i < (kp >> 1); i += T) {
                    const int lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));
                    const int hi = lo + stride;
                    const bool desc = (lo & size) == 0;
                    const u64 a = sel[lo], c = sel[hi];
                    const bool sw = desc ? (c > a) : (c < a);
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


// Radix-descent selection: exact top-k of the `count` distinct composites at cand[0..count)
// (LDS), written largest first to row `row_out`.  Needs (pow2_ceil(k) + kSelWredWords) * 8 +
// kSelU32Words * 4 bytes of LDS behind cand.
template <int ELT>
__device__ __forceinline__ void select_radix_write(u64 *cand, int count, int k, void *out_vals, int32_t *out_idx, int64_t row_out) {
    const int tid = threadIdx.x, T = blockDim.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6, n_waves = T >> 6;
    const int kp = pow2_ceil_dev(k);
    u64 *sel = cand + count;                              // [kp]
    u64 *wred = sel + kp;                                 // [32]
    uint32_t *hist = (uint32_t *)(wred + kSelWredWords);  // [2][256]
    uint32_t *res = hist + 512;                           // [0]=digit [1]=need [2]=bucket count
    uint32_t *cursor = res + 8;                           // [0]
    uint32_t *rk = cursor + 8;                            // [kRankMax]

    // ---- common leading bits
    for (int i = tid; i < kSelU32Words; i += T) hist[i] = 0;
    u64 x_or = 0ull, x_and = ~0ull;
    for (int i = tid; i < count; i += T) {
        const u64 c = cand[i];
        x_or |= c;
        x_and &= c;
    }
    wave_or_and_u64(x_or, x_and);
    if (lane == 0) {
        wred[2 * wave] = x_or;
        wred[2 * wave + 1] = x_and;
    }
    __syncthreads();
    for (int w = 0; w < n_waves; ++w) {
        x_or |= wred[2 * w];
        x_and &= wred[2 * w + 1];
    }
    const u64 diff = x_or ^ x_and;
    const int top = diff ? 63 - __clzll((long long)diff) : 0;
    // the digit of a pass is bits [shift + width - 1 : shift]; bits above it are decided (prefix)
    int shift = top > 7 ? top - 7 : 0;
    uint32_t dmask = (1u << (top - shift + 1)) - 1u;
    u64 hi_mask = (top >= 63) ? 0ull : (~0ull << (top + 1));
    u64 prefix = x_and & hi_mask;
    int need = k;

    // ---- radix descent: find prefix such that exactly k composites are >= prefix
    int pb = 0;
    while (true) {
        uint32_t *h = hist + 256 * pb;
        for (int i = tid; i < count; i += T) {
            const u64 c = cand[i];
            if ((c & hi_mask) == prefix) atomicAdd(&h[(uint32_t)(c >> shift) & dmask], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns the four bins 252-4l .. 255-4l, so lane order is descending bin order
            const uint32_t *hl = &h[252 - 4 * lane];
            const uint32_t b4[4] = {hl[0], hl[1], hl[2], hl[3]};
            const uint32_t lane_sum = b4[0] + b4[1] + b4[2] + b4[3];
            uint32_t above = wave_incl_scan_u32(lane_sum) - lane_sum;  // elements in higher bins
#pragma unroll
            for (int q = 3; q >= 0; --q) {
                const uint32_t with = above + b4[q];
                if (above < (uint32_t)need && with >= (uint32_t)need) {
                    res[0] = 252 - 4 * lane + q;
                    res[1] = (uint32_t)need - above;
                    res[2] = b4[q];
                }
                above = with;
            }
        }
        // the other histogram is cleared for the next pass while wavefront 0 scans
        if (n_waves > 1) {
            if (wave >= 1)
                for (int i = tid - kWave; i < 256; i += T - kWave) hist[256 * (pb ^ 1) + i] = 0;
        } else {
            for (int i = tid; i < 256; i += T) hist[256 * (pb ^ 1) + i] = 0;
        }
        __syncthreads();
        const uint32_t digit = res[0];
        const int bucket_count = (int)res[2];
        need = (int)res[1];
        prefix |= (u64)digit << shift;
        if (bucket_count == need || shift == 0) break;
        const int next = shift >= 8 ? shift - 8 : 0;  // the last digit may be narrower than 8 bits
        hi_mask = ~0ull << shift;
        dmask = (1u << (shift - next)) - 1u;
        shift = next;
        pb ^= 1;
    }
    // every composite >= prefix is selected (bits below `shift` of prefix are zero)
    const u64 thr = prefix;

    // ---- compaction into sel[0..k): one LDS atomic per wavefront and round
    for (int i0 = 0; i0 < count; i0 += T) {
        const int i = i0 + tid;
        const u64 c = (i < count) ? cand[i] : 0ull;
        const bool keep = (i < count) && (c >= thr);
        const u64 mask = __ballot(keep);
        const int n_keep = __popcll(mask);
        uint32_t base = 0;
        if (lane == 0 && n_keep) base = atomicAdd(&cursor[0], (uint32_t)n_keep);
        base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
        const uint32_t pos =
            base + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        if (keep) sel[pos] = c;
    }
    __syncthreads();

    order_write<ELT>(sel, k, rk, out_vals, out_idx, row_out);
}

// Exact top-k of the `count` distinct composites at cand[0..count) (LDS), written largest
// first to row `row_out` (row stride k).  `cand` must be followed by
// select_lds_bytes(count, pow2_ceil(k)) - count*8 bytes of free LDS.  All threads of the
// workgroup call it, after a barrier that made cand visible; blockDim.x is a multiple of 64.
//
// Fast path ("bucket rank", at most kBkSlots candidates per lane): the candidates move into
// registers; one histogram over 2048 bins that are linear in (composite - minimum); a
// descending prefix sum over the bins; then every candidate that can still be among the k
// largest is filed into its bin's segment (in place of cand) and finds its exact rank as
// (elements in higher bins) + (larger elements of its own bin), which is its output slot.
// No digit-by-digit descent, no compaction, no separate ordering.  If some bin is too full
// for the in-bin count to stay cheap (heavy ties, values clustered far below the maximum)
// the radix descent takes over.
//
// idx_bits: the candidates' column indices are below 2^idx_bits (1..31); it tells which index
// bits vary, so that equal values can be spread over bins by index.
template <int ELT, int NS, bool TR>
__device__ __forceinline__ void select_bucket_rank(u64 *cand, int count, int k, int idx_bits, void *out_vals,
                                                   int32_t *out_idx, int64_t row_out, u64 *tr);

template <int ELT, bool TR = false>
__device__ __forceinline__ void select_write(u64 *cand, int count, int k, int idx_bits, void *out_vals, int32_t *out_idx,
                             int64_t row_out, u64 *tr = nullptr) {
    const int T = blockDim.x;
    if (count > kBkSlots * T || T > kBkBins) {
        select_radix_write<ELT>(cand, count, k, out_vals, out_idx, row_out);
        return;
    }
    // the tail is a chain of dependent instructions in one workgroup: code for as many register
    // slots as the candidates need, not for the maximum
    if (count <= T)
        select_bucket_rank<ELT, 1, TR>(cand, count, k, idx_bits, out_vals, out_idx, row_out, tr);
    else if (count <= 2 * T)
        select_bucket_rank<ELT, 2, TR>(cand, count, k, idx_bits, out_vals, out_idx, row_out, tr);
    else
        select_bucket_rank<ELT, kBkSlots, TR>(cand, count, k, idx_bits, out_vals, out_idx, row_out, tr);
}

// The fast path of select_write with NS candidates per lane in registers (count <= NS * blockDim.x).
template <int ELT, int NS, bool TR>
__device__ __forceinline__ void select_bucket_rank(u64 *cand, int count, int k, int idx_bits, void *out_vals,
                                                   int32_t *out_idx, int64_t row_out, u64 *tr) {
    const int tid = threadIdx.x, T = blockDim.x;
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    // as many bins as it takes for about one candidate in four bins, 256 at least: clearing and
    // scanning them is serial work per lane, which a small workgroup with few candidates cannot afford
    int lg_bins = 8;
    while ((1 << lg_bins) < kBkBins && (1 << lg_bins) < 4 * count) ++lg_bins;
    if ((1 << lg_bins) < T) lg_bins = 31 - __builtin_clz(T) + (((T & (T - 1)) != 0) ? 1 : 0);  // a bin per lane at least
    if (lg_bins > 11) lg_bins = 11;
    const int n_bins = 1 << lg_bins;
    const int lane = tid & (kWave - 1), n_waves = T >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // LDS behind the candidates (16-byte aligned pieces): counts, "above" table, small words
    // (cand is 16-byte aligned; plain pointer arithmetic, so that the compiler still knows this is LDS)
    uint32_t *cnt = (uint32_t *)(cand + ((count + 1) & ~1));  // [2048], 16-byte aligned
    uint32_t *abv = cnt + kBkBins;   // abv[b + 4] = elements in bins above b, for b = -1 .. 2047
    uint32_t *misc = abv + kBkBins + 8;  // [0] overflow flag, [1] min key, [2] max key, [3] OR of keys, [8..24) wavefront totals

    // ---- candidates into registers (0 = none); clear the counts
    u64 c[NS];
    uint32_t k_min = 0xffffffffu, k_max = 0u, k_or = 0u;
#pragma unroll
    for (int e = 0; e < NS; ++e) {
        const int i = tid + e * T;
        c[e] = (i < count) ? cand[i] : 0ull;
    }
    {
        const v4u zero = {0u, 0u, 0u, 0u};
        for (int i = tid; i < n_bins / 4; i += T) ((v4u *)cnt)[i] = zero;
        if (tid == 0) {
            misc[0] = 0u;
            misc[1] = 0xffffffffu;
            misc[2] = 0u;
            misc[3] = 0u;
        }
    }
#pragma unroll
    for (int e = 0; e < NS; ++e)
        if (c[e]) {
            const uint32_t key = (uint32_t)(c[e] >> 32);
            k_min = key < k_min ? key : k_min;
            k_max = key > k_max ? key : k_max;
            k_or |= key;
        }
    // The lower end of the bins need not be the smallest candidate: any value that k candidates reach will do, and
    // what lies below it is out of the running.  Such a value comes for free: split the candidates into k or more
    // groups (the lanes' own candidates, those of 2, 4, 8, 16 or 64 lanes side by side - as large as still leaves k
    // groups); every group's maximum is a candidate, so the smallest of these maxima is reached by k candidates.  With
    // k far below the count this drops most candidates before the histogram; with k close to the count it still drops
    // the stragglers (small or negative values, whose keys lie far below the rest and would stretch the bins' range
    // until the winners crowd into a few of them).
    {
        const int lanes_with = count < T ? count : T;  // lanes that hold a candidate: 0 .. lanes_with - 1
        int g = 0;
        if (lanes_with >= k) {
            g = 1;
            if (lanes_with / 2 >= k) g = 2;
            if (lanes_with / 4 >= k) g = 4;
            if (lanes_with / 8 >= k) g = 8;
            if (lanes_with / 16 >= k) g = 16;
            if (lanes_with / 64 >= k) g = 64;
        }
        if (g) {
            uint32_t gm = k_max;  // (0 in a lane without candidates)
            if (g >= 2) gm = max(gm, dpp_u32<0xB1>(gm));
            if (g >= 4) gm = max(gm, dpp_u32<0x4E>(gm));
            if (g >= 8) gm = max(gm, dpp_u32<0x141>(gm));
            if (g >= 16) gm = max(gm, dpp_u32<0x140>(gm));
            if (g >= 64) gm = wave_max_u32(gm);
            k_min = gm ? gm : 0xffffffffu;  // (a group without candidates does not count: full groups alone are k)
        }
    }
    __syncthreads();
    // ---- range of the value keys: fold inside the wavefront, one set of LDS atomics per wavefront
    k_min = wave_min_u32(k_min);
    k_max = wave_max_u32(k_max);
    k_or = wave_or_u32(k_or);
    if (lane == 0) {
        atomicMin(&misc[1], k_min);
        atomicMax(&misc[2], k_max);
        atomicOr(&misc[3], k_or);
    }
    __syncthreads();
    trace_mark<TR>(tr, 4);  // key range known
    k_min = misc[1];
    k_max = misc[2];
    k_or = misc[3];
    // Bin key: the value key relative to the minimum, with the low bits that are zero in every
    // key squeezed out (bf16 values widened to f32 have 16 of them), followed by the varying
    // index bits; n_bins bins, linear over that range.  Equal values thus spread over bins by
    // index when the values alone do not fill the bins.
    const int tz = k_or ? __builtin_ctz(k_or) : 0;
    const uint32_t imask = (idx_bits >= 31) ? 0x7fffffffu : ((1u << idx_bits) - 1u);
    const u64 span = ((u64)((k_max - k_min) >> tz) + 1ull) << idx_bits;  // bin keys are below span
    const int rbits = 64 - __clzll((long long)span);
    const int bshift = rbits > lg_bins ? rbits - lg_bins : 0;
    uint32_t bin[NS];
    bool live[NS];  // a candidate, and not below the lower end
#pragma unroll
    for (int e = 0; e < NS; ++e) {
        const uint32_t key = (uint32_t)(c[e] >> 32);
        live[e] = c[e] != 0ull && key >= k_min;
        const u64 bk = ((u64)((key - k_min) >> tz) << idx_bits) | (((uint32_t)c[e] >> 1) & imask);
        bin[e] = live[e] ? (uint32_t)(bk >> bshift) : 0u;
        if (live[e]) atomicAdd(&cnt[bin[e]], 1u);
    }
    __syncthreads();
    trace_mark<TR>(tr, 5);  // histogram done

    // ---- descending exclusive prefix over the bins: thread t owns the q bins below 2048 - t*q
    const int q = n_bins / T;  // T is a multiple of 64 and at most n_bins; q*T may fall short of n_bins
    {
        // general q: walk the own bins from the top; q is 2, 4, 8 ... for the usual workgroup sizes
        const int hi = n_bins - 1 - tid * q;
        uint32_t s = 0;
        for (int j = 0; j < q; ++j) s += cnt[hi - j];
        // bins not covered because 2048 is not a multiple of T go to the last thread
        if (tid == T - 1)
            for (int bb = hi - q; bb >= 0; --bb) s += cnt[bb];
        const uint32_t incl = wave_incl_scan_u32(s);
        if (lane == kWave - 1) misc[8 + wave] = incl;
        __syncthreads();
        const uint32_t tot = (lane < n_waves) ? misc[8 + lane] : 0u;
        const uint32_t tot_incl = wave_incl_scan_u32(tot);
        uint32_t run = incl - s;
        if (wave > 0) run += (uint32_t)__builtin_amdgcn_readlane((int)tot_incl, wave - 1);
        bool crowded = false;  // a bin that may hold winners and is too full for the in-bin count to stay cheap
        for (int j = 0; j < q; ++j) {
            const uint32_t v = cnt[hi - j];
            abv[hi - j + 4] = run;
            crowded = crowded || (run < (uint32_t)k && v > (uint32_t)kBkBinMax);
            run += v;
        }
        if (tid == T - 1) {
            for (int bb = hi - q; bb >= 0; --bb) {
                const uint32_t v = cnt[bb];
                abv[bb + 4] = run;
                crowded = crowded || (run < (uint32_t)k && v > (uint32_t)kBkBinMax);
                run += v;
            }
            abv[3] = run;  // "bin -1" starts behind every candidate that was counted
        }
        if (crowded) misc[0] = 1u;
    }
    __syncthreads();
    trace_mark<TR>(tr, 6);  // prefix done
    if (misc[0] != 0u) {
        // A bin is too full: cand still holds the candidates, take the radix descent.  Every
        // lane reads the same flag; the barrier keeps the descent from reusing this area
        // before all of them have.
        __syncthreads();
        select_radix_write<ELT>(cand, count, k, out_vals, out_idx, row_out);
        return;
    }

    // ---- file the possible winners by bin, in place of cand (every lane has its own in registers)
    uint32_t start[NS];
#pragma unroll
    for (int e = 0; e < NS; ++e) {
        start[e] = live[e] ? abv[bin[e] + 4] : 0xffffffffu;
        if (start[e] < (uint32_t)k) cand[start[e] + atomicSub(&cnt[bin[e]], 1u) - 1u] = c[e];
    }
    __syncthreads();
    trace_mark<TR>(tr, 7);  // filed
#pragma unroll
    for (int e = 0; e < NS; ++e)
        if (start[e] < (uint32_t)k) {
            const uint32_t end = abv[bin[e] + 3];  // start of the next lower bin
            uint32_t r = start[e];
            for (uint32_t j = start[e]; j < end; ++j) r += (cand[j] > c[e]) ? 1u : 0u;
            if (r < (uint32_t)k) write_composite<ELT>(c[e], out_vals, out_idx, row_out * k + r);
        }
}

// ---- Stage 2 for callers that know the candidates' key range before the workgroup's barrier -------------
// select_bucket_rank() spends two barriers on the range of the keys and two on a prefix sum that every
// wavefront takes part in.  A kernel that touches every candidate anyway before its barrier (the fused
// Stage 1 merging its lanes' running maxima) folds the range into that step, and then this shorter form
// does: one histogram (the atomic's return value is the candidate's place among its bin's arrivals), a
// prefix sum by the first wavefront alone (it is a chain of dependent steps either way; with one
// wavefront there is no second level and one barrier less), filing by bin, exact rank inside the bin.
//
// LDS behind cand (count rounded up to even, 16-byte aligned): cnt[kBkBins], abv[kBkBins + 8], misc[32].
// Before the barrier that precedes the call, the caller has: zeroed cnt[0 .. 1 << binned_lg_bins(count)) and
// misc[0]; set misc[2] / misc[3] to an upper bound and the OR (or a superset of its bits) of the candidates'
// value keys, and misc[1] and misc[4] each to a lower bound (the larger is used; a bound far below the
// candidates costs bin resolution, and with it the short form: crowded bins send the row to the digit-by-digit
// selection); put the candidates at cand[0 .. count), zeros for none.
__device__ __forceinline__ int binned_lg_bins(int count) {
    int lg = 8;
    while (lg < 11 && (2 << lg) < count) ++lg;
    return lg;
}
__device__ __forceinline__ uint32_t *binned_cnt(u64 *cand, int count) { return (uint32_t *)(cand + ((count + 1) & ~1)); }
__device__ __forceinline__ uint32_t *binned_misc(u64 *cand, int count) { return binned_cnt(cand, count) + 2 * kBkBins + 8; }

// The prefix sum of select_binned(): run by the first wavefront; lane l owns the Q bins below n_bins - l*Q, so lane
// order is descending bin order.  All of a lane's counts are loaded before any is used.
template <int Q>
__device__ __forceinline__ void binned_scan(const uint32_t *cnt, uint32_t *abv, uint32_t *misc, int n_bins, int k, int lane) {
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    const int hi = n_bins - 1 - lane * Q;
    v4u v[Q / 4];
#pragma unroll
    for (int j = 0; j < Q / 4; ++j) v[j] = *(const v4u *)&cnt[hi - 4 * j - 3];
    uint32_t s = 0;
#pragma unroll
    for (int j = 0; j < Q / 4; ++j) s += v[j].x + v[j].y + v[j].z + v[j].w;
    uint32_t run = wave_incl_scan_u32(s) - s;
    bool crowded = false;
#pragma unroll
    for (int j = 0; j < Q / 4; ++j) {
        v4u a;
        a.w = run;
        a.z = run + v[j].w;
        a.y = a.z + v[j].z;
        a.x = a.y + v[j].y;
        // a bin that may hold winners and is too full for the in-bin count to stay cheap
        crowded = crowded || (a.w < (uint32_t)k && v[j].w > (uint32_t)kBkBinMax) || (a.z < (uint32_t)k && v[j].z > (uint32_t)kBkBinMax) ||
                  (a.y < (uint32_t)k && v[j].y > (uint32_t)kBkBinMax) || (a.x < (uint32_t)k && v[j].x > (uint32_t)kBkBinMax);
        *(v4u *)&abv[hi - 4 * j - 3 + 4] = a;
        run = a.x + v[j].x;
    }
    if (lane == kWave - 1) abv[3] = run;  // "bin -1" starts behind everything
    if (__ballot(crowded) != 0ull && lane == 0) misc[0] = 1u;
}

template <int ELT, int NS, bool TR>
__device__ __forceinline__ void select_binned_ns(u64 *cand, int count, int k, int idx_bits, void *out_vals,
                                                 int32_t *out_idx, int64_t row_out, u64 *tr) {
    const int tid = threadIdx.x, T = blockDim.x;
    const int lg_bins = binned_lg_bins(count), n_bins = 1 << lg_bins;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    uint32_t *cnt = binned_cnt(cand, count);
    uint32_t *abv = cnt + kBkBins;       // abv[b + 4] = candidates in bins above b, for b = -1 .. n_bins - 1
    uint32_t *misc = abv + kBkBins + 8;  // [0] overflow flag, [1] and [4] lower bounds, [2] largest key
    // (the bounds and the candidates are loaded together)
    const uint32_t lb1 = misc[1], k_max = misc[2], lb4 = misc[4];
    u64 c[NS];
#pragma unroll
    for (int e = 0; e < NS; ++e) {
        const int i = tid + e * T;
        c[e] = (i < count) ? cand[i] : 0ull;
    }
    const uint32_t k_min = lb4 > lb1 ? lb4 : lb1;
    // Bin key as in select_bucket_rank(): the value key relative to the lower bound (below it: 0), without the
    // low bits that are zero in every key of the element type, the varying index bits appended; n_bins bins,
    // linear over that range.
    constexpr int tz = (ELT == ATK_BF16) ? 16 : 0;
    const uint32_t imask = (idx_bits >= 31) ? 0x7fffffffu : ((1u << idx_bits) - 1u);
    const u64 span = ((u64)((k_max - k_min) >> tz) + 1ull) << idx_bits;
    const int rbits = 64 - __clzll((long long)span);
    const int bshift = rbits > lg_bins ? rbits - lg_bins : 0;
    uint32_t bin[NS], pos[NS];
#pragma unroll
    for (int e = 0; e < NS; ++e) {
        const uint32_t key = (uint32_t)(c[e] >> 32);
        const uint32_t rel = key > k_min ? key - k_min : 0u;
        const u64 bk = ((u64)(rel >> tz) << idx_bits) | (((uint32_t)c[e] >> 1) & imask);
        bin[e] = (uint32_t)(bk >> bshift);
    }
#pragma unroll
    for (int e = 0; e < NS; ++e) pos[e] = c[e] ? atomicAdd(&cnt[bin[e]], 1u) : 0u;  // its place among its bin's arrivals
    __syncthreads();
    trace_mark<TR>(tr, 5);  // histogram done
    if (wave == 0) {
        const int q = n_bins >> 6;
        if (q == 4)
            binned_scan<4>(cnt, abv, misc, n_bins, k, lane);
        else if (q == 8)
            binned_scan<8>(cnt, abv, misc, n_bins, k, lane);
        else if (q == 16)
            binned_scan<16>(cnt, abv, misc, n_bins, k, lane);
        else
            binned_scan<32>(cnt, abv, misc, n_bins, k, lane);
    }
    __syncthreads();
    trace_mark<TR>(tr, 6);  // prefix done
    // where the candidate's bin starts and ends (= where the next lower bin starts), loaded together with the flag
    uint32_t start[NS], end[NS];
#pragma unroll
    for (int e = 0; e < NS; ++e) {
        start[e] = abv[bin[e] + 4];
        end[e] = abv[bin[e] + 3];
    }
    if (misc[0] != 0u) {
        // cand still holds the candidates: the digit-by-digit selection takes over (every lane has read the flag
        // before the descent reuses this area)
        __syncthreads();
        select_radix_write<ELT>(cand, count, k, out_vals, out_idx, row_out);
        return;
    }
    // ---- file the possible winners by bin, in place of cand (every lane has its own in registers)
#pragma unroll
    for (int e = 0; e < NS; ++e) {
        if (!c[e]) start[e] = 0xffffffffu;
        if (start[e] < (uint32_t)k) cand[start[e] + pos[e]] = c[e];
    }
    __syncthreads();
    trace_mark<TR>(tr, 7);  // filed
    // ---- exact rank = start of the bin + larger elements of the bin.  The first four of the bin are read in one go,
    // wanted or not (a bin seldom holds more; past its end lies another bin or stale data, masked out).
    u64 peer[NS][4];
#pragma unroll
    for (int e = 0; e < NS; ++e)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = start[e] + (uint32_t)u;
            peer[e][u] = cand[(start[e] < (uint32_t)k && j < end[e]) ? j : 0u];
        }
    // With few winners among many candidates they go to their output slots through LDS (the counts' area is free
    // by now), so that the row is written by whole wavefronts with two stores each, instead of by a few lanes of
    // every wavefront each (1024 candidates, k = 64: -0.2 us; level at 512; a loss below).
    u64 *sorted = (u64 *)cnt;
    const bool staged = (size_t)k * 8 <= (size_t)(2 * kBkBins + 8) * 4 && count >= 8 * k;  // (few winners per wavefront)
#pragma unroll
    for (int e = 0; e < NS; ++e)
        if (start[e] < (uint32_t)k) {
            uint32_t r = start[e];
#pragma unroll
            for (int u = 0; u < 4; ++u) r += (start[e] + (uint32_t)u < end[e] && peer[e][u] > c[e]) ? 1u : 0u;
            for (uint32_t j = start[e] + 4u; j < end[e]; ++j) r += (cand[j] > c[e]) ? 1u : 0u;
            if (r < (uint32_t)k) {
                if (staged)
                    sorted[r] = c[e];
                else
                    write_composite<ELT>(c[e], out_vals, out_idx, row_out * k + r);
            }
        }
    if (staged) {
        __syncthreads();
        for (int i = tid; i < k; i += T) write_composite<ELT>(sorted[i], out_vals, out_idx, row_out * k + i);
    }
}

// true when select_binned() takes the short form for this many candidates (else the caller need not
// prepare the range and the counts: the digit-by-digit selection runs)
__device__ __forceinline__ bool binned_fits(int count) { return count <= kBkSlots * (int)blockDim.x; }

template <int ELT, bool TR = false>
__device__ __forceinline__ void select_binned(u64 *cand, int count, int k, int idx_bits, void *out_vals,
                                              int32_t *out_idx, int64_t row_out, u64 *tr = nullptr) {
    const int T = blockDim.x;
    if (!binned_fits(count)) {
        select_radix_write<ELT>(cand, count, k, out_vals, out_idx, row_out);
        return;
    }
    if (count <= T)
        select_binned_ns<ELT, 1, TR>(cand, count, k, idx_bits, out_vals, out_idx, row_out, tr);
    else if (count <= 2 * T)
        select_binned_ns<ELT, 2, TR>(cand, count, k, idx_bits, out_vals, out_idx, row_out, tr);
    else
        select_binned_ns<ELT, kBkSlots, TR>(cand, count, k, idx_bits, out_vals, out_idx, row_out, tr);
}

#endif  // __HIPCC__


}  // namespace atk
