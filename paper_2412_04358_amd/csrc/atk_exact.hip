// exact_topk: the exact comparison point (Section 1; RadixSelect of Appendix D.2).
//
// Small rows: one workgroup per row; the row's composites live in LDS and go through the
// same radix select + ordering as Stage 2.
//
// Long rows: the RadixSelect scheme on the 64-bit composite (value key, then index, so that
// ties at the k-th value resolve to the lowest indices - the "second collect step" the
// listing's caption mentions), most significant digit first, 11-bit digits over the bits of the
// composite that can differ between elements (see Squeeze).  One pass = a histogram kernel over
// the whole row (every workgroup a chunk, LDS histogram flushed to a global one), whose last
// workgroup per row - or, on big launches, a small kernel - picks the digit bucket holding the
// k-th element.  A row is finished as soon as its bucket holds exactly the number of elements
// still needed.  Then one more sweep collects every element at or above the threshold, and the
// k survivors are ordered: in LDS when they fit, else by a partition sort (bins that are linear
// in the squeezed composite, one wavefront per bin), with a least-significant-digit radix sort
// in global memory for rows whose values pile up in a few bins.
// Small k has two shortcuts: rows whose first digit leaves few elements in play have them copied
// out and selected in LDS, and on big inputs the threshold for that copy is first guessed from a
// sample of the row (rows where the guess lets too much through start over digit by digit).
#include <cstdlib>
#include <cstring>

#include "atk_common.h"
#include "atk_select.h"

namespace atk {

namespace {

constexpr int kExBins = 2048;            // 11-bit digits
constexpr int kExDigit = 11;             // bits per pass of the digit descent (the last pass takes what is left)
constexpr int kExChunk = 16384;          // elements per workgroup of the sweeps (inputs that fill the chip with that)
constexpr int kExChunkMin = 4096;        // ... down to this on smaller inputs, while a sweep stays within kExFusedMaxWgs workgroups
constexpr int kExFusedMaxWgs = 1024;     // largest sweep whose last workgroup per row also decides the digit (see ex_hist_kernel)
constexpr int kExRow = kExBins + kTicketStride;  // words per row of the global histograms: the bins, then the row's ticket
constexpr int kSortTile = 2048;          // granule of the sort buffers' sizes
constexpr int kSortLdsMaxK = 4096;       // survivors ordered in LDS by one workgroup
constexpr int kPartTile = 4096;          // survivors per workgroup of the partition sort's sweeps
constexpr int kPartMaxBins = 2048;
constexpr int kPartWaveMax = 512;        // largest bin that one wavefront orders on its own
constexpr int kFilterMaxK = 1024;        // largest k that takes the copy-out path (its selection must fit 64 KB of LDS)
constexpr int kFilterMaxKBig = 4096;     // ... with at most one row per CU: the selection may take all of a CU's LDS
constexpr int kFilterCapBig = 8192;      // ... and chooses from this many elements
constexpr int kSampleMaxK = 512;        // largest k whose threshold is first guessed from a sample of the row
constexpr int kSampleChunk = 4096;       // the sample: every 16th run of 4096 elements
constexpr int kSampleStride = 16;         // ... for k <= 128; every 8th up to 256, every 4th up to 512: about 2048 elements reach the guess
inline int sample_stride(int64_t k) { return k <= 128 ? kSampleStride : (k <= 256 ? kSampleStride / 2 : kSampleStride / 4); }
constexpr int64_t kSampleMinBytes = 128ll << 20;  // smaller inputs are not worth the extra launches
constexpr uint32_t kSampledPass = 0xfffffffeu, kSampledLast = 0xffffffffu;  // in place of a copy-out limit: see decide_row()
constexpr int kFilterCap = 4096;         // elements at or above the first digit's bucket that one workgroup selects from in LDS

struct ExRowState {  // one per row, 32 bytes
    u64 prefix;      // decided high bits of the threshold (of its squeezed form: see Squeeze)
    uint32_t need;   // elements still needed inside the current bucket
    uint32_t done;   // threshold known
    uint32_t cursor; // survivors written so far
    uint32_t mode;   // 0: digit by digit; 1: few enough elements share the first digit's bucket or lie above it -
                     // they are copied out and selected in LDS; 2: finished that way; 3 (large k): the
                     // survivors are ordered by the digit-by-digit global sort, not by the partition sort
    u64 cmax;        // largest survivor (large k)
};

int64_t pow2_ceil64(int64_t v) {
    int64_t p = 1;
    while (p < v) p <<= 1;
    return p;
}
int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace

int make_exact_plan(int64_t m, int64_t n, int64_t k, int dtype, ExactPlan *pl) {
    ExactPlan p;
    p.dtype = dtype;
    p.m = m;
    p.n = n;
    p.k = k;
    p.T = kMaxThreads;
    p.chunks = 1;
    p.chunk_elems = kExChunk;
    p.scratch_bytes = 0;
    p.state_bytes = 0;
    p.lds_bytes = 0;
    p.filter = false;
    p.filter_cap = kFilterCap;
    p.sample = false;
    p.idx_n = n;
    if (m >= (1ll << 31)) return ATK_ERR_UNSUPPORTED;
    const int64_t lds = select_lds_bytes(n, (int)pow2_ceil64(k < (1 << 20) ? k : (1 << 20)));
    // One workgroup per row while the row fits 64 KB of LDS; up to all 160 KB of a CU (about 18000
    // elements) when there is at most one row per CU: one launch instead of ten (128 x 8192: 41 -> 24 us).
    // With more rows the sweeps of the long-row path use the chip better (2048 x 8192: 110 against 270 us).
    p.single_wg = lds <= kLdsBudget || (lds <= kLdsBudgetWholeRow && m <= kNumCU);
    if (p.single_wg) {
        p.lds_bytes = (int)lds;
        *pl = p;
        return ATK_OK;
    }
    // inputs that do not fill the chip with 16384-element chunks: smaller ones, as long as the sweep stays a launch
    // whose last workgroup per row decides the digit (128 x 65536, k = 64: 55 -> 44 us; 1 x 2^20: 47 -> 34 us)
    while (p.chunk_elems > kExChunkMin && m * ceil_div64(n, p.chunk_elems / 2) <= kExFusedMaxWgs) p.chunk_elems >>= 1;
    if (plan_override().xc) p.chunk_elems = plan_override().xc;  // "XC=<elements>": the sweep's chunk (sweeps, tests)
    p.chunks = (int)ceil_div64(n, p.chunk_elems);
    if (m > 65535) return ATK_ERR_UNSUPPORTED;  // rows are the grid's y dimension: exact_topk() passes blocks of rows
    // state pool: global histograms (left zero by every call)
    p.state_bytes = m * (int64_t)kExRow * 4;
    // data pool: row states, survivors, and for the global sort a second buffer + tile histograms
    int64_t bytes = m * (int64_t)sizeof(ExRowState);
    bytes = ceil_div64(bytes, 256) * 256;
    bytes += m * k * 8;
    // copy-out buffer of the small-k path, as long as it stays modest (256 MB)
    p.filter = k <= kFilterMaxK && m * (int64_t)kFilterCap * 8 <= (256ll << 20);
    if (!p.filter && k <= kFilterMaxKBig) {
        // k up to 4096: twice the elements, selected in up to 160 KB of LDS, one row per CU at a time (128 x 2^20,
        // k = 4096: two sweeps instead of four or five).  With more rows than CUs the selections queue up, about
        // 50 us per round of rows: then only where the saved sweeps are worth more (384 x 2^19: 600 -> 476 us;
        // 2048 x 32768 would go from 327 to 526 us).
        const int64_t es = (dtype == ATK_F32) ? 4 : 2;
        const int64_t rounds = ceil_div64(m, kNumCU);
        if (rounds == 1 || (m * n * es > rounds * (120ll << 20) && m * (int64_t)kFilterCapBig * 8 <= (256ll << 20))) {
            p.filter = true;
            p.filter_cap = kFilterCapBig;
        }
    }
    if (p.filter) bytes += m * (int64_t)p.filter_cap * 8;
    {
        // ATK_PLAN="XS=1" takes the sampled threshold on small inputs too, "XS=0" never (tests, sweeps)
        const bool force = plan_override().xs > 0, off = plan_override().xs < 0;
        const int64_t es = (dtype == ATK_F32) ? 4 : 2;
        p.sample = p.filter && !off && k <= kSampleMaxK && n >= 4 * (int64_t)kSampleChunk * kSampleStride &&
                   (force || m * n * es >= kSampleMinBytes * (k > 256 ? 2 : 1));  // (64 x 2^19 f32, k = 512: 75 us without, 86 with)
    }
    if (k > kSortLdsMaxK) {
        bytes += m * k * 8;
        bytes += m * ceil_div64(k, kSortTile) * 256 * 4;
        bytes += 256 + m * (int64_t)kPartMaxBins * 4 * 4;  // partition sort: list of big bins, counts, starts, cursors
    }
    p.scratch_bytes = bytes;
    *pl = p;
    return ATK_OK;
}

// ------------------------------------------------------------------------------------ small rows
template <int ELT>
__global__ void __launch_bounds__(kMaxThreads) exact_small_kernel(const void *x, const int32_t *xi, int n, int k, int idx_bits,
                                                                  void *out_vals, int32_t *out_idx) {
    extern __shared__ __align__(16) unsigned char smem[];
    u64 *cand = (u64 *)smem;
    const int r = blockIdx.x;
    const int T = blockDim.x;
    auto load_bits = [&](int i) -> uint32_t {
        if (ELT == ATK_F32) return ((const uint32_t *)x)[(int64_t)r * n + i];
        return ((uint32_t)((const uint16_t *)x)[(int64_t)r * n + i]) << 16;
    };
    auto index_of = [&](int i) -> int32_t { return xi ? xi[(int64_t)r * n + i] : i; };
    int i = threadIdx.x;
    for (; i + 3 * T < n; i += 4 * T) {  // four loads in flight
        uint32_t b0 = load_bits(i), b1 = load_bits(i + T), b2 = load_bits(i + 2 * T), b3 = load_bits(i + 3 * T);
        const int32_t i0 = index_of(i), i1 = index_of(i + T), i2 = index_of(i + 2 * T), i3 = index_of(i + 3 * T);
        cand[i] = make_composite(b0, i0);
        cand[i + T] = make_composite(b1, i1);
        cand[i + 2 * T] = make_composite(b2, i2);
        cand[i + 3 * T] = make_composite(b3, i3);
    }
    for (; i < n; i += T) cand[i] = make_composite(load_bits(i), index_of(i));
    __syncthreads();
    select_write<ELT>(cand, n, k, idx_bits, out_vals, out_idx, (int64_t)r);
}

// ------------------------------------------------------------------------------------ long rows
// Calls f(composite, valid) for every element of this workgroup's chunk of row r, in an order that only
// depends on the launch (two sweeps of a chunk see the same order), four loads per lane in flight.
// xi: when not NULL, the column index that element i of a row stands for (the rows are then lists of
// (value, index) pairs, such as Stage-1 candidates), else i itself.
// Rows of a whole number of 16-byte vectors at a 16-byte aligned base, without xi, are read 16 bytes per
// load (a lane then takes 4 or 8 adjacent elements): with 4-byte loads a CU has too few bytes in flight
// to keep HBM busy (a first-digit pass over 128 x 65536 fp32 took 16 us, the bytes alone take 5).
typedef uint32_t ex_v4u __attribute__((ext_vector_type(4)));
template <int ELT, typename F>
__device__ __forceinline__ void for_chunk(const void *x, const int32_t *xi, int64_t n, int r, int chunk, F f,
                                          int chunk_elems = kExChunk) {
    const int64_t e0 = (int64_t)chunk * chunk_elems;
    const int64_t e1 = (e0 + chunk_elems < n) ? e0 + chunk_elems : n;
    const int T = blockDim.x;
    // both paths keep whole wavefronts together (f may use wavefront-wide operations and carry
    // wavefront-uniform state): their loop conditions only look at the wavefront's first element
    const int lane = threadIdx.x & (kWave - 1);
    constexpr int VE = (ELT == ATK_F32) ? 4 : 8;  // elements per 16-byte vector
    if (!xi && n % VE == 0 && ((uintptr_t)x & 15) == 0) {  // uniform over the launch; e0, e1 are then multiples of VE too
        const ex_v4u *row = (const ex_v4u *)((const unsigned char *)x + ((int64_t)r * n + e0) * (ELT == ATK_F32 ? 4 : 2));
        const int nv = (int)((e1 - e0) / VE);
        auto feed = [&](const ex_v4u &q, int v, bool ok) {
            const int64_t i = e0 + (int64_t)v * VE;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (ELT == ATK_F32) {
                    f(ok ? make_composite(q[j], (int32_t)(i + j)) : 0ull, ok);
                } else {
                    f(ok ? make_composite(q[j] << 16, (int32_t)(i + 2 * j)) : 0ull, ok);
                    f(ok ? make_composite(q[j] & 0xffff0000u, (int32_t)(i + 2 * j + 1)) : 0ull, ok);
                }
            }
        };
        int v = threadIdx.x;
        for (; v - lane + 3 * T + (kWave - 1) < nv; v += 4 * T) {
            const ex_v4u q0 = __builtin_nontemporal_load(row + v), q1 = __builtin_nontemporal_load(row + v + T),
                         q2 = __builtin_nontemporal_load(row + v + 2 * T), q3 = __builtin_nontemporal_load(row + v + 3 * T);
            feed(q0, v, true);
            feed(q1, v + T, true);
            feed(q2, v + 2 * T, true);
            feed(q3, v + 3 * T, true);
        }
        for (; v - lane < nv; v += T) {
            const bool ok = v < nv;
            const ex_v4u q = __builtin_nontemporal_load(row + (ok ? v : 0));  // lanes past the end re-read the chunk's first vector
            feed(q, v, ok);
        }
        return;
    }
    auto load_bits = [&](int64_t i) -> uint32_t {
        if (ELT == ATK_F32) return __builtin_nontemporal_load((const uint32_t *)x + (int64_t)r * n + i);
        return ((uint32_t)__builtin_nontemporal_load((const uint16_t *)x + (int64_t)r * n + i)) << 16;
    };
    int64_t i = e0 + threadIdx.x;
    auto index_of = [&](int64_t i) -> int32_t { return xi ? xi[(int64_t)r * n + i] : (int32_t)i; };
    for (; i - lane + 3 * T + (kWave - 1) < e1; i += 4 * T) {
        const uint32_t b0 = load_bits(i), b1 = load_bits(i + T), b2 = load_bits(i + 2 * T), b3 = load_bits(i + 3 * T);
        const int32_t i0 = index_of(i), i1 = index_of(i + T), i2 = index_of(i + 2 * T), i3 = index_of(i + 3 * T);
        f(make_composite(b0, i0), true);
        f(make_composite(b1, i1), true);
        f(make_composite(b2, i2), true);
        f(make_composite(b3, i3), true);
    }
    for (; i - lane < e1; i += T) {
        const bool ok = i < e1;
        f(ok ? make_composite(load_bits(i), index_of(i)) : 0ull, ok);
    }
}

// The radix select and the partition sort work on a squeezed form of the composite, from which the bits
// that carry nothing are taken out: the low `drop` bits of the order key (16 for bf16: they only repeat
// the sign) and the high bits of the index field (column indices are below 2^(keep - 1), so the bits
// of 0x7fffffff - idx above them are all ones).  The map keeps the order and loses nothing on the
// elements of one call.  The digit descent then has (32 - drop) + keep bits to decide instead of 64
// (bf16, n = 65536: 3 passes instead of 6 when ties take it down to the index), and equal values with
// different indices lie `1` apart per index step instead of 2^32: linear bins also divide long runs
// of ties (bf16 rows hold few distinct values).
struct Squeeze {
    int drop, keep;
    __device__ __forceinline__ u64 operator()(u64 c) const {
        return ((c >> (32 + drop)) << keep) | (c & ((1ull << keep) - 1ull));
    }
    // The composite that t is the squeezed form of, with the bits that were taken out put back as the
    // elements of this call have them: for an element c, c >= expand(t) exactly when (*this)(c) >= t
    // (the sweep that collects the survivors compares composites as they are: it has no instruction to spare).
    __device__ __forceinline__ u64 expand(u64 t) const {
        const u64 kh = t >> keep;  // the key without its low `drop` bits
        u64 key = kh << drop;
        if (drop && !((kh >> (31 - drop)) & 1ull)) key |= (1ull << drop) - 1ull;  // keys of negative bf16 values end in ones
        const u64 kept = (1ull << keep) - 1ull;
        return (key << 32) | (0xffffffffull & ~kept) | (t & kept);
    }
};

// The digit bucket that holds the need-th largest element of row r, from the row's global
// histogram `gh`; updates the row state and leaves the histogram zeroed.  Called by a whole
// workgroup of at least 256 lanes (uniformly); wave_tot: four words of LDS.
// The histogram is read and cleared with agent-scope atomic accesses: they act on memory, not
// on one XCD's L2, as the atomics that filled it did.
// FIRST: the first pass; the row state is not read (no digit decided, k elements needed) but set up.
// filter_cap > 0 (first pass only): a row with at most that many elements in or above the chosen
// bucket, and not finished by this pass alone, is handed to the copy-out path (mode 1).
// filter_cap == kSampledPass (a pass over a sample of the row): the counts say nothing about the whole
// row, so the row is never finished here; kSampledLast (the last such pass): the row goes to the
// copy-out path with the digits decided so far as its threshold.
template <bool FIRST>
__device__ __forceinline__ void decide_row(ExRowState *st, uint32_t *gh, int r, u64 prefix, uint32_t need, int shift,
                                           int last_pass, uint32_t filter_cap, uint32_t *wave_tot) {
    const int tid = threadIdx.x;
    // lane t of the first 256 owns bins 2047-8t-7 .. 2047-8t: lane order is descending bin order
    const bool owner = tid < 256;
    uint32_t hb[8], s = 0;
    const int base = owner ? kExBins - 8 - 8 * tid : 0;
    // one condition around the eight loads, so that they are issued together (a condition per load
    // puts each in a branch of its own, where it waits for the one before it)
#pragma unroll
    for (int q = 0; q < 8; ++q) hb[q] = 0u;
    if (owner) {
#pragma unroll
        for (int q = 0; q < 8; ++q) hb[q] = __hip_atomic_load(&gh[base + q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        if (hb[q]) __hip_atomic_store(&gh[base + q], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s += hb[q];
    }
    const uint32_t incl = wave_incl_scan_u32(s);
    if (owner && (tid & 63) == 63) wave_tot[tid >> 6] = incl;
    __syncthreads();
    if (!owner) return;
    uint32_t above = incl - s;
    for (int w = 0; w < (tid >> 6); ++w) above += wave_tot[w];
#pragma unroll
    for (int q = 7; q >= 0; --q) {
        const uint32_t with = above + hb[q];
        if (above < need && with >= need) {
            const uint32_t left = need - above;
            const bool sampled = filter_cap >= kSampledPass;
            const bool done = !sampled && (hb[q] == left || last_pass);
            ExRowState ns;
            ns.prefix = prefix | ((u64)(uint32_t)(base + q) << shift);
            ns.need = left;
            ns.done = done ? 1u : 0u;
            ns.cursor = FIRST ? 0u : st[r].cursor;
            ns.mode = (filter_cap == kSampledLast || (!sampled && filter_cap && !done && with <= filter_cap))
                          ? 1u
                          : (FIRST ? 0u : st[r].mode);
            ns.cmax = FIRST ? 0ull : st[r].cmax;
            st[r] = ns;
        }
        above = with;
    }
}

// One pass of the digit descent for row blockIdx.y: every workgroup counts the digits of its chunk
// (LDS histogram, flushed to the row's global one with agent-scope atomics).
// FUSED (launches of few workgroups, where a second launch costs as much as the sweep): the
// workgroup that finishes the row last - a ticket, taken after its own counts have been
// acknowledged - goes on to decide_row().  Big launches leave that to ex_decide_kernel: there the
// wait for the acknowledgement at the end of every workgroup would idle lanes that could stream.
template <int ELT, bool FIRST, bool FUSED>
__global__ void __launch_bounds__(kMaxThreads) ex_hist_kernel(const void *x, const int32_t *xi, int64_t n, ExRowState *st,
                                                              uint32_t *ghist, int shift, int width, int last_pass,
                                                              uint32_t filter_cap, uint32_t k, int chunk_elems,
                                                              int chunk_stride, int runs, Squeeze sq) {
    __shared__ uint32_t lh[kExBins];
    __shared__ uint32_t wave_tot[4];
    __shared__ uint32_t is_last;
    const int r = blockIdx.y, tid = threadIdx.x;
    if (!FIRST && st[r].done) return;  // uniform over the workgroup
    const u64 prefix = FIRST ? 0ull : st[r].prefix;
    const uint32_t need = FIRST ? k : st[r].need;
    const u64 hi_mask = (shift + width >= 64) ? 0ull : (~0ull << (shift + width));
    const uint32_t dmask = (1u << width) - 1u;
    for (int i = tid; i < kExBins; i += blockDim.x) lh[i] = 0;
    __syncthreads();
    // chunk_stride > 1: a sample of the row, in small chunks; runs > 1: several chunks per workgroup
    // A digit that lies in the key alone (the first pass always does) is read off the composite with one
    // shift; only a digit that reaches into the index field needs the squeezed form of every element.
    const bool key_digit = shift >= sq.keep;  // uniform over the launch
    const int key_shift = 32 + sq.drop, dshift = shift - sq.keep;
    const u64 key_mask = hi_mask >> sq.keep, key_prefix = prefix >> sq.keep;
    for (int q = 0; q < runs; ++q) {
        const int64_t chunk = ((int64_t)blockIdx.x * runs + q) * chunk_stride;
        if (chunk * chunk_elems >= n) break;  // uniform over the workgroup
        if (key_digit)
            for_chunk<ELT>(
                x, xi, n, r, (int)chunk,
                [&](u64 c, bool ok) {
                    const u64 q = c >> key_shift;
                    if (ok && (q & key_mask) == key_prefix) atomicAdd(&lh[(uint32_t)(q >> dshift) & dmask], 1u);
                },
                chunk_elems);
        else
            for_chunk<ELT>(
                x, xi, n, r, (int)chunk,
                [&](u64 c, bool ok) {
                    const u64 q = sq(c);
                    if (ok && (q & hi_mask) == prefix) atomicAdd(&lh[(uint32_t)(q >> shift) & dmask], 1u);
                },
                chunk_elems);
    }
    __syncthreads();
    uint32_t *gh = ghist + (int64_t)r * kExRow;
    for (int i = tid; i < kExBins; i += blockDim.x) {
        const uint32_t v = lh[i];
        if (v) __hip_atomic_fetch_add(&gh[i], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!FUSED) return;
    // this lane's counts have been acknowledged (a barrier alone does not wait for them); the memory clobber keeps the
    // compiler from moving the atomics above past it, or the ticket below before it
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        const uint32_t ticket = __hip_atomic_fetch_add(&gh[kExBins], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        is_last = (ticket == gridDim.x - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return;
    if (tid == 0) __hip_atomic_store(&gh[kExBins], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    decide_row<FIRST>(st, gh, r, prefix, need, shift, last_pass, filter_cap, wave_tot);
}

// The same decision as a launch of its own, one workgroup of 256 lanes per row.
template <bool FIRST>
__global__ void __launch_bounds__(256) ex_decide_kernel(ExRowState *st, uint32_t *ghist, int shift, int last_pass,
                                                        uint32_t filter_cap, uint32_t k) {
    __shared__ uint32_t wave_tot[4];
    const int r = blockIdx.x;
    if (!FIRST && st[r].done) return;
    decide_row<FIRST>(st, ghist + (int64_t)r * kExRow, r, FIRST ? 0ull : st[r].prefix, FIRST ? k : st[r].need, shift, last_pass,
                      filter_cap, wave_tot);
}

// Every element at or above the row's threshold goes to sel[row][..] (exactly k of them, any order).
// A workgroup sweeps its chunk once, counting its survivors and parking the first kStash of
// them in LDS, then reserves their places with one atomic on the row's cursor (one per 16384
// elements: at large k, one per wavefront and load had every wavefront of a row queueing on
// the same counter).  Few survivors (small k) are written from LDS; if they did not all fit,
// the chunk is swept a second time and written straight from registers.
// FILTER: the same sweep for the rows in mode 1, whose threshold so far is just the first digit:
// at most the plan's filter_cap elements per row reach it, and they go to a buffer of that stride.
// kStash: 2048 keeps the sweep's occupancy up when few survive; 6144 saves the second sweep when about a
// quarter of a chunk does.
template <int ELT, bool FILTER, int kStash>
__global__ void __launch_bounds__(kMaxThreads) ex_collect_kernel(const void *x, const int32_t *xi, int64_t n, ExRowState *st, u64 *sel,
                                                                 int64_t k, int chunk_elems, Squeeze sq) {
    __shared__ u64 stash[kStash];
    __shared__ uint32_t wave_cnt[kMaxThreads / kWave];
    __shared__ uint32_t wave_base[kMaxThreads / kWave];
    __shared__ uint32_t stash_n, first_pos;
    const int r = blockIdx.y;
    if (FILTER ? st[r].mode != 1u : st[r].mode == 2u) return;  // uniform over the workgroup
    const u64 thr = sq.expand(st[r].prefix);
    u64 *dst = sel + (int64_t)r * k;  // k: the row stride of sel (the buffer's for FILTER)
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    if (threadIdx.x == 0) stash_n = 0;
    __syncthreads();
    uint32_t mine = 0;  // survivors of this wavefront's share (the same number in each of its lanes)
    u64 cmax_local = 0ull;
    for_chunk<ELT>(x, xi, n, r, blockIdx.x, [&](u64 c, bool ok) {
        const bool keep = ok && c >= thr;
        if (!FILTER && keep && c > cmax_local) cmax_local = c;
        const u64 mask = __ballot(keep);
        if (mask) {  // uniform over the wavefront
            const uint32_t cnt = (uint32_t)__popcll(mask);
            uint32_t at = 0;
            if (lane == 0) at = atomicAdd(&stash_n, cnt);
            at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at) +
                 __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            if (keep && at < (uint32_t)kStash) stash[at] = c;
            mine += cnt;
        }
    }, chunk_elems);
    if (lane == 0) wave_cnt[wave] = mine;
    if (!FILTER) {  // the row's largest survivor, for the partition sort's bins
        u64 lo = ~0ull, hi = cmax_local;
        wave_min_max_u64(lo, hi);
        if (lane == 0 && hi) atomicMax((unsigned long long *)&st[r].cmax, (unsigned long long)hi);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t total = 0;
        for (int w = 0; w < n_waves; ++w) {
            wave_base[w] = total;
            total += wave_cnt[w];
        }
        first_pos = total ? atomicAdd(&st[r].cursor, total) : 0u;
    }
    __syncthreads();
    const uint32_t total = stash_n, first = first_pos;
    if (total <= (uint32_t)kStash) {
        for (uint32_t i = threadIdx.x; i < total; i += blockDim.x)
            if (first + i < (uint32_t)k) dst[first + i] = stash[i];
        return;
    }
    uint32_t cursor = first + wave_base[wave];
    for_chunk<ELT>(x, xi, n, r, blockIdx.x, [&](u64 c, bool ok) {
        const bool keep = ok && c >= thr;
        const u64 mask = __ballot(keep);
        const uint32_t pos = cursor + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        if (keep && pos < (uint32_t)k) dst[pos] = c;
        cursor += (uint32_t)__popcll(mask);
    }, chunk_elems);
}

// Small k on rows of moderate length, after the first digit and the copy-out path: the rows that are still open
// (more elements in play than the copy-out buffer holds: ties, values on few levels) are rare, and a launch cannot
// be skipped without asking the device.  So instead of one launch per remaining digit plus two to collect and order,
// all of which usually find nothing to do, this is one launch whose workgroups return at once unless their row is
// open; a workgroup that stays takes its row through the remaining digits alone (LDS histogram over the whole row
// per digit), collects the k survivors in LDS and writes them in order.
constexpr int64_t kRestMaxRow = 1 << 18;  // longest row handled this way (one workgroup re-reads it once per digit)
template <int ELT>
__global__ void __launch_bounds__(kMaxThreads) ex_rest_kernel(const void *x, const int32_t *xi, int64_t n, ExRowState *st, int k,
                                                              int sq_bits, int n_passes, int chunk_elems, Squeeze sq,
                                                              void *out_vals, int32_t *out_idx) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ uint32_t lh[kExBins];
    __shared__ uint32_t wave_tot[4];
    __shared__ u64 s_prefix;
    __shared__ uint32_t s_need, s_done, s_cursor;
    const int r = blockIdx.x, tid = threadIdx.x;
    if (st[r].mode == 2u) return;  // finished by the copy-out path (uniform over the workgroup)
    u64 prefix = st[r].prefix;
    uint32_t need = st[r].need;
    bool done = st[r].done != 0u;
    const int chunks = (int)((n + chunk_elems - 1) / chunk_elems);
    for (int p = 1; p < n_passes && !done; ++p) {
        const int shift = p == n_passes - 1 ? 0 : sq_bits - kExDigit * (p + 1);
        const int width = p == n_passes - 1 ? sq_bits - kExDigit * (n_passes - 1) : kExDigit;
        const u64 hi_mask = (shift + width >= 64) ? 0ull : (~0ull << (shift + width));
        const uint32_t dmask = (1u << width) - 1u;
        for (int i = tid; i < kExBins; i += blockDim.x) lh[i] = 0u;
        __syncthreads();
        for (int c = 0; c < chunks; ++c)
            for_chunk<ELT>(
                x, xi, n, r, c,
                [&](u64 cc, bool ok) {
                    const u64 q = sq(cc);
                    if (ok && (q & hi_mask) == prefix) atomicAdd(&lh[(uint32_t)(q >> shift) & dmask], 1u);
                },
                chunk_elems);
        __syncthreads();
        // the digit bucket that holds the need-th largest: lane t owns bins 2047-8t-7 .. 2047-8t (descending)
        uint32_t hb[8], sum = 0;
        const int base = kExBins - 8 - 8 * tid;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            hb[q] = lh[base + q];
            sum += hb[q];
        }
        const uint32_t incl = wave_incl_scan_u32(sum);
        if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
        __syncthreads();
        uint32_t above = incl - sum;
        for (int w = 0; w < (tid >> 6); ++w) above += wave_tot[w];
#pragma unroll
        for (int q = 7; q >= 0; --q) {
            const uint32_t with = above + hb[q];
            if (above < need && with >= need) {
                s_prefix = prefix | ((u64)(uint32_t)(base + q) << shift);
                s_need = need - above;
                s_done = (hb[q] == need - above || p == n_passes - 1) ? 1u : 0u;
            }
            above = with;
        }
        __syncthreads();
        prefix = s_prefix;
        need = s_need;
        done = s_done != 0u;
        __syncthreads();
    }
    // every element at or above the threshold: exactly k of them, into LDS
    u64 *sel = (u64 *)smem;
    uint32_t *rk = (uint32_t *)(sel + pow2_ceil_dev(k));
    if (tid == 0) s_cursor = 0u;
    for (int i = tid; i < kRankMax; i += blockDim.x) rk[i] = 0u;
    __syncthreads();
    const u64 thr = sq.expand(prefix);
    const int lane = tid & (kWave - 1);
    for (int c = 0; c < chunks; ++c)
        for_chunk<ELT>(
            x, xi, n, r, c,
            [&](u64 cc, bool ok) {
                const bool keep = ok && cc >= thr;
                const u64 mask = __ballot(keep);
                if (mask) {  // uniform over the wavefront
                    uint32_t at = 0;
                    if (lane == 0) at = atomicAdd(&s_cursor, (uint32_t)__popcll(mask));
                    at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at) +
                         __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                    if (keep && at < (uint32_t)k) sel[at] = cc;
                }
            },
            chunk_elems);
    __syncthreads();
    order_write<ELT>(sel, k, rk, out_vals, out_idx, (int64_t)r);
}

// k <= kSortLdsMaxK: one workgroup per row orders the survivors in LDS and writes the outputs.
template <int ELT>
__global__ void __launch_bounds__(kMaxThreads) ex_order_lds_kernel(const u64 *sel, const ExRowState *st, int k,
                                                                   void *out_vals, int32_t *out_idx) {
    extern __shared__ __align__(16) unsigned char smem[];
    u64 *s = (u64 *)smem;
    const int kp = pow2_ceil_dev(k);
    uint32_t *rk = (uint32_t *)(s + kp);
    const int r = blockIdx.x;
    if (st[r].mode == 2u) return;  // already written by the copy-out path
    for (int i = threadIdx.x; i < k; i += blockDim.x) s[i] = sel[(int64_t)r * k + i];
    for (int i = threadIdx.x; i < kRankMax; i += blockDim.x) rk[i] = 0;
    __syncthreads();
    order_write<ELT>(s, k, rk, out_vals, out_idx, (int64_t)r);
}

// Rows in mode 1: the copied-out elements (at most cap) contain the k largest; one workgroup
// selects and orders them in LDS, writes the outputs and marks the row finished.
template <int ELT>
__global__ void __launch_bounds__(kMaxThreads) ex_filter_select_kernel(const u64 *buf, ExRowState *st, int k, int idx_bits,
                                                                       int cap, void *out_vals, int32_t *out_idx) {
    extern __shared__ __align__(16) unsigned char smem[];
    u64 *cand = (u64 *)smem;
    const int r = blockIdx.x;
    if (st[r].mode != 1u) return;  // uniform; read by every lane before lane 0 changes it below
    const int count = (int)st[r].cursor;
    if (count > cap) {
        // only after a threshold guessed from a sample: more elements reach it than were copied out.
        // The row starts over, digit by digit over all its elements.
        __syncthreads();  // every lane has read the state
        if (threadIdx.x == 0) {
            ExRowState ns;
            ns.prefix = 0ull;
            ns.need = (uint32_t)k;
            ns.done = 0u;
            ns.cursor = 0u;
            ns.mode = 0u;
            ns.cmax = 0ull;
            st[r] = ns;
        }
        return;
    }
    for (int i = threadIdx.x; i < count; i += blockDim.x) cand[i] = buf[(int64_t)r * cap + i];
    __syncthreads();
    select_write<ELT>(cand, count, k, idx_bits, out_vals, out_idx, (int64_t)r);
    if (threadIdx.x == 0) {
        st[r].mode = 2u;
        st[r].done = 1u;
    }
}

// ---- partition sort of many survivors (k > kSortLdsMaxK) -------------------------------------------
// The k survivors of a row lie between its threshold and its largest element.  They are cut
// into nb bins that are linear in (composite - threshold), a counting pass and a scatter pass
// bring every bin together (highest bin first), and one workgroup per bin orders it in LDS.
// Composites are distinct, so the order is total.  A row in which some bin is too big for LDS
// (values piled on a few levels) is marked mode 3 and left to the digit-by-digit sort below.
struct PartRow {  // per row
    uint32_t shift;
    uint32_t pad;
};
__device__ __forceinline__ uint32_t part_shift(u64 span, int nb) {  // smallest s with (span >> s) < nb
    const int bits = span ? 64 - __clzll((long long)span) : 0;
    int lg = 0;
    while ((1 << lg) < nb) ++lg;
    return bits > lg ? (uint32_t)(bits - lg) : 0u;
}

__global__ void __launch_bounds__(256) part_zero_kernel(uint32_t *words, int64_t count) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) words[i] = 0u;
}

// counts[row][bin] += elements of this tile in bin
__global__ void __launch_bounds__(256) part_hist_kernel(const u64 *sel, const ExRowState *st, int64_t k, int nb,
                                                        uint32_t *counts, Squeeze sq) {
    __shared__ uint32_t lh[kPartMaxBins];
    const int r = blockIdx.y, tid = threadIdx.x;
    const u64 thr = st[r].prefix;  // squeezed already
    const uint32_t shift = part_shift(sq(st[r].cmax) - thr, nb);
    for (int i = tid; i < nb; i += 256) lh[i] = 0;
    __syncthreads();
    const int64_t e0 = (int64_t)blockIdx.x * kPartTile;
    const u64 *row = sel + (int64_t)r * k;
    // the tile's loads are all issued before the first is used (a load under `if (i < k)` would sit in a
    // branch of its own and wait for the one before it): past the end the last element is re-read and dropped
    u64 c[kPartTile / 256];
#pragma unroll
    for (int j = 0; j < kPartTile / 256; ++j) {
        const int64_t i = e0 + j * 256 + tid;
        c[j] = row[i < k ? i : k - 1];
    }
#pragma unroll
    for (int j = 0; j < kPartTile / 256; ++j)
        if (e0 + j * 256 + tid < k) atomicAdd(&lh[(uint32_t)((sq(c[j]) - thr) >> shift)], 1u);
    __syncthreads();
    uint32_t *gc = counts + (int64_t)r * nb;
    for (int i = tid; i < nb; i += 256) {
        const uint32_t v = lh[i];
        if (v) atomicAdd(&gc[i], v);
    }
}

// one workgroup per row: starts[row][bin] = survivors in higher bins; cursors cleared; rows with a
// bin beyond what one workgroup orders in LDS go to the other sort
// (and the bins too big for one wavefront to rank are listed in big[1..], their number in big[0])
__global__ void __launch_bounds__(256) part_scan_kernel(ExRowState *st, int nb, const uint32_t *counts, uint32_t *starts,
                                                        uint32_t *cursors, uint32_t *big) {
    __shared__ uint32_t wave_tot[4];
    __shared__ uint32_t too_big;
    const int r = blockIdx.x, tid = threadIdx.x;
    const uint32_t *gc = counts + (int64_t)r * nb;
    if (tid == 0) too_big = 0;
    __syncthreads();
    // lane t owns the q bins below nb - t*q: lane order is descending bin order
    const int q = nb / 256 > 0 ? nb / 256 : 1;
    const int hi = nb - 1 - tid * q;
    uint32_t s = 0, mx = 0;
    for (int j = 0; j < q; ++j) {
        const uint32_t v = (hi - j >= 0) ? gc[hi - j] : 0u;
        s += v;
        mx = v > mx ? v : mx;
    }
    if (mx > (uint32_t)kSortLdsMaxK) too_big = 1;
    const uint32_t incl = wave_incl_scan_u32(s);
    if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
    __syncthreads();
    uint32_t run = incl - s;
    for (int w = 0; w < (tid >> 6); ++w) run += wave_tot[w];
    for (int j = 0; j < q; ++j)
        if (hi - j >= 0) {
            starts[(int64_t)r * nb + hi - j] = run;
            cursors[(int64_t)r * nb + hi - j] = 0u;
            run += gc[hi - j];
        }
    if (too_big) {
        if (tid == 0) st[r].mode = 3u;
        return;
    }
    for (int j = 0; j < q; ++j)
        if (hi - j >= 0 && gc[hi - j] > (uint32_t)kPartWaveMax) big[1 + atomicAdd(&big[0], 1u)] = (uint32_t)r * kPartMaxBins + (uint32_t)(hi - j);
}

// every element of the tile goes to its bin's segment of dst (any order inside the bin)
__global__ void __launch_bounds__(256) part_scatter_kernel(const u64 *sel, u64 *dst, const ExRowState *st, int64_t k, int nb,
                                                           const uint32_t *starts, uint32_t *cursors, Squeeze sq) {
    __shared__ uint32_t lh[kPartMaxBins];    // count of the tile per bin, then position of the next element
    const int r = blockIdx.y, tid = threadIdx.x;
    if (st[r].mode == 3u) return;
    const u64 thr = st[r].prefix;  // squeezed already
    const uint32_t shift = part_shift(sq(st[r].cmax) - thr, nb);
    for (int i = tid; i < nb; i += 256) lh[i] = 0;
    __syncthreads();
    const int64_t e0 = (int64_t)blockIdx.x * kPartTile;
    const u64 *row = sel + (int64_t)r * k;
    u64 c[kPartTile / 256];
    uint32_t bin[kPartTile / 256];
#pragma unroll
    for (int j = 0; j < kPartTile / 256; ++j) {  // all loads first, as in part_hist_kernel
        const int64_t i = e0 + j * 256 + tid;
        c[j] = row[i < k ? i : k - 1];
    }
#pragma unroll
    for (int j = 0; j < kPartTile / 256; ++j) {
        if (e0 + j * 256 + tid >= k) c[j] = 0ull;
        bin[j] = c[j] ? (uint32_t)((sq(c[j]) - thr) >> shift) : 0u;
        if (c[j]) atomicAdd(&lh[bin[j]], 1u);
    }
    __syncthreads();
    // reserve the tile's share of every bin it touches
    for (int i = tid; i < nb; i += 256) {
        const uint32_t v = lh[i];
        lh[i] = starts[(int64_t)r * nb + i] + (v ? atomicAdd(&cursors[(int64_t)r * nb + i], v) : 0u);
    }
    __syncthreads();
    u64 *orow = dst + (int64_t)r * k;
#pragma unroll
    for (int j = 0; j < kPartTile / 256; ++j)
        if (c[j]) orow[atomicAdd(&lh[bin[j]], 1u)] = c[j];
}

// One wavefront per (row, bin), four to a workgroup, for bins of at most kPartWaveMax elements.  The
// wavefront works alone (no workgroup barrier), its elements in registers and its tables in its own
// pieces of LDS: it cuts the bin once more into kPartSub sub-bins that are linear between the bin's
// smallest and largest element (inside one bin the values are spread almost evenly, so a sub-bin
// holds a couple of elements at most), takes a descending prefix sum over the sub-bin counts,
// files every element into its sub-bin's segment, and an element's rank is its segment's start
// plus the larger elements of that segment.
constexpr int kPartSub = 512;
constexpr int kPartCrowd = 24;  // a sub-bin with more elements than this sends the bin to the bitonic sort
constexpr int kPartSlots = kPartWaveMax / kWave;  // elements a lane holds
__device__ __forceinline__ void wave_sync_lds() {  // orders this wavefront's LDS writes before its later reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
template <int ELT>
__global__ void __launch_bounds__(256) part_sort_small_kernel(const u64 *src, const ExRowState *st, int64_t k, int nb,
                                                              int64_t total_bins, const uint32_t *counts,
                                                              const uint32_t *starts, uint32_t *big, Squeeze sq,
                                                              void *out_vals, int32_t *out_idx) {
    __shared__ u64 filed[4][kPartWaveMax];
    __shared__ uint32_t sub_cnt[4][kPartSub];
    __shared__ uint32_t sub_off[4][kPartSub + 8];  // [sb + 1] = start of sub-bin sb's segment, [0] = end of sub-bin 0's
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & (kWave - 1);
    const int64_t g = (int64_t)blockIdx.x * 4 + wave;
    if (g >= total_bins) return;
    const int r = (int)(g / nb), bin = (int)(g % nb);
    if (st[r].mode == 3u) return;
    const int cnt = (int)counts[(int64_t)r * nb + bin];
    if (cnt == 0 || cnt > kPartWaveMax) return;
    const int64_t start = starts[(int64_t)r * nb + bin];
    const u64 *seg = src + (int64_t)r * k + start;
    u64 *fl = filed[wave];
    uint32_t *sc = sub_cnt[wave], *so = sub_off[wave];

    u64 c[kPartSlots];  // 0 = none
    u64 lo = ~0ull, hi = 0ull;
#pragma unroll
    for (int e = 0; e < kPartSlots; ++e) {
        const int i = lane + e * kWave;
        c[e] = (i < cnt) ? seg[i] : 0ull;
    }
#pragma unroll
    for (int e = 0; e < kPartSlots; ++e)
        if (c[e]) {
            const u64 q = sq(c[e]);
            lo = q < lo ? q : lo;
            hi = q > hi ? q : hi;
        }
    for (int i = lane; i < kPartSub; i += kWave) sc[i] = 0u;
    wave_min_max_u64(lo, hi);
    const uint32_t sh = part_shift(hi - lo, kPartSub);
    uint32_t sb[kPartSlots];
    wave_sync_lds();
#pragma unroll
    for (int e = 0; e < kPartSlots; ++e) {
        sb[e] = c[e] ? (uint32_t)((sq(c[e]) - lo) >> sh) : 0u;
        if (c[e]) atomicAdd(&sc[sb[e]], 1u);
    }
    wave_sync_lds();
    {
        // lane l owns the Q sub-bins below kPartSub - Q*l: lane order is descending sub-bin order
        constexpr int Q = kPartSub / kWave;
        const int top = kPartSub - 1 - lane * Q;
        uint32_t sum = 0, crowd = 0;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            sum += sc[top - q];
            crowd = sc[top - q] > crowd ? sc[top - q] : crowd;
        }
        // Elements piled on a few places of the bin's range (several values with many ties each: the sub-bins
        // tell the values apart, not the indices) would be ranked by comparing each with all of its sub-bin:
        // such a bin joins the list of part_sort_big_kernel, which runs after this launch.
        if (__ballot(crowd > (uint32_t)kPartCrowd)) {  // uniform over the wavefront
            if (lane == 0) big[1 + atomicAdd(&big[0], 1u)] = (uint32_t)r * kPartMaxBins + (uint32_t)bin;
            return;
        }
        uint32_t run = wave_incl_scan_u32(sum) - sum;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            so[top - q + 1] = run;
            run += sc[top - q];
        }
        if (lane == kWave - 1) so[0] = (uint32_t)cnt;
    }
    wave_sync_lds();
#pragma unroll
    for (int e = 0; e < kPartSlots; ++e)
        if (c[e]) fl[so[sb[e] + 1] + atomicSub(&sc[sb[e]], 1u) - 1u] = c[e];
    wave_sync_lds();
#pragma unroll
    for (int e = 0; e < kPartSlots; ++e)
        if (c[e]) {
            const uint32_t s0 = so[sb[e] + 1], s1 = so[sb[e]];
            uint32_t rank = s0;
            for (uint32_t q = s0; q < s1; ++q) rank += (fl[q] > c[e]) ? 1u : 0u;
            write_composite<ELT>(c[e], out_vals, out_idx, (int64_t)r * k + start + rank);
        }
}

// The bins listed by the scan (more than kPartWaveMax elements): workgroups take them in turn and
// order each in LDS with a bitonic network, largest first.
template <int ELT>
__global__ void __launch_bounds__(256) part_sort_big_kernel(const u64 *src, const ExRowState *st, int64_t k, int nb,
                                                            const uint32_t *counts, const uint32_t *starts,
                                                            const uint32_t *big, void *out_vals, int32_t *out_idx) {
    __shared__ u64 s[kSortLdsMaxK];
    const int tid = threadIdx.x;
    const uint32_t n_big = big[0];
    for (uint32_t w = blockIdx.x; w < n_big; w += gridDim.x) {  // the same trips for every lane of the workgroup
        const int r = (int)(big[1 + w] / kPartMaxBins), bin = (int)(big[1 + w] % kPartMaxBins);
        const int cnt = (int)counts[(int64_t)r * nb + bin];
        const int64_t start = starts[(int64_t)r * nb + bin];
        const u64 *seg = src + (int64_t)r * k + start;
        const int kp = pow2_ceil_dev(cnt);
        __syncthreads();  // the previous bin's reads of s are over
        for (int i = tid; i < kp; i += 256) s[i] = (i < cnt) ? seg[i] : 0ull;  // empties sort to the end
        __syncthreads();
        for (int size = 2; size <= kp; size <<= 1) {
            for (int stride = size >> 1; stride >= 1; stride >>= 1) {
                for (int i = tid; i < (kp >> 1); i += 256) {
                    const int lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));
                    const int hi = lo + stride;
                    const bool desc = (lo & size) == 0;
                    const u64 a = s[lo], b = s[hi];
                    const bool sw = desc ? (b > a) : (b < a);
                    if (sw) {
                        s[lo] = b;
                        s[hi] = a;
                    }
                }
                __syncthreads();
            }
        }
        for (int i = tid; i < cnt; i += 256) write_composite<ELT>(s[i], out_vals, out_idx, (int64_t)r * k + start + i);
    }
}

// ---- least-significant-digit radix sort of the survivors of one row, descending, 8-bit digits ----
// For the rows the partition sort could not take (mode 3: values piled on a few levels).  Such rows are rare,
// and a launch cannot be skipped without asking the device: so this is one launch whose workgroups return at
// once unless their row is in that mode, and a workgroup that stays sorts its row alone, digit by digit,
// ping-pong between the row's two buffers - no hand-over between workgroups, no launch per digit.
// bin = 255 - digit, so that ascending bins are descending digits.  shifts: bit s set = the digit at bit 8*s
// differs between elements (the high bytes of the index field are the same in all of them).
template <int ELT>
__global__ void __launch_bounds__(256) sort_rows_kernel(u64 *buf0, u64 *buf1, const ExRowState *st, int64_t k, uint32_t shifts,
                                                        void *out_vals, int32_t *out_idx) {
    __shared__ uint32_t running[256];
    __shared__ uint32_t wcnt[4][256];
    __shared__ uint32_t wave_tot[4];
    const int r = blockIdx.x, tid = threadIdx.x;
    if (st[r].mode != 3u) return;  // uniform over the workgroup
    const int lane = tid & 63, wave = tid >> 6;
    u64 *src = buf0 + (int64_t)r * k, *dst = buf1 + (int64_t)r * k;
    for (int d = 0; d < 8; ++d) {
        if (!((shifts >> d) & 1u)) continue;
        const int shift = 8 * d;
        // count the digits
        running[tid] = 0u;
        __syncthreads();
        for (int64_t i = tid; i < k; i += 256) atomicAdd(&running[255u - ((uint32_t)(src[i] >> shift) & 255u)], 1u);
        __syncthreads();
        // running[bin] <- elements in lower bins
        const uint32_t total = running[tid];
        const uint32_t incl = wave_incl_scan_u32(total);
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        uint32_t start = incl - total;
        for (int w = 0; w < wave; ++w) start += wave_tot[w];
        running[tid] = start;
#pragma unroll
        for (int w = 0; w < 4; ++w) wcnt[w][tid] = 0u;
        __syncthreads();
        // Stable scatter in rounds of 256 consecutive elements: an element's rank among equal bins of its round is
        // its rank among the lanes of its wavefront with that bin (eight ballots) plus the counts of the lower wavefronts.
        for (int64_t base = 0; base < k; base += 256) {
            const int64_t i = base + tid;
            const bool ok = i < k;
            const u64 c = ok ? src[i] : 0ull;
            const uint32_t bin = 255u - ((uint32_t)(c >> shift) & 255u);
            u64 peers = __ballot(ok);
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const u64 vote = __ballot((bin >> bit) & 1u);
                peers &= ((bin >> bit) & 1u) ? vote : ~vote;
            }
            const uint32_t rank_in_wave =
                __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u));
            if (ok && rank_in_wave == 0) wcnt[wave][bin] = (uint32_t)__popcll(peers);
            __syncthreads();
            if (ok) {
                uint32_t pos = running[bin] + rank_in_wave;
                for (int w = 0; w < wave; ++w) pos += wcnt[w][bin];
                dst[pos] = c;
            }
            __syncthreads();
            running[tid] += wcnt[0][tid] + wcnt[1][tid] + wcnt[2][tid] + wcnt[3][tid];
#pragma unroll
            for (int w = 0; w < 4; ++w) wcnt[w][tid] = 0u;
            __syncthreads();
        }
        u64 *t = src;
        src = dst;
        dst = t;
        __syncthreads();  // this workgroup's writes to the new source are visible to its own reads (same CU)
    }
    for (int64_t i = tid; i < k; i += 256) write_composite<ELT>(src[i], out_vals, out_idx, (int64_t)r * k + i);
}

// A kernel that is about to be launched with more dynamic LDS than a launch may ask for by default is
// told so, once per device (told: that kernel's own flags).
static hipError_t allow_whole_cu_lds(const void *kernel, bool (&told)[64]) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && told[dev]) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudgetWholeRow);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64) told[dev] = true;
    return hipSuccess;
}

template <int ELT>
static hipError_t launch_exact_t(const ExactPlan &pl, const void *x, const int32_t *xi, void *out_vals, int32_t *out_idx,
                                 void *state, void *data, hipStream_t stream) {
    const int64_t m = pl.m, n = pl.n, k = pl.k;
    if (pl.single_wg) {
        int small_bits = 1;
        while (((int64_t)1 << small_bits) < pl.idx_n) ++small_bits;
        if (pl.lds_bytes > 64 * 1024) {
            static bool told[64] = {};
            const hipError_t ea = allow_whole_cu_lds((const void *)exact_small_kernel<ELT>, told);
            if (ea != hipSuccess) return ea;
        }
        hipLaunchKernelGGL(exact_small_kernel<ELT>, dim3((unsigned)m), dim3(pl.T), (size_t)pl.lds_bytes, stream, x, xi, (int)n,
                           (int)k, small_bits, out_vals, out_idx);
        return hipGetLastError();
    }
    uint32_t *ghist = (uint32_t *)state;
    ExRowState *st = (ExRowState *)data;
    const int64_t st_bytes = ceil_div64(m * (int64_t)sizeof(ExRowState), 256) * 256;
    u64 *sel = (u64 *)((unsigned char *)data + st_bytes);
    const dim3 sweep((unsigned)pl.chunks, (unsigned)m);

    // Small k: after the first digit most rows have only a handful of elements left in play; those
    // are copied out in one more sweep and finished in LDS instead of being swept digit by digit.
    int idx_bits = 1;  // column indices are below 2^idx_bits
    while (((int64_t)1 << idx_bits) < pl.idx_n) ++idx_bits;
    // One pass of the digit descent over every `stride`-th chunk of the rows; small launches let the
    // row's last workgroup decide, big ones take a launch of their own for it.
    // few: a pass with little to do (a sample of the rows; most rows finished): as many chunks per workgroup
    // as keep it a launch of the first kind
    Squeeze sq;
    sq.drop = ELT == ATK_BF16 ? 16 : 0;
    sq.keep = idx_bits + 1;  // the index field: 0x7fffffff - idx, then the zero-sign flag
    const int sq_bits = 32 - sq.drop + sq.keep;                    // bits the descent has to decide
    const int n_passes = (sq_bits + kExDigit - 1) / kExDigit;      // 2..6; digits of 11 bits from the top, the last one narrower
    auto digit_shift = [&](int p) { return p == n_passes - 1 ? 0 : sq_bits - kExDigit * (p + 1); };
    auto digit_width = [&](int p) { return p == n_passes - 1 ? sq_bits - kExDigit * (n_passes - 1) : kExDigit; };
    auto pass = [&](int p, bool first, uint32_t fcap, int elems, int stride, bool few) {
        const int last = p == n_passes - 1 ? 1 : 0;
        const int64_t per_row = ceil_div64(n, (int64_t)elems * stride);
        const int runs = few ? (int)ceil_div64(per_row * m, kExFusedMaxWgs) : 1;
        const dim3 grid((unsigned)ceil_div64(per_row, runs), (unsigned)m);
        const bool fused = (int64_t)grid.x * m <= kExFusedMaxWgs;
#define ATK_HIST(FIRST, FUSED)                                                                                             \
    hipLaunchKernelGGL((ex_hist_kernel<ELT, FIRST, FUSED>), grid, dim3(kMaxThreads), 0, stream, x, xi, n, st, ghist,        \
                       digit_shift(p), digit_width(p), last, fcap, (uint32_t)k, elems, stride, runs, sq)
        if (fused) {
            if (first) ATK_HIST(true, true);
            else ATK_HIST(false, true);
        } else {
            if (first) {
                ATK_HIST(true, false);
                hipLaunchKernelGGL(ex_decide_kernel<true>, dim3((unsigned)m), dim3(256), 0, stream, st, ghist, digit_shift(p), last,
                                   fcap, (uint32_t)k);
            } else {
                ATK_HIST(false, false);
                hipLaunchKernelGGL(ex_decide_kernel<false>, dim3((unsigned)m), dim3(256), 0, stream, st, ghist, digit_shift(p),
                                   last, fcap, (uint32_t)k);
            }
        }
#undef ATK_HIST
    };
    auto copy_out = [&]() {  // rows in mode 1: everything at or above their threshold so far, selected in LDS
        u64 *fbuf = sel + m * k;
        hipLaunchKernelGGL((ex_collect_kernel<ELT, true, 2048>), sweep, dim3(kMaxThreads), 0, stream, x, xi, n, st, fbuf,
                           (int64_t)pl.filter_cap, pl.chunk_elems, sq);
        const size_t flds = (size_t)select_lds_bytes(pl.filter_cap, (int)pow2_ceil64(k));
        hipLaunchKernelGGL(ex_filter_select_kernel<ELT>, dim3((unsigned)m), dim3(kMaxThreads), flds, stream, fbuf, st, (int)k,
                           idx_bits, pl.filter_cap, out_vals, out_idx);
    };
    if (pl.filter && select_lds_bytes(pl.filter_cap, (int)pow2_ceil64(k)) > 64 * 1024) {
        static bool told[64] = {};
        const hipError_t ea = allow_whole_cu_lds((const void *)ex_filter_select_kernel<ELT>, told);
        if (ea != hipSuccess) return ea;
    }
    // Very small k on big inputs: the k-th largest of a sample (every 16th run of 4096 elements), to
    // two digits, is a threshold that at least k elements of the row reach, and about 16 k of them on
    // data without order along the row: one sweep copies them out, instead of one sweep to count the
    // first digit and one to copy.  A row where more than the buffer holds reach it starts over below; the
    // passes below then mostly find nothing to do, so they are launches of few workgroups, each with many chunks.
    const bool sample = pl.sample;
    if (sample) {
        pass(0, true, kSampledPass, kSampleChunk, sample_stride(k), true);
        pass(1, false, kSampledLast, kSampleChunk, sample_stride(k), true);
        copy_out();
    }
    // (Not with few rows: when every row is open - values piled up on few levels - each hangs on one workgroup, and the
    // sweeps by the whole chip below are several times faster: 16 x 2^18 on three levels, k = 64: 77 us against 502.
    // With 128 such rows the one launch loses by half; with 1024 it wins.)
    if (pl.filter && !sample && k <= kSortLdsMaxK && n <= kRestMaxRow && m >= 64) {
        // first digit, copy-out path, and one launch for whatever rows are left
        pass(0, true, (uint32_t)pl.filter_cap, pl.chunk_elems, 1, false);
        copy_out();
        const size_t lds = (size_t)pow2_ceil64(k) * 8 + kRankMax * 4;
        hipLaunchKernelGGL(ex_rest_kernel<ELT>, dim3((unsigned)m), dim3(kMaxThreads), lds, stream, x, xi, n, st, (int)k, sq_bits,
                           n_passes, pl.chunk_elems, sq, out_vals, out_idx);
        return hipGetLastError();
    }
    for (int p = 0; p < n_passes; ++p) {
        const bool filter_now = p == 0 && pl.filter && !sample;
        pass(p, p == 0 && !sample, filter_now ? (uint32_t)pl.filter_cap : 0u, pl.chunk_elems, 1, sample);
        if (filter_now) copy_out();
    }
    if (k * pl.chunk_elems / n <= 1536)  // expected survivors per chunk
        hipLaunchKernelGGL((ex_collect_kernel<ELT, false, 2048>), sweep, dim3(kMaxThreads), 0, stream, x, xi, n, st, sel, k, pl.chunk_elems, sq);
    else
        hipLaunchKernelGGL((ex_collect_kernel<ELT, false, 6144>), sweep, dim3(kMaxThreads), 0, stream, x, xi, n, st, sel, k, pl.chunk_elems, sq);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    if (k <= kSortLdsMaxK) {
        const size_t lds = (size_t)pow2_ceil64(k) * 8 + kRankMax * 4;
        hipLaunchKernelGGL(ex_order_lds_kernel<ELT>, dim3((unsigned)m), dim3(kMaxThreads), lds, stream, sel, st, (int)k,
                           out_vals, out_idx);
        return hipGetLastError();
    }
    u64 *bufs[2] = {sel, sel + m * k};
    uint32_t *tile_hist = (uint32_t *)(bufs[1] + m * k);
    const int tiles = (int)ceil_div64(k, kSortTile);  // (the area behind the buffers, sized in tiles, holds the partition sort's tables)
    // partition sort: about 128 survivors per bin
    {
        int nb = 16;
        while (nb < kPartMaxBins && (int64_t)nb * 128 < k) nb <<= 1;
        uint32_t *big = tile_hist + m * (int64_t)tiles * 256;  // [0] count, [1..] listed bins
        uint32_t *counts = big + 64 + m * (int64_t)nb;
        uint32_t *starts = counts + m * (int64_t)nb;
        uint32_t *cursors = starts + m * (int64_t)nb;
        const int ptiles = (int)ceil_div64(k, kPartTile);
        const int64_t total_bins = m * (int64_t)nb;
        // the list's counter and the counts start from zero (a fill kernel, so that the call can be captured in a graph)
        hipLaunchKernelGGL(part_zero_kernel, dim3((unsigned)ceil_div64(64 + 2 * total_bins, 256)), dim3(256), 0, stream, big,
                           64 + 2 * total_bins);
        hipLaunchKernelGGL(part_hist_kernel, dim3((unsigned)ptiles, (unsigned)m), dim3(256), 0, stream, sel, st, k, nb, counts,
                           sq);
        hipLaunchKernelGGL(part_scan_kernel, dim3((unsigned)m), dim3(256), 0, stream, st, nb, counts, starts, cursors, big);
        hipLaunchKernelGGL(part_scatter_kernel, dim3((unsigned)ptiles, (unsigned)m), dim3(256), 0, stream, sel, bufs[1], st, k,
                           nb, starts, cursors, sq);
        hipLaunchKernelGGL(part_sort_small_kernel<ELT>, dim3((unsigned)ceil_div64(total_bins, 4)), dim3(256), 0, stream,
                           bufs[1], st, k, nb, total_bins, counts, starts, big, sq, out_vals, out_idx);
        hipLaunchKernelGGL(part_sort_big_kernel<ELT>, dim3(1024), dim3(256), 0, stream, bufs[1], st, k, nb, counts, starts,
                           big, out_vals, out_idx);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // rows the partition sort could not take (mode 3): one launch, a workgroup per such row; digits that are the same
    // for every element (high bytes of the index field) are skipped
    // (the index field holds 0x7fffffff - idx in bits [31:1]; bit 0 is the zero-sign flag)
    uint32_t shifts = 0;
    for (int shift = 0; shift < 64; shift += 8)
        if (!(shift < 32 && shift >= idx_bits + 1)) shifts |= 1u << (shift / 8);
    hipLaunchKernelGGL(sort_rows_kernel<ELT>, dim3((unsigned)m), dim3(256), 0, stream, bufs[0], bufs[1], st, k, shifts, out_vals,
                       out_idx);
    return hipGetLastError();
}

hipError_t launch_exact(const ExactPlan &pl, const void *x, const int32_t *xi, void *out_vals, int32_t *out_idx,
                        void *state, void *data, hipStream_t stream) {
    if (pl.dtype == ATK_F32) return launch_exact_t<ATK_F32>(pl, x, xi, out_vals, out_idx, state, data, stream);
    return launch_exact_t<ATK_BF16>(pl, x, xi, out_vals, out_idx, state, data, stream);
}

}  // namespace atk
