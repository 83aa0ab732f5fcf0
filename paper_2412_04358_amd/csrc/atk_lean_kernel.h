// The k_b = 1 kernels of approx_topk for rows of whole, aligned 16-byte vectors (Section 2, Stage 1 with one
// survivor per bucket + Stage 2; Appendix A.1, interleaved buckets): the shapes of the paper's headline
// sweep (Figure 1 left), kept apart from the general kernel so that nothing but their own code shapes
// the schedule of the streaming loop.
//
// A row is an L x b matrix; a lane owns V adjacent columns (one 16-byte load per matrix row), P lanes
// (row phases) share a column group and walk the matrix rows ph, ph + P, ...  Every lane keeps the running
// maximum of its columns.  At the end the lanes of a column meet in LDS by atomic maximum on the composite
// word - the merge of Appendix A's per-thread queues for queues of one slot - straight into the candidate
// array, and the range of the value keys that Stage 2 spreads its bins over is folded into the same
// step, before the workgroup's one barrier.
//
// Three shapes of launch:
//   kLeanOut    no Stage 2 (b*k_b = k): a workgroup owns a block of columns of one row and writes its maxima.
//   kLeanSelect Stage 2, one workgroup per row.
//   kLeanPair   Stage 2, two workgroups per row on different CUs.  A workgroup of 512 lanes cannot pull a
//               row through one CU as fast as memory delivers (measured: 128 CUs end their rows 1.1 us after
//               256 CUs end half rows), and a symmetric hand-over (lists out, acknowledgement, ticket, lists in)
//               costs what the second CU saves.  So the pair is asymmetric: the helper (blockIdx < m) takes the
//               first, smaller share of the matrix rows, leaves its b maxima in a mailbox in memory and exits;
//               the finisher takes the rest, then reads the mailbox - whose words are their own flags: a
//               composite is never 0 - and carries on.  The helper is done before the finisher needs it, so the
//               hand-over adds one read of the mailbox to the finisher's path and nothing else.  The finisher
//               leaves the mailbox zeroed for the next call.  A finisher only ever waits for a workgroup with a
//               lower index, which is dispatched before it and waits for nobody; the wait is bounded all the
//               same, and a finisher that gives up marks its row (index -1 in every output slot).
//   kLeanMulti  the same with several helpers per finisher, for few long rows: workgroup w of a row (and column block)
//               takes the w-th share of the matrix rows, the last one is the finisher and reads one mailbox per
//               helper.  With or without Stage 2.  (Kernels of their own: the pair keeps its code.)
#pragma once
#include <cstring>

#include "atk_common.h"
#include "atk_select.h"
#include "atk_stream.h"

namespace atk {

struct LeanParams {
    const void *x;
    void *out_vals;
    int32_t *out_idx;
    u64 *mail;            // kLeanPair: [row][slot] composites, zero between calls
    int64_t n;
    int b, L, G, Gw, P, colblocks;
    int gw_shift, cb_shift;
    int k, idx_bits;
    int m;                // rows
    int Lh;               // kLeanPair: matrix rows [0, Lh) are the helper's; kLeanMulti: matrix rows per helper
    int H;                // kLeanMulti: helpers per finisher
    int spin_limit;       // kLeanPair: polls of the mailbox before the finisher gives up
    int bound_ok;         // the lower bound on the smallest candidate's key that comes with the merge is tight enough
    u64 *trace;
};

enum { kLeanOut = 0, kLeanSelect = 1, kLeanPair = 2, kLeanMulti = 3 };
constexpr int kFormOut = 8;  // value of NS in a pair without Stage 2 (b*k_b = k): the finisher writes the row of maxima
constexpr int kLeanU = 8;  // loads in flight per lane

// NS, BINNED: the form of Stage 2, fixed by the host so that a kernel holds the code of one form only (all of them
// in one kernel make 60 KB of code, of which a call runs a few KB, and the tail after the last load - a chain of
// dependent steps through code that no wavefront has run yet in this launch - is as fast as its instructions arrive):
// NS candidates per lane in registers (1, 2 or 4; b <= NS * blockDim.x), selected by bins with the key range that
// comes out of the merge (BINNED) or with a range found from the merged candidates; NS = 0: digit by digit.
template <int ELT, int MODE, int NS, bool BINNED, bool TR>
__global__ void __launch_bounds__(512) lean_kernel(LeanParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int ES = (ELT == ATK_F32) ? 4 : 2;
    constexpr int V = 16 / ES;
    constexpr int U = kLeanU;
    trace_mark<TR>(p.trace, 0);
    const int tid = threadIdx.x, T = blockDim.x;
    int r, cb = 0, ph, cgl, w = 0;
    bool helper = false;
    constexpr bool shared_row = MODE == kLeanPair || MODE == kLeanMulti;  // workgroups hand maxima over through memory
    if (MODE == kLeanPair) {
        helper = (int)blockIdx.x < p.m;
        r = helper ? (int)blockIdx.x : (int)blockIdx.x - p.m;
    } else if (MODE == kLeanMulti) {
        // helpers first (lower indices are dispatched first): share w of (row, column block) rc
        const int per = p.m * p.colblocks;
        w = (int)blockIdx.x / per;
        const int rc = (int)blockIdx.x - w * per;
        helper = w < p.H;
        divmod(rc, p.colblocks, p.cb_shift, r, cb);
    } else {
        divmod((int)blockIdx.x, p.colblocks, p.cb_shift, r, cb);
    }
    divmod(tid, p.Gw, p.gw_shift, ph, cgl);
    const int cg = cb * p.Gw + cgl;
    const bool active = ph < p.P && cg < p.G;
    const int col0 = cg * V;
    const int colbase = cb * p.Gw * V;
    const int wcols = min(p.Gw * V, p.b - colbase);  // columns of this workgroup
    const int t_lo = MODE == kLeanMulti ? w * p.Lh : ((MODE == kLeanPair && !helper) ? p.Lh : 0);
    const int t_hi = MODE == kLeanMulti ? (helper ? (w + 1) * p.Lh : p.L) : ((MODE == kLeanPair && helper) ? p.Lh : p.L);

    u64 *cand = (u64 *)(smem + 16);
    constexpr bool binned = MODE != kLeanOut && BINNED;
    // the candidate array and the counts of Stage 2's histogram start from zero
    for (int i = tid; i < wcols; i += T) cand[i] = 0ull;
    if (tid == 0) *(uint32_t *)(smem + 4) = 0u;
    if (MODE != kLeanOut && !helper && binned) {
        uint32_t *cnt = binned_cnt(cand, wcols), *misc = binned_misc(cand, wcols);
        for (int i = tid; i < (1 << binned_lg_bins(wcols)); i += T) cnt[i] = 0u;
        // [0] overflow flag, [1] and [4] lower bounds on the smallest candidate's key, [2] largest key
        // (pairs wider than a wavefront: [4] is a minimum too, see below)
        if (tid < 8) misc[tid] = (tid == 1 || (tid == 4 && shared_row && p.Gw > kWave)) ? 0xffffffffu : 0u;
    }
    __syncthreads();

    // ---------------------------------------------------------------- streaming scan: running maximum per column
    float val[V];
    int tt[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        val[e] = __uint_as_float(0x7fc00000u);  // "!(x <= NaN)" is true: the first element always enters
        tt[e] = kEmptyT;
    }
    if (active) {
        const unsigned char *base = (const unsigned char *)p.x + ((int64_t)r * p.n + col0) * ES;
        const int64_t row_bytes = (int64_t)p.b * ES;
        const int step = p.P;
        int t = t_lo + ph;
        auto feed = [&](const RowVec<ELT, V> &v, int row) {
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float x = __uint_as_float(elem_bits<ELT, V>(v, e));
                const bool c = !(x <= val[e]);  // ">" for numbers: equal values never displace earlier (lower-index) ones
                val[e] = c ? x : val[e];
                tt[e] = c ? row : tt[e];
            }
        };
        for (; t + (U - 1) * step < t_hi; t += U * step) {
            RowVec<ELT, V> v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = load_vec<ELT, V>(base + (int64_t)(t + u * step) * row_bytes);
#pragma unroll
            for (int u = 0; u < U; ++u) feed(v[u], t + u * step);
        }
        if (t < t_hi) {
            // fewer than U rows left: one more batch whose loads past the end re-read row t (a row fed twice changes
            // nothing for a running maximum), all issued together - one memory latency, not one per row
            const int nr = (t_hi - t + step - 1) / step;
            if (nr > U / 2) {
                RowVec<ELT, V> v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int tu = t + u * step;
                    v[u] = load_vec<ELT, V>(base + (int64_t)(tu < t_hi ? tu : t) * row_bytes);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int tu = t + u * step;
                    feed(v[u], tu < t_hi ? tu : t);
                }
            } else {
                RowVec<ELT, V> v[U / 2];
#pragma unroll
                for (int u = 0; u < U / 2; ++u) {
                    const int tu = t + u * step;
                    v[u] = load_vec<ELT, V>(base + (int64_t)(tu < t_hi ? tu : t) * row_bytes);
                }
#pragma unroll
                for (int u = 0; u < U / 2; ++u) {
                    const int tu = t + u * step;
                    feed(v[u], tu < t_hi ? tu : t);
                }
            }
        }
    }
    // (Without Stage 2: nothing of what follows is scheduled among the last loads' uses.  Measured, 128 x 65536 f32,
    // b = 64: 7.56 -> 7.20 us; the kernels with Stage 2 lose 0.2 us by the same barrier.)
    if constexpr (MODE == kLeanOut) __builtin_amdgcn_sched_barrier(0);
    trace_mark<TR>(p.trace, 1);  // this wavefront's share of the row is in

    // the finisher's look at the helper's mailbox
    u64 cm[kBkSlots];  // slots tid, tid + T, ... (the host sends at most kBkSlots * T buckets this way)
    auto look = [&]() {
        const u64 *mail = p.mail + (int64_t)r * p.b;
#pragma unroll
        for (int q = 0; q < kBkSlots; ++q) {  // all loads in flight together
            const int i = tid + q * T;
            cm[q] = 1ull;
            if (q * T < wcols)  // (the same for every lane)
                cm[q] = __hip_atomic_load(&mail[i < wcols ? i : 0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    // ---------------------------------------------------------------- the lanes of a column meet in LDS
    uint32_t k_own_min = 0xffffffffu, k_mail_min = 0xffffffffu, k_max = 0u;
    if (active) {
#pragma unroll
        for (int e = 0; e < V; ++e)
            if (tt[e] != kEmptyT) {
                const u64 c = make_composite(__float_as_uint(val[e]), tt[e] * p.b + col0 + e);
                // column e of column group cgl sits at e*Gw + cgl: side-by-side lanes, side-by-side words
                __hip_atomic_fetch_max(&cand[e * p.Gw + cgl], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                const uint32_t key = (uint32_t)(c >> 32);
                k_own_min = key < k_own_min ? key : k_own_min;
                k_max = key > k_max ? key : k_max;
            }
    }
    if (MODE == kLeanOut) {
        __syncthreads();
        trace_mark<TR>(p.trace, 2);
        for (int lc = tid; lc < wcols; lc += T)
            write_composite<ELT>(cand[(lc % V) * p.Gw + lc / V], p.out_vals, p.out_idx, (int64_t)r * p.k + colbase + lc);
        trace_mark<TR>(p.trace, 9);
        return;
    }
    if (MODE == kLeanPair && helper) {
        // the helper's maxima go to the mailbox, slot for slot, with agent-scope atomic stores (written through to
        // memory, not left in this XCD's L2); nothing waits for them
        __syncthreads();
        u64 *mail = p.mail + (int64_t)r * p.b;
        for (int i = tid; i < wcols; i += T) __hip_atomic_store(&mail[i], cand[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        trace_mark<TR>(p.trace, 2);
        trace_mark<TR>(p.trace, 9);
        return;
    }
    if (MODE == kLeanMulti && helper) {
        __syncthreads();
        u64 *mail = p.mail + (((int64_t)r * p.colblocks + cb) * p.H + w) * ((int64_t)p.Gw * V);
        for (int i = tid; i < wcols; i += T) __hip_atomic_store(&mail[i], cand[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    bool gave_up = false;
    if (MODE == kLeanMulti) {
        // the finisher: one mailbox per helper, side by side in memory, each Gw*V words of which wcols are used.  Up
        // to kMultiSlots words per lane are in flight together, and the host plans no more than that: a second round
        // of loads costs a second trip to memory (1.6 us each, measured), and four times the slots make enough code
        // after the last load to cost 1.5 to 3 us on launches that need a few (32 x 2^17 f32, b = 64: 6.1 -> 9.3 us).
        // Words still empty are asked for again.
        const int stride = p.Gw * V;
        u64 *mail = p.mail + ((int64_t)r * p.colblocks + cb) * p.H * (int64_t)stride;
        const int total = p.H * stride;
        constexpr int MB = kMultiSlots;
        const int mask = (stride & (stride - 1)) == 0 ? stride - 1 : 0;
        int spins = 0;
        for (int i0 = 0; i0 < total && !gave_up; i0 += MB * T) {
            u64 got[MB];
            int col[MB];
#pragma unroll
            for (int q = 0; q < MB; ++q) {
                const int i = i0 + tid + q * T;
                col[q] = i < total ? (mask ? (i & mask) : i % stride) : wcols;  // (words past a short last column block are not used)
                got[q] = col[q] < wcols ? __hip_atomic_load(&mail[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 1ull;
            }
            for (;;) {
                bool missing = false;
#pragma unroll
                for (int q = 0; q < MB; ++q) missing = missing || got[q] == 0ull;
                if (__ballot(missing) == 0ull) break;
                if (++spins >= p.spin_limit) {
                    gave_up = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
#pragma unroll
                for (int q = 0; q < MB; ++q)
                    if (got[q] == 0ull)
                        got[q] = __hip_atomic_load(&mail[i0 + tid + q * T], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int q = 0; q < MB; ++q)
                if (col[q] < wcols && got[q] != 0ull) {
                    __hip_atomic_store(&mail[i0 + tid + q * T], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_fetch_max(&cand[col[q]], got[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    const uint32_t key = (uint32_t)(got[q] >> 32);
                    // (the first helper's maxima hold one value per column: a lower bound on the smallest candidate;
                    // the minimum over all helpers' would be a looser one)
                    if (i0 + tid + q * T < stride) k_mail_min = key < k_mail_min ? key : k_mail_min;
                    k_max = key > k_max ? key : k_max;
                }
        }
    }
    if (MODE == kLeanPair) {
        // the finisher: the helper's maxima, slot for slot (every slot holds a composite, and a composite is never 0)
        // (A first look issued before this wavefront's own maxima go to LDS, to hide its latency, measured slower:
        // it comes back empty more often than not, and the second look then starts later than a single late one.)
        u64 *mail = p.mail + (int64_t)r * p.b;
        look();
        for (int spins = 0;;) {
            bool missing = false;
#pragma unroll
            for (int q = 0; q < kBkSlots; ++q) missing = missing || (tid + q * T < wcols && cm[q] == 0ull);
            if (__ballot(missing) == 0ull) break;
            if (++spins >= p.spin_limit) {
                gave_up = true;
                break;
            }
            __builtin_amdgcn_s_sleep(2);
            look();
        }
#pragma unroll
        for (int q = 0; q < kBkSlots; ++q) {
            const int i = tid + q * T;
            if (i < wcols && cm[q] != 0ull) {
                __hip_atomic_store(&mail[i], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
                __hip_atomic_fetch_max(&cand[i], cm[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                const uint32_t key = (uint32_t)(cm[q] >> 32);
                k_mail_min = key < k_mail_min ? key : k_mail_min;
                k_max = key > k_max ? key : k_max;
            }
        }
        trace_mark<TR>(p.trace, 11);  // the helper's maxima are in
    }
    if (binned) {
        // Range of the value keys that Stage 2 spreads its bins over.  The largest of the lanes' maxima is the largest
        // candidate.  The smallest candidate is bounded from below by the minimum over any set of values that holds,
        // for every column, one that the column's maximum is not below: the helper's mailbox (pairs); else all
        // lanes' maxima, and - tighter - those of a fully active wavefront when a workgroup row of lanes is at most
        // a wavefront long.  (The host keeps launches whose only bound would be loose - lanes that see few rows may
        // hold small or negative values, whose keys lie far below the candidates' - off this path.)
        uint32_t *misc = binned_misc(cand, wcols);
        // In a pair two bounds are taken and the larger is used: the smallest of the helper's maxima, and one from the
        // finisher's own lanes - the cover bound where a wavefront covers the row's columns, else the smallest of all
        // its lanes' maxima (every column's candidate is at least each of its lanes' maxima; every finisher has lanes
        // that have seen a matrix row, so that minimum is always set).  On rows with a trend - sorted rows - one share
        // lies far from the other, and either bound alone stretches the bins for one direction of the trend.
        constexpr bool pair = shared_row;
        const bool wide = p.Gw > kWave;
        const uint32_t w_own = wave_min_u32(k_own_min);
        const uint32_t w_mail = pair ? wave_min_u32(k_mail_min) : 0u;
        const uint32_t w_max = wave_max_u32(k_max);
        const bool cover = !wide && __ballot(active) == ~0ull;
        if ((tid & (kWave - 1)) == 0) {
            atomicMin(&misc[1], pair ? w_mail : w_own);
            atomicMax(&misc[2], w_max);
            if (cover) atomicMax(&misc[4], w_own);
            if (pair && wide) atomicMin(&misc[4], w_own);
        }
    }
    trace_mark<TR>(p.trace, 2);  // this wavefront's maxima are in LDS
    if (shared_row) {
        // (one word of LDS in front of the candidates: did any wavefront give up waiting)
        if (gave_up && (tid & (kWave - 1)) == 0) *(volatile uint32_t *)(smem + 4) = 1u;
    }
    __syncthreads();
    trace_mark<TR>(p.trace, 3);  // all candidates of the row are in LDS, their key range is known
    if constexpr (NS == kFormOut) {
        for (int lc = tid; lc < wcols; lc += T)
            write_composite<ELT>(cand[(lc % V) * p.Gw + lc / V], p.out_vals, p.out_idx, (int64_t)r * p.k + colbase + lc);
    } else if constexpr (NS == 0)
        select_radix_write<ELT>(cand, wcols, p.k, p.out_vals, p.out_idx, (int64_t)r);
    else if constexpr (binned)
        select_binned_ns<ELT, NS, TR>(cand, wcols, p.k, p.idx_bits, p.out_vals, p.out_idx, (int64_t)r, p.trace);
    else
        select_bucket_rank<ELT, NS, TR>(cand, wcols, p.k, p.idx_bits, p.out_vals, p.out_idx, (int64_t)r, p.trace);
    trace_mark<TR>(p.trace, 8);
    if (shared_row) {
        if (*(volatile uint32_t *)(smem + 4) != 0u) {
            __syncthreads();  // the selection's own writes are issued
            if constexpr (NS == kFormOut) {  // (this workgroup's columns)
                for (int i = tid; i < wcols; i += T) p.out_idx[(int64_t)r * p.k + colbase + i] = -1;
            } else {
                for (int i = tid; i < p.k; i += T) p.out_idx[(int64_t)r * p.k + i] = -1;
            }
        }
    }
    trace_mark<TR>(p.trace, 9);
}

static int log2_exact_lean(int v) {
    if (v < 1 || (v & (v - 1))) return -1;
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

template <int ELT, int MODE, int NS, bool BINNED>
static hipError_t launch_lean_form(const Plan &pl, const LeanParams &prm, hipStream_t stream) {
    const unsigned grid = (unsigned)pl.grid;
    if (prm.trace)
        hipLaunchKernelGGL((lean_kernel<ELT, MODE, NS, BINNED, true>), dim3(grid), dim3((unsigned)pl.T), (size_t)pl.lds_bytes, stream, prm);
    else
        hipLaunchKernelGGL((lean_kernel<ELT, MODE, NS, BINNED, false>), dim3(grid), dim3((unsigned)pl.T), (size_t)pl.lds_bytes, stream, prm);
    return hipGetLastError();
}

template <int ELT, int MODE>
static hipError_t launch_lean_mode(const Plan &pl, const LeanParams &prm, hipStream_t stream) {
    if constexpr (MODE == kLeanOut) {
        return launch_lean_form<ELT, MODE, 0, false>(pl, prm, stream);
    } else {
        if constexpr (MODE == kLeanPair || MODE == kLeanMulti)
            if (!pl.stage2) return launch_lean_form<ELT, MODE, kFormOut, false>(pl, prm, stream);
        // Stage 2 over the b candidates of the row (one column block): candidates per lane, and whether the merge's
        // key range serves the bins
        const int64_t per_lane = (pl.b + pl.T - 1) / pl.T;
        if (per_lane > kBkSlots) return launch_lean_form<ELT, MODE, 0, false>(pl, prm, stream);
        const bool binned = pl.bound_ok != 0;
        if (per_lane <= 1) return binned ? launch_lean_form<ELT, MODE, 1, true>(pl, prm, stream) : launch_lean_form<ELT, MODE, 1, false>(pl, prm, stream);
        if (per_lane <= 2) return binned ? launch_lean_form<ELT, MODE, 2, true>(pl, prm, stream) : launch_lean_form<ELT, MODE, 2, false>(pl, prm, stream);
        return binned ? launch_lean_form<ELT, MODE, kBkSlots, true>(pl, prm, stream)
                      : launch_lean_form<ELT, MODE, kBkSlots, false>(pl, prm, stream);
    }
}

// kLeanMulti's kernels, in a source file of their own (atk_multi.hip: the code object of the other three shapes of launch
// stays as it is when these change - their timing moves by some tenths of a microsecond with where their code lies)
hipError_t launch_lean_multi(const Plan &pl, const LeanParams &prm, hipStream_t stream);

}  // namespace atk
