// Fused kernel of approx_topk: Stage 1 (per-bucket top-k_b), the merges needed when one
// bucket is spread over several lanes / workgroups, and Stage 2 (exact top-k of the
// b*k_b candidates) when b*k_b > k.   Section 2 and Appendix A of arxiv 2412.04358.
//
// Mapping.  Bucket j of a row holds the elements i = j (mod b) (Appendix A.1), so the row
// is an L x b row-major matrix whose column j is bucket j.  A lane owns V adjacent columns
// (one 16-byte load per matrix row) and keeps, per column, the k_b largest elements seen
// so far in registers ("a max priority queue of size k_b ... in per-thread registers",
// Appendix A).  Lanes side by side read consecutive addresses, so the interleaved layout
// costs nothing.  When b is small, several lanes (row phases) share a column group, and
// when m*b is too small to fill the chip, several workgroups (row splits) do; their sorted
// lists are merged once at the end (Appendix A, mode (2): "merge the per-thread queues
// once"), first in LDS, then - across workgroups - by whichever workgroup of the row
// finishes last (a ticket counter), which also runs Stage 2.
#include <cstdlib>
#include <cstring>

#include <type_traits>

#include "atk_common.h"
#include "atk_select.h"
#include "atk_stream.h"

namespace atk {

struct S1Params {
    const void *x;
    void *out_vals;
    int32_t *out_idx;
    u64 *lists;          // scratch: [row][split][column][k_b] composites
    uint32_t *tickets;   // scratch: one counter per row (kTicketStride words apart), zero between calls
    int64_t n;
    int b, L, G, Gw, P, colblocks, S, rows_per_split;
    int rem, extra_ph;   // n mod b, and the row phase that takes the ragged last matrix row
    int idx_bits;        // column indices are below 2^idx_bits
    int k, k_b;
    int stage2, direct, use_scratch, vec_store;
    int wave_merge;      // Gw < 64 and a power of two: lanes of one wavefront share columns
    int nparts;          // partial lists per column left after the wavefront merge
    int lds_xch_off, lds_cand_off;  // byte offsets of the exchange and candidate areas in LDS
    int cb_shift, s_shift, gw_shift;  // log2 of colblocks, S, Gw when those are powers of two, else -1
    int tail_tpc_shift;  // log2 of the lanes that share a column in the last workgroup's merge
    int wgs_per_ticket;  // workgroups that share a ticket: a row's (Stage 2), else a column block's row splits
    // contiguous assignment only
    int Gs, gs_shift;    // lanes per bucket (a power of two) and its log2
    int bblocks;         // workgroups side by side across the b buckets
    int chunks_per_split;
    int NB;              // short buckets: buckets a lane group takes in turn (0: one bucket per group)
    int lds_max;         // k_b = 1, no scratch: the lanes' running maxima meet in LDS by atomic maximum (see the kernel)
    int bound_ok;        // ... and the lower bound on the smallest candidate that comes with that merge is tight enough for select_binned()
    int refresh;         // eight unpacked slots: the lanes of a column pool their queues' floors after this many load batches, then twice as many, ... (0: never)
    u64 *trace;          // measurement build only: phase timestamps, [workgroup][wavefront][phase]
};

// Insert (v, t) into the descending list (val, tt); later elements never displace equal
// earlier ones ("!(v <= slot)" is "v > slot" for numbers and true for the NaN that marks
// an empty slot).
template <int KB>
__device__ __forceinline__ void insert(float (&val)[KB], int (&tt)[KB], float v, int t) {
    bool c[KB];
#pragma unroll
    for (int j = 0; j < KB; ++j) c[j] = !(v <= val[j]);
#pragma unroll
    for (int j = KB - 1; j >= 1; --j) {
        val[j] = c[j - 1] ? val[j - 1] : (c[j] ? v : val[j]);
        tt[j] = c[j - 1] ? tt[j - 1] : (c[j] ? t : tt[j]);
    }
    val[0] = c[0] ? v : val[0];
    tt[0] = c[0] ? t : tt[0];
}

// ---- batch scan for long queues (k_b > 8) -------------------------------------------------------------------------
// Inserting element by element costs about five lane operations per slot and element.  Where most elements enter
// the queue (short buckets: the top quarter of every bucket is kept when b*k_b = k = n/4) it is cheaper to take
// k_b matrix rows at a time, sort them with a network, and fold the sorted batch into the queue with the
// bitonic merge that also joins the lanes' queues: about 3.3 lane operations per slot and element.  A network has no
// notion of "earlier element wins ties", so the queues hold words that are distinct: [63:32] the value's order
// key, [31:1] 0x7fffffff - matrix row, [0] "was -0" (the composite word with the row in place of the column index).
__device__ __forceinline__ u64 row_word(uint32_t bits, int t) {
    return ((u64)ukey_of_bits(bits) << 32) | ((0x7fffffffu - (uint32_t)t) << 1) | (bits == 0x80000000u ? 1u : 0u);
}
// Batcher's odd-even merge sort of N words, largest first (N a power of two; 19 compare-exchanges for 8, 63 for 16).
template <int N>
__device__ __forceinline__ void sort_desc(u64 (&a)[N]) {
#pragma unroll
    for (int p = 1; p < N; p *= 2)
#pragma unroll
        for (int k = p; k >= 1; k /= 2)
#pragma unroll
            for (int j = k % p; j + k < N; j += 2 * k)
#pragma unroll
                for (int i = 0; i < k; ++i)
                    if (i + j + k < N && (i + j) / (2 * p) == (i + j + k) / (2 * p)) {
                        const u64 x = a[i + j], y = a[i + j + k];
                        const bool sw = y > x;
                        a[i + j] = sw ? y : x;
                        a[i + j + k] = sw ? x : y;
                    }
}
// one word into a queue sorted largest first
template <int KB>
__device__ __forceinline__ void insert_word(u64 (&q)[KB], u64 c) {
#pragma unroll
    for (int j = KB - 1; j >= 1; --j) q[j] = (c > q[j - 1]) ? q[j - 1] : (c > q[j] ? c : q[j]);
    q[0] = c > q[0] ? c : q[0];
}

// mine <- the N largest of (mine U theirs), as multisets; both sorted descending, result sorted descending.
template <int N>
__device__ __forceinline__ void merge_keys(uint32_t (&mine)[N], const uint32_t (&theirs)[N]) {
#pragma unroll
    for (int j = 0; j < N; ++j) mine[j] = max(mine[j], theirs[N - 1 - j]);
#pragma unroll
    for (int stride = N / 2; stride >= 1; stride >>= 1)
#pragma unroll
        for (int i = 0; i < N; ++i)
            if ((i & stride) == 0) {
                const uint32_t a = mine[i], c = mine[i + stride];
                mine[i] = max(a, c);
                mine[i + stride] = min(a, c);
            }
}

// Feed the V elements of one load into the lane's V queues.  With k_b > 1 the insertion costs
// about 5*k_b lane operations per element, so it is skipped whenever no lane of the wavefront
// holds an element that beats the last slot of its queue (one compare per element and a
// wavefront-uniform branch): on long buckets almost every load is rejected that way.
template <int ELT, int V, int KB, bool PER_COLUMN = false>
__device__ __forceinline__ void scan_vec(float (&val)[V][KB], int (&tt)[V][KB], const RowVec<ELT, V> &v, int t) {
    float x[V];
#pragma unroll
    for (int e = 0; e < V; ++e) x[e] = __uint_as_float(elem_bits<ELT, V>(v, e));
    if constexpr (PER_COLUMN) {
        // where insertions are rare (pooled floors) the test is made per column: a wavefront that needs the insertion
        // for one of its columns does not pay for the others
#pragma unroll
        for (int e = 0; e < V; ++e)
            if (__ballot(!(x[e] <= val[e][KB - 1])) != 0ull) insert<KB>(val[e], tt[e], x[e], t);
        return;
    }
    if (KB > 1) {
        bool any = false;
#pragma unroll
        for (int e = 0; e < V; ++e) any = any || !(x[e] <= val[e][KB - 1]);
        if (__ballot(any) == 0ull) return;
    }
#pragma unroll
    for (int e = 0; e < V; ++e) insert<KB>(val[e], tt[e], x[e], t);
}

// ---- packed queues for bf16 with k_b >= 3 -------------------------------------------------------
// A bf16 element and its matrix row fit one 32-bit word: [31:16] order-preserving key of the
// value (-0 folded onto +0), [15:1] 0x7fff - (row - first row of this lane's split), [0] "was -0".
// Larger word <=> larger value, or equal value and earlier row, so inserting into a descending
// list is one median-of-three per slot instead of compares and selects on two arrays (measured
// faster from four slots on; with two the conversion costs what it saves).  0 = empty.
__device__ __forceinline__ uint32_t pack_bf16(uint32_t xb, uint32_t tl) {  // xb: the bf16 in the high half
    const uint32_t sgn = (uint32_t)((int32_t)xb >> 31);
    const uint32_t key = xb ^ ((sgn & 0x7fff0000u) | 0x80000000u);
    return (xb == 0x80000000u) ? (0x80000001u | tl) : (key | tl);
}
__device__ __forceinline__ void unpack_bf16(uint32_t c, int t_first, float &v, int &t) {
    if (c == 0u) {
        v = __uint_as_float(0x7fc00000u);
        t = kEmptyT;
        return;
    }
    const uint32_t key = c >> 16;
    uint32_t bits = (key & 0x8000u) ? (key ^ 0x8000u) : (~key & 0xffffu);
    if (c & 1u) bits = 0x8000u;
    v = __uint_as_float(bits << 16);
    t = t_first + 0x7fff - (int)((c >> 1) & 0x7fffu);
}
__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c) {
    return max(min(a, b), min(max(a, b), c));
}
template <int KB>
__device__ __forceinline__ void insert_pk(uint32_t (&q)[KB], uint32_t c) {
#pragma unroll
    for (int j = KB - 1; j >= 1; --j) q[j] = umed3(q[j - 1], q[j], c);  // q[j-1] >= q[j]: c clamped between them
    q[0] = max(q[0], c);
}
template <int ELT, int V, int KB>
__device__ __forceinline__ void scan_vec_pk(uint32_t (&q)[V][KB], const RowVec<ELT, V> &v, int t_local) {
    const uint32_t tl = (uint32_t)(0x7fff - t_local) << 1;
    uint32_t c[V];
#pragma unroll
    for (int e = 0; e < V; ++e) c[e] = pack_bf16(elem_bits<ELT, V>(v, e), tl);
    if (KB >= 8) {  // the insertion is cheap: only long queues are worth a wavefront-uniform skip
        bool any = false;
#pragma unroll
        for (int e = 0; e < V; ++e) any = any || c[e] > q[e][KB - 1];
        if (__ballot(any) == 0ull) return;
    }
#pragma unroll
    for (int e = 0; e < V; ++e) insert_pk<KB>(q[e], c[e]);
}

// Stage-1 result of bucket `col`, as seen by row split `sp` of row r: to the scratch lists (when
// several workgroups share the row), to the candidate area in LDS (Stage 2 inside this
// workgroup), or straight to the output.
template <int ELT, int KB>
__device__ __forceinline__ void emit_list(const S1Params &p, int r, int sp, int col, const u64 (&list)[KB], u64 *cand) {
    if (p.use_scratch) {
        // agent-scope atomic stores: written through to memory, not left in this XCD's L2
        u64 *dst = p.lists + (((int64_t)r * p.S + sp) * p.b + col) * p.k_b;
#pragma unroll
        for (int j = 0; j < KB; ++j)
            if (j < p.k_b) __hip_atomic_store(&dst[j], list[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else if (p.stage2) {
#pragma unroll
        for (int j = 0; j < KB; ++j)
            if (j < p.k_b) cand[col * p.k_b + j] = list[j];
    } else {
        const int64_t o = (int64_t)r * p.k + (int64_t)col * p.k_b;
#pragma unroll
        for (int j = 0; j < KB; ++j)
            if (j < p.k_b) write_composite<ELT>(list[j], p.out_vals, p.out_idx, o + j);
    }
}

// What follows the last emit_list() of a workgroup: the hand-over between the workgroups that
// share a ticket, and Stage 2.  Every thread calls it.
// With Stage 2 the whole row shares one ticket (one workgroup must see all b*k_b candidates);
// without it every block of columns [c_lo, c_hi) has its own (ticket number `tk`), and whoever
// draws the last one merges the row splits of just those columns.  Column c of the block is
// bucket c - rot (mod b).
template <int ELT, int KB, bool TR = false>
__device__ __forceinline__ void row_tail(const S1Params &p, int r, int64_t tk, int c_lo, int c_hi, int rot,
                                         unsigned char *smem) {
    const int tid = threadIdx.x, T = blockDim.x;
    u64 *cand = (u64 *)(smem + p.lds_cand_off);
    if (!p.use_scratch) {
        if (!p.stage2) return;
        __syncthreads();
    } else {
        // ------------------------------------------------------------ ticket
        // Cross-workgroup hand-over without cache-wide fences: the lists were written, and are
        // read below, with agent-scope atomic accesses (they go through to memory instead of
        // staying in one XCD's L2, so there is nothing for a cache write-back or invalidate to do);
        // every lane waits until its own stores have been acknowledged (a barrier alone does not:
        // inside a workgroup the compiler lets global stores stay in flight across it), and only
        // after the barrier one lane takes the ticket.  Whoever draws the last one knows that every
        // other workgroup's lists are complete.  The wait is an asm statement with a memory clobber,
        // so the compiler can move neither the stores below it nor the ticket above it.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        uint32_t *flag = (uint32_t *)smem;
        uint32_t *ticket_word = p.tickets + tk * kTicketStride;
        if (tid == 0) {
            uint32_t ticket = __hip_atomic_fetch_add(ticket_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            flag[0] = (ticket == (uint32_t)(p.wgs_per_ticket - 1)) ? 1u : 0u;
        }
        __syncthreads();
        if (flag[0] == 0) return;
        trace_mark<TR>(p.trace, 10);  // drew the last ticket
        if (tid == 0)  // ready for the next call
            __hip_atomic_store(ticket_word, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

        // The last workgroup merges the splits of its columns, SU splits per batch of loads.
        constexpr int SU = tail_split_batch(KB);
        const int ncols = c_hi - c_lo;
        const u64 *src = p.lists + (int64_t)r * p.S * p.b * p.k_b;
        // The lists of NB consecutive splits from s0 on, merged into acc.  All NB loads are issued
        // before the first merge; the k_b <= KB slots that exist are loaded, the rest stay empty.
        // (Loads under a per-load condition would each sit in a branch of their own and wait for
        // one another.)
        auto batch = [&](auto nb_tag, int col, int s0, u64(&acc)[KB]) {
            constexpr int NB = decltype(nb_tag)::value;
            u64 th[NB][KB];
#pragma unroll
            for (int u = 0; u < NB; ++u)
#pragma unroll
                for (int j = 0; j < KB; ++j)
                    th[u][j] = __hip_atomic_load(&src[((int64_t)(s0 + u) * p.b + col) * p.k_b + (j < p.k_b ? j : p.k_b - 1)],
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int u = 0; u < NB; ++u) {
#pragma unroll
                for (int j = 0; j < KB; ++j)
                    if (j >= p.k_b) th[u][j] = 0ull;
                merge_topk<KB>(acc, th[u]);
            }
        };
        // lists of the splits [s0, s0 + SU) for s0 = s_first, s_first + s_step, ... of column `col`, merged
        // into acc; a batch cut short by the last split goes in pieces of 4, 2 and 1
        auto gather = [&](int col, int s_first, int s_step, u64(&acc)[KB]) {
            int s0 = s_first;
            for (; s0 + SU <= p.S; s0 += s_step) batch(std::integral_constant<int, SU>(), col, s0, acc);
            if (s0 < p.S) {  // s_step >= SU: at most one batch is cut short
                const int rem = p.S - s0;
                if (SU > 4 && (rem & 4)) {
                    batch(std::integral_constant<int, 4>(), col, s0, acc);
                    s0 += 4;
                }
                if (SU > 2 && (rem & 2)) {
                    batch(std::integral_constant<int, 2>(), col, s0, acc);
                    s0 += 2;
                }
                if (rem & 1) batch(std::integral_constant<int, 1>(), col, s0, acc);
            }
        };
        auto put = [&](int col, const u64(&acc)[KB]) {
            if (p.stage2) {
#pragma unroll
                for (int j = 0; j < KB; ++j)
                    if (j < p.k_b) cand[col * p.k_b + j] = acc[j];
            } else {
                const int64_t o = (int64_t)r * p.k + (int64_t)col * p.k_b;
#pragma unroll
                for (int j = 0; j < KB; ++j)
                    if (j < p.k_b) write_composite<ELT>(acc[j], p.out_vals, p.out_idx, o + j);
            }
        };
        if (p.tail_tpc_shift == 0) {
            // one lane per column (a plain loop: the compiler may overlap its iterations)
            for (int ci = tid; ci < ncols; ci += T) {
                u64 acc[KB];
#pragma unroll
                for (int j = 0; j < KB; ++j) acc[j] = 0ull;
                const int col = c_lo + ci - rot + (c_lo + ci < rot ? p.b : 0);
                gather(col, 0, SU, acc);
                put(col, acc);
            }
        } else {
            // Fewer columns than lanes and many splits: tpc lanes side by side share a column,
            // each merges every tpc-th batch, then a butterfly of shuffles joins them.
            const int tpc_shift = p.tail_tpc_shift, tpc = 1 << tpc_shift;  // chosen on the host: tpc * ncols <= T
            const int part = tid & (tpc - 1);
            const int ci = tid >> tpc_shift;
            const bool ok = ci < ncols;
            u64 acc[KB];
#pragma unroll
            for (int j = 0; j < KB; ++j) acc[j] = 0ull;
            const int col = c_lo + ci - rot + (c_lo + ci < rot ? p.b : 0);
            if (ok) gather(col, part * SU, tpc * SU, acc);
            for (int off = 1; off < tpc; off <<= 1) {
                u64 theirs[KB];
#pragma unroll
                for (int j = 0; j < KB; ++j) theirs[j] = shfl_xor_u64(acc[j], off);
                merge_topk<KB>(acc, theirs);
            }
            if (ok && part == 0) put(col, acc);
        }
        trace_mark<TR>(p.trace, 11);  // the other workgroups' lists are merged
        if (!p.stage2) return;
        __syncthreads();
    }

    // ---------------------------------------------------------------- Stage 2 in LDS
    trace_mark<TR>(p.trace, 3);  // all candidates of the row are in LDS
    select_write<ELT, TR>(cand, p.b * p.k_b, p.k, p.idx_bits, p.out_vals, p.out_idx, (int64_t)r, p.trace);
    trace_mark<TR>(p.trace, 8);  // outputs written
}

template <int ELT, int V, int KB, int U, int MAXT, bool PKF, bool TR = false, bool RF = false>
__global__ void __launch_bounds__(MAXT) stage1_kernel(S1Params p) {
    extern __shared__ __align__(16) unsigned char smem[];
    trace_mark<TR>(p.trace, 0);  // the wavefront has started
    constexpr int ES = (ELT == ATK_F32) ? 4 : 2;
    constexpr bool PK = PKF && ELT == ATK_BF16 && KB >= 4;  // packed 32-bit queues (host: rows per split < 32766)
    // queues of distinct 64-bit words, fed k_b matrix rows at a time: pays from sixteen slots on (128 x 65536 f32,
    // k = 16384, k_b = 16: 44.8 -> 36.0 us; with eight slots the 64-bit compares cost more than the shorter
    // network saves: 19.2 -> 21.8 us, and 164 -> 185 us on 128 x 2^20, b = 8)
    constexpr bool BATCH = KB >= 16 && !PK;
    const int tid = threadIdx.x, T = blockDim.x;
    int wg = blockIdx.x, cb, sp, r, cgl, ph;
    divmod(wg, p.colblocks, p.cb_shift, wg, cb);
    divmod(wg, p.S, p.s_shift, r, sp);
    divmod(tid, p.Gw, p.gw_shift, ph, cgl);
    const int cg = cb * p.Gw + cgl;
    const bool active = (ph < p.P) && (cg < p.G);
    const int col0 = cg * V;
    // Rows whose first element is not aligned to a V-element load (n not a multiple of V) are
    // read from the aligned address just before: the row is taken as a virtual row that starts
    // `rot` elements early, so virtual column c holds bucket c - rot (mod b) and element
    // (t, c) of the virtual matrix is column t*b + c - rot of the row.  The first `rot` virtual
    // elements belong to the previous row and are skipped.
    const int rot = (V > 1) ? (int)(((int64_t)r * p.n) & (V - 1)) : 0;
    const bool carry = p.rem + rot >= p.b;       // the virtual row has one more full matrix row
    const int Lr = p.L + (carry ? 1 : 0);       // full matrix rows of the virtual row
    const int remr = p.rem + rot - (carry ? p.b : 0);  // columns of its ragged last matrix row
    int eph = p.extra_ph + (carry ? 1 : 0);     // the row phase that takes the ragged row
    if (eph >= p.P) eph -= p.P;
    const int t0 = sp * p.rows_per_split;
    const int t1 = (sp == p.S - 1) ? Lr : min(Lr, t0 + p.rows_per_split);
    auto bucket_of = [&](int c) { return c - rot + (c < rot ? p.b : 0); };

    // One slot per bucket, no hand-over through memory: the lanes that share a column meet in LDS by
    // atomic maximum on the composite (the merge of Appendix A's per-thread queues, for queues of one
    // slot), straight into the candidate array that Stage 2 selects from.  The array - and the counts
    // of Stage 2's histogram - are cleared here, while nothing else is going on.
    if constexpr (KB == 1) {
        if (p.lds_max) {
            u64 *cand = (u64 *)(smem + p.lds_cand_off);
            const int wcols = min(p.Gw * V, p.b - cb * p.Gw * V);
            for (int i = tid; i < wcols; i += T) cand[i] = 0ull;
            if (p.stage2 && binned_fits(wcols) && p.bound_ok) {
                uint32_t *cnt = binned_cnt(cand, wcols), *misc = binned_misc(cand, wcols);
                for (int i = tid; i < (1 << binned_lg_bins(wcols)); i += T) cnt[i] = 0u;
                if (tid < 8) misc[tid] = (tid == 1) ? 0xffffffffu : 0u;  // (see select_binned: flag, range, lower bounds)
            }
            __syncthreads();
        }
    }

    float val[V][KB];
    int tt[V][KB];
    uint32_t pk[PK ? V : 1][PK ? KB : 1];
    u64 qw[BATCH ? V : 1][BATCH ? KB : 1];  // BATCH: the queues, as row words
    float last_f[BATCH ? V : 1];            // ... and the value of each queue's last slot (NaN while it is empty)
#pragma unroll
    for (int e = 0; e < V; ++e)
#pragma unroll
        for (int j = 0; j < KB; ++j) {
            val[e][j] = __uint_as_float(0x7fc00000u);
            tt[e][j] = kEmptyT;
            if constexpr (PK) pk[e][j] = 0u;
            if constexpr (BATCH) {
                qw[e][j] = 0ull;
                last_f[e] = __uint_as_float(0x7fc00000u);
            }
        }
#define ATK_FEED_ELEM(e, xb, row)                                                                    \
    do {                                                                                             \
        if constexpr (PK)                                                                            \
            insert_pk<KB>(pk[e], pack_bf16(xb, (uint32_t)(0x7fff - ((row) - t0)) << 1));             \
        else if constexpr (BATCH)                                                                    \
            insert_word<KB>(qw[e], row_word(xb, (row)));                                             \
        else                                                                                         \
            insert<KB>(val[e], tt[e], __uint_as_float(xb), (row));                                   \
    } while (0)
#define ATK_FEED_VEC(vec, row)                                                                       \
    do {                                                                                             \
        if constexpr (PK)                                                                            \
            scan_vec_pk<ELT, V, KB>(pk, vec, (row) - t0);                                            \
        else if constexpr (BATCH) {                                                                  \
            _Pragma("unroll") for (int e_ = 0; e_ < V; ++e_) ATK_FEED_ELEM(e_, (elem_bits<ELT, V>(vec, e_)), (row)); \
        } else                                                                                       \
            scan_vec<ELT, V, KB, RF>(val, tt, vec, (row));                                           \
    } while (0)

    // ---------------------------------------------------------------- pooled floors (instances of their own: RF)
    // Eight unpacked slots, several lanes of the workgroup on a column, many matrix rows per lane, rows that start on a
    // load boundary (rot = 0; the host sees to all of it).  What a lane has seen alone is a poor bound on what still
    // matters: after t rows one element in t/8 still enters its queue, and with 128 lane-columns per wavefront some
    // lane always needs the insertion.  So after `stop` load batches - the same number in every lane, and every lane
    // has at least that many - the lanes of a column pool what they hold: between them they have seen all elements of
    // a stretch of the row; the eighth best of that stretch bounds the column's final eighth best from below, and every
    // element still to come has a higher index than all of the stretch, so it has to beat that value outright.  Slots
    // below it, and empty ones, are set to it and marked empty.  The lanes pool their queues' value keys: a butterfly
    // inside the wavefront where lanes of a column sit side by side, then through the exchange area in LDS (free
    // until the lists are merged at the end).  Again after twice as many batches, and so on.
    int t_resume = t0 + ph;  // the lane's next matrix row
    if constexpr (RF) {
        static_assert(!RF || (KB == 8 && !PKF), "pooled floors: eight unpacked slots");
        const unsigned char *base = (const unsigned char *)p.x + ((int64_t)r * p.n + (int64_t)col0) * ES;
        const int64_t row_bytes = (int64_t)p.b * ES;
        const int step = p.P;
        const int nfull = ((t1 - t0) / p.P) / U;  // full batches that every row phase has
        int done = 0;
        for (int stop = p.refresh; stop > 0 && stop < nfull; stop *= 2) {
            if (active) {
                // the batches up to the stop; the next batch's loads are issued before the current one is worked on
                const int nb = stop - done;
                int t = t_resume;
                RowVec<ELT, V> v[U], w[U];
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = load_vec<ELT, V>(base + (int64_t)(t + u * step) * row_bytes);
                for (int i = 0; i < nb; ++i) {
                    const int tn = t + U * step;
                    if (i + 1 < nb) {
#pragma unroll
                        for (int u = 0; u < U; ++u) w[u] = load_vec<ELT, V>(base + (int64_t)(tn + u * step) * row_bytes);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) ATK_FEED_VEC(v[u], t + u * step);
#pragma unroll
                    for (int u = 0; u < U; ++u) v[u] = w[u];
                    t = tn;
                }
                t_resume = t;
            }
            done = stop;
            uint32_t keys[V][KB];
#pragma unroll
            for (int e = 0; e < V; ++e)
#pragma unroll
                for (int j = 0; j < KB; ++j)
                    keys[e][j] = (active && tt[e][j] != kEmptyT) ? ukey_of_bits(__float_as_uint(val[e][j])) : 0u;
            if (p.wave_merge) {
                for (int off = p.Gw; off < kWave; off <<= 1) {
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        uint32_t theirs[KB];
#pragma unroll
                        for (int j = 0; j < KB; ++j) theirs[j] = (uint32_t)__shfl_xor((int)keys[e][j], off, kWave);
                        merge_keys<KB>(keys[e], theirs);
                    }
                }
            }
            if (p.nparts > 1) {
                uint32_t *xk = (uint32_t *)(smem + p.lds_xch_off);  // [part][column of the workgroup][slot]
                const int part = p.wave_merge ? (tid >> 6) : ph;
                const bool holder = active && (!p.wave_merge || (tid & (kWave - 1)) < p.Gw);
                const int64_t pstride = (int64_t)p.Gw * V;
                if (holder) {
#pragma unroll
                    for (int e = 0; e < V; ++e)
#pragma unroll
                        for (int j = 0; j < KB; ++j) xk[((int64_t)part * pstride + cgl * V + e) * KB + j] = keys[e][j];
                }
                __syncthreads();
                if (active) {
#pragma unroll
                    for (int e = 0; e < V; ++e) {
#pragma unroll
                        for (int j = 0; j < KB; ++j) keys[e][j] = xk[((int64_t)cgl * V + e) * KB + j];
                        for (int q = 1; q < p.nparts; ++q) {
                            uint32_t theirs[KB];
#pragma unroll
                            for (int j = 0; j < KB; ++j) theirs[j] = xk[((int64_t)q * pstride + cgl * V + e) * KB + j];
                            merge_keys<KB>(keys[e], theirs);
                        }
                    }
                }
                __syncthreads();  // (the area is written again at the next stop, and by the merge at the end)
            }
            if (active) {
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const uint32_t fk = keys[e][KB - 1];
                    if (fk != 0u) {  // eight elements of the column have been seen
                        const float floor_v = __uint_as_float(bits_of_ukey(fk));
#pragma unroll
                        for (int j = 0; j < KB; ++j)
                            if (tt[e][j] == kEmptyT || val[e][j] < floor_v) {
                                val[e][j] = floor_v;
                                tt[e][j] = kEmptyT;
                            }
                    }
                }
            }
        }
    }

    // ---------------------------------------------------------------- streaming scan
    if (active) {
        const unsigned char *base = (const unsigned char *)p.x + ((int64_t)r * p.n - rot + (int64_t)col0) * ES;
        const int64_t row_bytes = (int64_t)p.b * ES;
        const int step = p.P;
        int t = t_resume;
        if (V > 1 && rot > 0 && cg == 0 && t == 0 && t < t1) {
            // the head of the virtual row: its first `rot` elements are not this row's
            RowVec<ELT, V> v = load_vec<ELT, V>(base);
#pragma unroll
            for (int e = 0; e < V; ++e)
                if (e >= rot) ATK_FEED_ELEM(e, (elem_bits<ELT, V>(v, e)), 0);
            t += step;
        }
        if constexpr (BATCH) {
            // k_b matrix rows at a time; the next batch's loads are issued before this one is worked on.  Rows past
            // the end re-read row t and are dropped.
            RowVec<ELT, V> v[KB], w[KB];
            bool have = t < t1;
            if (have) {
#pragma unroll
                for (int u = 0; u < KB; ++u) {
                    const int tu = t + u * step;
                    v[u] = load_vec<ELT, V>(base + (int64_t)(tu < t1 ? tu : t) * row_bytes);
                }
            }
            while (have) {
                const int tn = t + KB * step;
                const bool more = tn < t1;
                if (more) {
#pragma unroll
                    for (int u = 0; u < KB; ++u) {
                        const int tu = tn + u * step;
                        w[u] = load_vec<ELT, V>(base + (int64_t)(tu < t1 ? tu : tn) * row_bytes);
                    }
                }
                // one compare per element, and a wavefront-uniform skip, keep long buckets cheap: an element enters
                // only if it beats the queue's last slot (equal values never displace earlier ones)
                bool any = false;
#pragma unroll
                for (int u = 0; u < KB; ++u)
#pragma unroll
                    for (int e = 0; e < V; ++e)
                        any = any || (t + u * step < t1 && !(__uint_as_float(elem_bits<ELT, V>(v[u], e)) <= last_f[e]));
                if (__ballot(any) != 0ull) {
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        u64 bt[KB];
#pragma unroll
                        for (int u = 0; u < KB; ++u) {
                            const int tu = t + u * step;
                            bt[u] = tu < t1 ? row_word(elem_bits<ELT, V>(v[u], e), tu) : 0ull;
                        }
                        sort_desc<KB>(bt);
                        merge_topk<KB>(qw[e], bt);
                        const uint32_t lk = (uint32_t)(qw[e][KB - 1] >> 32);
                        last_f[e] = __uint_as_float(qw[e][KB - 1] ? bits_of_ukey(lk) : 0x7fc00000u);
                    }
                }
#pragma unroll
                for (int u = 0; u < KB; ++u) v[u] = w[u];
                t = tn;
                have = more;
            }
        } else if (KB == 8) {
            // The next batch's loads are issued before the current one is worked on (measured:
            // 4-7 % at eight slots, nothing or a loss at other queue lengths).
            RowVec<ELT, V> v[U], w[U];
            bool have = t + (U - 1) * step < t1;
            if (have) {
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = load_vec<ELT, V>(base + (int64_t)(t + u * step) * row_bytes);
            }
            while (have) {
                const int tn = t + U * step;
                const bool more = tn + (U - 1) * step < t1;
                if (more) {
#pragma unroll
                    for (int u = 0; u < U; ++u) w[u] = load_vec<ELT, V>(base + (int64_t)(tn + u * step) * row_bytes);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) ATK_FEED_VEC(v[u], t + u * step);
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = w[u];
                t = tn;
                have = more;
            }
        } else {
            if (KB == 1 && ELT == ATK_BF16) {
                // One pointer per lane, advanced by a batch at a time, the batch's loads at fixed strides
                // from it, and the whole batch in flight before the first row is looked at: the barrier
                // keeps the scheduler from starting on the first rows while the addresses of the last are
                // still being worked out, as it does for bf16 in the plain form below (2048 x 8192:
                // 8.6 -> 8.3 us).  For f32 and with queues the plain form schedules as well or better.
                const int64_t stride_bytes = (int64_t)step * row_bytes;
                const unsigned char *ptr = base + (int64_t)t * row_bytes;
                for (; t + (U - 1) * step < t1; t += U * step, ptr += U * stride_bytes) {
                    RowVec<ELT, V> v[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) v[u] = load_vec<ELT, V>(ptr + u * stride_bytes);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int u = 0; u < U; ++u) ATK_FEED_VEC(v[u], t + u * step);
                }
            } else {
                for (; t + (U - 1) * step < t1; t += U * step) {
                    RowVec<ELT, V> v[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) v[u] = load_vec<ELT, V>(base + (int64_t)(t + u * step) * row_bytes);
#pragma unroll
                    for (int u = 0; u < U; ++u) ATK_FEED_VEC(v[u], t + u * step);
                }
            }
        }
        if (t < t1) {
            // Fewer than U rows are left: they go in pieces of U/2, U/4, ... 1 rows, each piece's loads
            // issued together.  One row at a time, every load would wait out a full memory latency, which
            // on rows of a few batches per lane is most of the kernel (n = 128256 against 131072: +3 us).
            int nr = (t1 - t + step - 1) / step;
            if (KB == 1 && U >= 8 && nr > U / 2) {
                // more than half a batch: a whole batch at once, the loads past the end re-reading row t
                // (for a running maximum a row fed twice changes nothing) - one memory latency, not three
                RowVec<ELT, V> v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int tu = t + u * step;
                    v[u] = load_vec<ELT, V>(base + (int64_t)(tu < t1 ? tu : t) * row_bytes);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int tu = t + u * step;
                    ATK_FEED_VEC(v[u], tu < t1 ? tu : t);
                }
                nr = 0;
            }
#define ATK_PIECE(NP)                                                                                          \
    if (NP < U && (nr & NP)) {                                                                                 \
        RowVec<ELT, V> v[NP];                                                                                  \
        _Pragma("unroll") for (int u = 0; u < NP; ++u) v[u] = load_vec<ELT, V>(base + (int64_t)(t + u * step) * row_bytes); \
        _Pragma("unroll") for (int u = 0; u < NP; ++u) ATK_FEED_VEC(v[u], t + u * step);                       \
        t += NP * step;                                                                                        \
    }
            ATK_PIECE(8)
            ATK_PIECE(4)
            ATK_PIECE(2)
            ATK_PIECE(1)
#undef ATK_PIECE
        }
        // The (virtual) row does not end on a matrix row: the last matrix row holds only its
        // first `remr` columns (the short buckets of Figure 2).  It has the highest indices, so
        // it is fed last.
        if (remr > 0 && sp == p.S - 1 && ph == eph && col0 < remr) {
            const unsigned char *last = base + (int64_t)Lr * row_bytes;
            if (col0 + V <= remr) {
                RowVec<ELT, V> v = load_vec<ELT, V>(last);
                ATK_FEED_VEC(v, Lr);
            } else {
#pragma unroll
                for (int e = 0; e < V; ++e)
                    if (col0 + e < remr) {
                        RowVec<ELT, 1> one = load_vec<ELT, 1>(last + e * ES);
                        ATK_FEED_ELEM(e, (elem_bits<ELT, 1>(one, 0)), Lr);
                    }
            }
        }
    }

#undef ATK_FEED_VEC
#undef ATK_FEED_ELEM
    trace_mark<TR>(p.trace, 1);  // its share of the row is in
    if constexpr (BATCH) {
#pragma unroll
        for (int e = 0; e < V; ++e)
#pragma unroll
            for (int j = 0; j < KB; ++j) {
                const u64 c = qw[e][j];
                if (c != 0ull) {
                    val[e][j] = __uint_as_float(((uint32_t)c & 1u) ? 0x80000000u : bits_of_ukey((uint32_t)(c >> 32)));
                    tt[e][j] = (int)(0x7fffffffu - ((uint32_t)c >> 1));
                }
            }
    }
    if constexpr (PK) {
#pragma unroll
        for (int e = 0; e < V; ++e)
#pragma unroll
            for (int j = 0; j < KB; ++j) unpack_bf16(pk[e][j], t0, val[e][j], tt[e][j]);
    }

    // ---------------------------------------------------------------- every lane owns whole buckets
    if (p.direct) {
        if (!active) return;
        const int64_t o = (int64_t)r * p.k + (int64_t)col0 * p.k_b;
        if (p.vec_store && rot == 0 && p.k_b == KB && (V * KB) % ((ELT == ATK_F32) ? 4 : 8) == 0) {
            constexpr int N = V * KB;  // contiguous outputs of this lane
            uint32_t ob[N];
            int32_t oi[N];
#pragma unroll
            for (int e = 0; e < V; ++e)
#pragma unroll
                for (int j = 0; j < KB; ++j) {
                    ob[e * KB + j] = __float_as_uint(val[e][j]);
                    oi[e * KB + j] = tt[e][j] * p.b + col0 + e;
                }
            typedef uint32_t v4u __attribute__((ext_vector_type(4)));
            v4u *pi = (v4u *)(p.out_idx + o);
#pragma unroll
            for (int q = 0; q < N / 4; ++q) {
                v4u w = {(uint32_t)oi[4 * q], (uint32_t)oi[4 * q + 1], (uint32_t)oi[4 * q + 2], (uint32_t)oi[4 * q + 3]};
                pi[q] = w;
            }
            if (ELT == ATK_F32) {
                v4u *pv = (v4u *)((uint32_t *)p.out_vals + o);
#pragma unroll
                for (int q = 0; q < N / 4; ++q) {
                    v4u w = {ob[4 * q], ob[4 * q + 1], ob[4 * q + 2], ob[4 * q + 3]};
                    pv[q] = w;
                }
            } else {
                v4u *pv = (v4u *)((uint16_t *)p.out_vals + o);
#pragma unroll
                for (int q = 0; q < N / 8; ++q) {
                    v4u w;
                    w.x = (ob[8 * q] >> 16) | (ob[8 * q + 1] & 0xffff0000u);
                    w.y = (ob[8 * q + 2] >> 16) | (ob[8 * q + 3] & 0xffff0000u);
                    w.z = (ob[8 * q + 4] >> 16) | (ob[8 * q + 5] & 0xffff0000u);
                    w.w = (ob[8 * q + 6] >> 16) | (ob[8 * q + 7] & 0xffff0000u);
                    pv[q] = w;
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e)
#pragma unroll
                for (int j = 0; j < KB; ++j)
                    if (j < p.k_b) {
                        const int64_t pos = (int64_t)r * p.k + (int64_t)bucket_of(col0 + e) * p.k_b + j;
                        store_val<ELT>(p.out_vals, pos, __float_as_uint(val[e][j]));
                        p.out_idx[pos] = tt[e][j] * p.b + col0 + e - rot;
                    }
        }
        return;
    }

    // ---------------------------------------------------------------- one slot, one workgroup per row or column block
    if constexpr (KB == 1) {
        if (p.lds_max) {
            u64 *cand = (u64 *)(smem + p.lds_cand_off);
            const int colbase = cb * p.Gw * V;
            const int wcols = min(p.Gw * V, p.b - colbase);
            const bool binned = p.stage2 && binned_fits(wcols) && p.bound_ok;
            uint32_t k_min = 0xffffffffu, k_max = 0u;
            bool whole = active;  // this lane holds an element of every one of its V columns
            if (active) {
#pragma unroll
                for (int e = 0; e < V; ++e) whole = whole && tt[e][0] != kEmptyT;
#pragma unroll
                for (int e = 0; e < V; ++e)
                    if (tt[e][0] != kEmptyT) {
                        const u64 c = make_composite(__float_as_uint(val[e][0]), tt[e][0] * p.b + col0 + e - rot);
                        // column e of column group cgl sits at e*Gw + cgl: side-by-side lanes, side-by-side words
                        __hip_atomic_fetch_max(&cand[e * p.Gw + cgl], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                        const uint32_t key = (uint32_t)(c >> 32);
                        k_min = key < k_min ? key : k_min;
                        k_max = key > k_max ? key : k_max;
                    }
            }
            if (binned) {
                // the range of the value keys that Stage 2 spreads its bins over: the lanes' maxima span at least
                // the range of the columns' maxima.  Folded here, before the barrier, it costs the wavefronts that
                // finish reading early nothing.
                uint32_t *misc = binned_misc(cand, wcols);
                k_min = wave_min_u32(k_min);
                k_max = wave_max_u32(k_max);
                // a wavefront whose 64 lanes between them hold an element of every column of the row: its minimum is
                // a lower bound on the smallest candidate, usually far tighter than the minimum over all lanes
                const bool cover = p.Gw <= kWave && __ballot(whole) == ~0ull;
                if ((tid & (kWave - 1)) == 0) {
                    atomicMin(&misc[1], k_min);
                    atomicMax(&misc[2], k_max);
                    if (cover) atomicMax(&misc[4], k_min);
                }
            }
            trace_mark<TR>(p.trace, 2);  // this wavefront's maxima are in
            __syncthreads();
            if (!p.stage2) {
                for (int lc = tid; lc < wcols; lc += T)
                    write_composite<ELT>(cand[(lc % V) * p.Gw + lc / V], p.out_vals, p.out_idx,
                                         (int64_t)r * p.k + bucket_of(colbase + lc));
                trace_mark<TR>(p.trace, 9);
                return;
            }
            trace_mark<TR>(p.trace, 3);  // all candidates of the row are in LDS, their key range is known
            if (binned)
                select_binned<ELT, TR>(cand, wcols, p.k, p.idx_bits, p.out_vals, p.out_idx, (int64_t)r, p.trace);
            else
                select_write<ELT, TR>(cand, wcols, p.k, p.idx_bits, p.out_vals, p.out_idx, (int64_t)r, p.trace);
            trace_mark<TR>(p.trace, 8);
            trace_mark<TR>(p.trace, 9);
            return;
        }
    }

    // ---------------------------------------------------------------- to composites
    u64 comp[V][KB];
#pragma unroll
    for (int e = 0; e < V; ++e)
#pragma unroll
        for (int j = 0; j < KB; ++j)
            comp[e][j] = (tt[e][j] != kEmptyT)
                             ? make_composite(__float_as_uint(val[e][j]), tt[e][j] * p.b + col0 + e - rot)
                             : 0ull;

    // ---------------------------------------------------------------- merge inside the wavefront
    // With fewer than 64 column groups the lanes l, l+Gw, l+2Gw, ... of a wavefront share
    // their columns: a butterfly over those lane strides leaves the merged list in all of them.
    if (p.wave_merge) {
        for (int off = p.Gw; off < kWave; off <<= 1) {
#pragma unroll
            for (int e = 0; e < V; ++e) {
                u64 theirs[KB];
#pragma unroll
                for (int j = 0; j < KB; ++j) theirs[j] = shfl_xor_u64(comp[e][j], off);
                merge_topk<KB>(comp[e], theirs);
            }
        }
    }

    // ---------------------------------------------------------------- where finished lists go
    u64 *cand = (u64 *)(smem + p.lds_cand_off);
    auto emit = [&](int col, const u64(&list)[KB]) { emit_list<ELT, KB>(p, r, sp, col, list, cand); };

    // ---------------------------------------------------------------- merge across wavefronts (LDS, one barrier)
    if (p.nparts > 1) {
        // columns are numbered from the first one of this workgroup's column block
        u64 *xch = (u64 *)(smem + p.lds_xch_off);  // [part][column][slot]
        const int lane = tid & (kWave - 1);
        const int part = p.wave_merge ? (tid >> 6) : ph;
        const bool holder = active && (!p.wave_merge || lane < p.Gw);
        const int colbase = cb * p.Gw * V;
        const int wcols = min(p.Gw * V, p.b - colbase);
        const int64_t pstride = (int64_t)p.Gw * V;  // columns per part
        if (holder) {
#pragma unroll
            for (int e = 0; e < V; ++e)
#pragma unroll
                for (int j = 0; j < KB; ++j) xch[((int64_t)part * pstride + cgl * V + e) * KB + j] = comp[e][j];
        }
        __syncthreads();
        for (int c = tid; c < wcols; c += T) {
            u64 acc[KB];
#pragma unroll
            for (int j = 0; j < KB; ++j) acc[j] = xch[(int64_t)c * KB + j];
            for (int q = 1; q < p.nparts; ++q) {
                u64 theirs[KB];
#pragma unroll
                for (int j = 0; j < KB; ++j) theirs[j] = xch[((int64_t)q * pstride + c) * KB + j];
                merge_topk<KB>(acc, theirs);
            }
            emit(bucket_of(colbase + c), acc);
        }
    } else if (active && (!p.wave_merge || (tid & (kWave - 1)) < p.Gw)) {
#pragma unroll
        for (int e = 0; e < V; ++e) emit(bucket_of(col0 + e), comp[e]);
    }

    trace_mark<TR>(p.trace, 2);  // this workgroup's lists are merged and handed on
    const bool whole = p.stage2 != 0;
    row_tail<ELT, KB, TR>(p, r, whole ? (int64_t)r : (int64_t)r * p.colblocks + cb, whole ? 0 : cb * p.Gw * V,
                          whole ? p.b : min(p.b, (cb + 1) * p.Gw * V), whole ? 0 : rot, smem);
    trace_mark<TR>(p.trace, 9);  // done
}

// ------------------------------------------------------------------------------------------------
// Contiguous assignment (Appendix A.1): bucket j is the run of elements i with floor(b*i/n) = j,
// that is [ceil(j*n/b), ceil((j+1)*n/b)).  Gs lanes side by side share a bucket: lane q reads the
// V-element chunks q, q+Gs, q+2Gs, ... of the run (consecutive lanes, consecutive addresses) into
// one queue, and the Gs queues are merged by a butterfly of shuffles (and, when a bucket takes
// more than one wavefront, once through LDS).  Long buckets of small batches are also split
// over S workgroups.  From the finished per-bucket lists on, everything is shared with the
// interleaved kernel (emit_list, row_tail).
// V > 1 is used only when every bucket has the same length L = n/b, V divides L and the rows
// are aligned; otherwise V = 1 and the runs may differ in length by one.
template <int ELT, int V, int KB, int U, int MAXT>
__global__ void __launch_bounds__(MAXT) contig_kernel(S1Params p) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int ES = (ELT == ATK_F32) ? 4 : 2;
    const int tid = threadIdx.x, T = blockDim.x;
    int wg = blockIdx.x, bb, sp, r;
    divmod(wg, p.bblocks, -1, wg, bb);
    divmod(wg, p.S, p.s_shift, r, sp);
    const int g = tid >> p.gs_shift, q = tid & (p.Gs - 1);
    const int bpw = T >> p.gs_shift;  // buckets the workgroup works on at a time

    // ---- short buckets: a bucket is one load per lane of its group; the group takes NB buckets in turn
    if (p.NB > 0) {
        const int first = bb * bpw * p.NB;  // first bucket of this workgroup
        u64 *cand = (u64 *)(smem + p.lds_cand_off);
        for (int i0 = 0; i0 < p.NB; i0 += U) {
            RowVec<ELT, V> v[U];
            int bj[U];
            int64_t r0[U];
            bool has[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int jj = first + (i0 + u) * bpw + g;
                const bool ok = (i0 + u < p.NB) && jj < p.b;
                int64_t a0 = 0, a1 = 0;
                if (ok) {
                    if (p.rem == 0) {
                        a0 = (int64_t)jj * p.L;
                        a1 = a0 + p.L;
                    } else {
                        a0 = ((int64_t)jj * p.n + p.b - 1) / p.b;
                        a1 = ((int64_t)(jj + 1) * p.n + p.b - 1) / p.b;
                    }
                }
                bj[u] = ok ? jj : -1;
                r0[u] = a0;
                has[u] = ok && (int64_t)q * V < a1 - a0;
            }
            // all loads of the batch are issued together; a lane without an element of its own re-reads the
            // start of the row and drops it (a load under a condition would wait for the one before it)
#pragma unroll
            for (int u = 0; u < U; ++u)
                v[u] = load_vec<ELT, V>((const unsigned char *)p.x +
                                        ((int64_t)r * p.n + (has[u] ? r0[u] + (int64_t)q * V : 0)) * ES);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float val[KB];
                int tt[KB];
#pragma unroll
                for (int i = 0; i < KB; ++i) {
                    val[i] = __uint_as_float(0x7fc00000u);
                    tt[i] = kEmptyT;
                }
                if (has[u]) {
#pragma unroll
                    for (int e = 0; e < V; ++e) insert<KB>(val, tt, __uint_as_float(elem_bits<ELT, V>(v[u], e)), q * V + e);
                }
                u64 comp[KB];
#pragma unroll
                for (int i = 0; i < KB; ++i)
                    comp[i] = (tt[i] != kEmptyT) ? make_composite(__float_as_uint(val[i]), (int32_t)(r0[u] + tt[i])) : 0ull;
                if (KB == 1) {
                    // one slot: the merge is a maximum over the group's lanes; inside a row of 16 lanes
                    // it goes through DPP (register to register), only groups of 32 and 64 lanes need
                    // a cross-row exchange on top
                    u64 v = comp[0], t;
                    if (p.Gs >= 2) { t = dpp_u64<0xB1>(v); v = t > v ? t : v; }
                    if (p.Gs >= 4) { t = dpp_u64<0x4E>(v); v = t > v ? t : v; }
                    if (p.Gs >= 8) { t = dpp_u64<0x141>(v); v = t > v ? t : v; }
                    if (p.Gs >= 16) { t = dpp_u64<0x140>(v); v = t > v ? t : v; }
                    if (p.Gs >= 32) { t = shfl_xor_u64(v, 16); v = t > v ? t : v; }
                    if (p.Gs >= 64) { t = shfl_xor_u64(v, 32); v = t > v ? t : v; }
                    comp[0] = v;
                } else {
                    for (int off = 1; off < p.Gs; off <<= 1) {
                        u64 theirs[KB];
#pragma unroll
                        for (int i = 0; i < KB; ++i) theirs[i] = shfl_xor_u64(comp[i], off);
                        merge_topk<KB>(comp, theirs);
                    }
                }
                if (q == 0 && bj[u] >= 0) emit_list<ELT, KB>(p, r, 0, bj[u], comp, cand);
            }
        }
        row_tail<ELT, KB>(p, r, (int64_t)r, 0, p.b, 0, smem);  // no row splits here: a ticket only with Stage 2
        return;
    }

    const int j = bb * bpw + g;       // this lane's bucket
    const bool active = j < p.b;

    float val[KB];
    int tt[KB];
#pragma unroll
    for (int i = 0; i < KB; ++i) {
        val[i] = __uint_as_float(0x7fc00000u);
        tt[i] = kEmptyT;
    }
    // the run of bucket j, in elements of the row
    int64_t run0 = 0, run1 = 0;
    if (active) {
        run0 = ((int64_t)j * p.n + p.b - 1) / p.b;
        run1 = ((int64_t)(j + 1) * p.n + p.b - 1) / p.b;
    }
    if (active) {
        const int chunks = (int)((run1 - run0) / V);
        const int c0 = sp * p.chunks_per_split;
        const int c1 = min(chunks, c0 + p.chunks_per_split);
        const unsigned char *base = (const unsigned char *)p.x + ((int64_t)r * p.n + run0) * ES;
        auto feed = [&](const RowVec<ELT, V> &v, int c) {
            float x[V];
#pragma unroll
            for (int e = 0; e < V; ++e) x[e] = __uint_as_float(elem_bits<ELT, V>(v, e));
            if (KB > 1) {
                bool any = false;
#pragma unroll
                for (int e = 0; e < V; ++e) any = any || !(x[e] <= val[KB - 1]);
                if (__ballot(any) == 0ull) return;
            }
#pragma unroll
            for (int e = 0; e < V; ++e) insert<KB>(val, tt, x[e], c * V + e);
        };
        int c = c0 + q;
        for (; c + (U - 1) * p.Gs < c1; c += U * p.Gs) {
            RowVec<ELT, V> v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = load_vec<ELT, V>(base + (int64_t)(c + u * p.Gs) * (V * ES));
#pragma unroll
            for (int u = 0; u < U; ++u) feed(v[u], c + u * p.Gs);
        }
        if (c < c1) {  // fewer than U loads left: in pieces of U/2 ... 1, each piece's loads issued together
            const int nr = (c1 - c + p.Gs - 1) >> p.gs_shift;
#define ATK_PIECE(NP)                                                                                                  \
    if (NP < U && (nr & NP)) {                                                                                         \
        RowVec<ELT, V> v[NP];                                                                                          \
        _Pragma("unroll") for (int u = 0; u < NP; ++u) v[u] = load_vec<ELT, V>(base + (int64_t)(c + u * p.Gs) * (V * ES)); \
        _Pragma("unroll") for (int u = 0; u < NP; ++u) feed(v[u], c + u * p.Gs);                                       \
        c += NP * p.Gs;                                                                                                \
    }
            ATK_PIECE(8)
            ATK_PIECE(4)
            ATK_PIECE(2)
            ATK_PIECE(1)
#undef ATK_PIECE
        }
    }
    u64 comp[KB];
#pragma unroll
    for (int i = 0; i < KB; ++i)
        comp[i] = (tt[i] != kEmptyT) ? make_composite(__float_as_uint(val[i]), (int32_t)(run0 + tt[i])) : 0ull;

    // ---- merge the Gs queues of a bucket: butterfly inside the wavefront ...
    const int span = p.Gs < kWave ? p.Gs : kWave;
    for (int off = 1; off < span; off <<= 1) {
        u64 theirs[KB];
#pragma unroll
        for (int i = 0; i < KB; ++i) theirs[i] = shfl_xor_u64(comp[i], off);
        merge_topk<KB>(comp, theirs);
    }
    // ... and across the wavefronts of the workgroup when the bucket owns all of it
    if (p.Gs > kWave) {
        u64 *xch = (u64 *)(smem + p.lds_xch_off);  // [wavefront][slot]
        const int lane = tid & (kWave - 1), wave = tid >> 6, n_waves = T >> 6;
        if (lane == 0) {
#pragma unroll
            for (int i = 0; i < KB; ++i) xch[wave * KB + i] = comp[i];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int i = 0; i < KB; ++i) comp[i] = (lane < n_waves) ? xch[lane * KB + i] : 0ull;
            for (int off = 1; off < n_waves; off <<= 1) {
                u64 theirs[KB];
#pragma unroll
                for (int i = 0; i < KB; ++i) theirs[i] = shfl_xor_u64(comp[i], off);
                merge_topk<KB>(comp, theirs);
            }
        }
    }
    u64 *cand = (u64 *)(smem + p.lds_cand_off);
    if (active && q == 0) emit_list<ELT, KB>(p, r, sp, j, comp, cand);
    const bool whole = p.stage2 != 0;
    row_tail<ELT, KB>(p, r, whole ? (int64_t)r : (int64_t)r * p.bblocks + bb, whole ? 0 : bb * bpw,
                      whole ? p.b : min(p.b, (bb + 1) * bpw), 0, smem);
}

// ------------------------------------------------------------------------------------------------
template <int ELT, int V, int KB, int U>
static hipError_t launch_one(const Plan &pl, const S1Params &prm, hipStream_t stream) {
    constexpr int MAXT = max_threads_for_kb(KB);
    if (pl.T > MAXT) return hipErrorInvalidValue;
    if constexpr (ELT == ATK_BF16 && KB >= 4) {
        if (pl.packed) {
            hipLaunchKernelGGL((stage1_kernel<ELT, V, KB, U, MAXT, true>), dim3((unsigned)pl.grid),
                               dim3((unsigned)pl.T), (size_t)pl.lds_bytes, stream, prm);
            return hipGetLastError();
        }
    }
    if (prm.trace) return hipErrorNotSupported;  // the measurement build exists for the lean kernels only
    if constexpr (KB == 8) {
        if (pl.refresh) {
            hipLaunchKernelGGL((stage1_kernel<ELT, V, KB, U, MAXT, false, false, true>), dim3((unsigned)pl.grid),
                               dim3((unsigned)pl.T), (size_t)pl.lds_bytes, stream, prm);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((stage1_kernel<ELT, V, KB, U, MAXT, false>), dim3((unsigned)pl.grid), dim3((unsigned)pl.T),
                       (size_t)pl.lds_bytes, stream, prm);
    return hipGetLastError();
}

static int log2_exact(int v) {
    if (v < 1 || (v & (v - 1))) return -1;
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

hipError_t launch_approx(const Plan &pl, const void *x, void *out_vals, int32_t *out_idx, void *state, void *data,
                         hipStream_t stream, void *trace) {
    S1Params prm;
    memset(&prm, 0, sizeof prm);
    prm.trace = (u64 *)trace;
    prm.x = x;
    prm.out_vals = out_vals;
    prm.out_idx = out_idx;
    prm.tickets = (uint32_t *)state;
    prm.lists = (u64 *)data;
    prm.n = pl.n;
    prm.b = (int)pl.b;
    prm.L = (int)pl.L;
    prm.G = (int)pl.G;
    prm.Gw = pl.Gw;
    prm.P = pl.P;
    prm.colblocks = pl.colblocks;
    prm.S = pl.S;
    prm.rows_per_split = pl.rows_per_split;
    prm.rem = (int)(pl.n % pl.b);
    prm.extra_ph = (int)(pl.L % pl.P);
    prm.idx_bits = 1;
    while (((int64_t)1 << prm.idx_bits) < pl.n) ++prm.idx_bits;
    prm.k = (int)pl.k;
    prm.k_b = pl.k_b;
    prm.stage2 = pl.stage2;
    prm.direct = pl.direct;
    prm.use_scratch = pl.use_scratch;
    prm.wave_merge = pl.wave_merge;
    prm.nparts = pl.nparts;
    prm.lds_xch_off = pl.lds_xch_off;
    prm.lds_cand_off = pl.lds_cand_off;
    prm.lds_max = pl.lds_max;
    prm.bound_ok = pl.bound_ok;
    prm.refresh = pl.refresh;
    prm.wgs_per_ticket = pl.stage2 ? pl.S * pl.colblocks : pl.S;
    prm.tail_tpc_shift = log2_exact(pl.tail_tpc);
    prm.cb_shift = log2_exact(pl.colblocks);
    prm.s_shift = log2_exact(pl.S);
    prm.gw_shift = log2_exact(pl.Gw);
    const uintptr_t ov = (uintptr_t)out_vals, oi = (uintptr_t)out_idx;
    prm.vec_store = ((ov | oi) & 15u) == 0;
#define ATK_CASE(ELT, VV, KK, UU) \
    if (pl.dtype == ELT && pl.V == VV && pl.KB == KK) return launch_one<ELT, VV, KK, UU>(pl, prm, stream);
    ATK_STAGE1_INSTANCES(ATK_CASE)
#undef ATK_CASE
    return hipErrorInvalidValue;
}

template <int ELT, int V, int KB, int U>
static hipError_t launch_contig_one(const Plan &pl, const S1Params &prm, hipStream_t stream) {
    constexpr int MAXT = max_threads_for_kb(KB);
    if (pl.T > MAXT) return hipErrorInvalidValue;
    hipLaunchKernelGGL((contig_kernel<ELT, V, KB, U, MAXT>), dim3((unsigned)pl.grid), dim3((unsigned)pl.T),
                       (size_t)pl.lds_bytes, stream, prm);
    return hipGetLastError();
}

hipError_t launch_approx_contig(const Plan &pl, const void *x, void *out_vals, int32_t *out_idx, void *state,
                                void *data, hipStream_t stream) {
    S1Params prm;
    memset(&prm, 0, sizeof prm);
    prm.x = x;
    prm.out_vals = out_vals;
    prm.out_idx = out_idx;
    prm.tickets = (uint32_t *)state;
    prm.lists = (u64 *)data;
    prm.n = pl.n;
    prm.b = (int)pl.b;
    prm.L = (int)pl.L;
    prm.S = pl.S;
    prm.s_shift = log2_exact(pl.S);
    prm.idx_bits = 1;
    while (((int64_t)1 << prm.idx_bits) < pl.n) ++prm.idx_bits;
    prm.k = (int)pl.k;
    prm.k_b = pl.k_b;
    prm.stage2 = pl.stage2;
    prm.use_scratch = pl.use_scratch;
    prm.lds_xch_off = pl.lds_xch_off;
    prm.lds_cand_off = pl.lds_cand_off;
    prm.wgs_per_ticket = pl.stage2 ? pl.S * pl.bblocks : pl.S;
    prm.tail_tpc_shift = log2_exact(pl.tail_tpc);
    prm.Gs = pl.Gs;
    prm.gs_shift = log2_exact(pl.Gs);
    prm.bblocks = pl.bblocks;
    prm.chunks_per_split = pl.chunks_per_split;
    prm.NB = pl.NB;
    prm.rem = (int)(pl.n % pl.b);
    if (prm.gs_shift < 0) return hipErrorInvalidValue;
#define ATK_CASE(ELT, VV, KK, UU) \
    if (pl.dtype == ELT && pl.V == VV && pl.KB == KK) return launch_contig_one<ELT, VV, KK, UU>(pl, prm, stream);
    ATK_CONTIG_INSTANCES(ATK_CASE)
#undef ATK_CASE
    return hipErrorInvalidValue;
}

}  // namespace atk
