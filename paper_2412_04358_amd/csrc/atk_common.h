// Shared declarations of the HIP library: plans, device helpers, launch entry points.
// gfx950 (MI355X) only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/approx_topk.h"

typedef unsigned long long u64;

namespace atk {

constexpr int kWave = 64;
constexpr int kMaxThreads = 256;          // threads per workgroup of the select kernels
// largest workgroup of the streaming kernel: big register queues (k_b >= 8) keep to 256 lanes
constexpr int max_threads_for_kb(int KB) { return KB <= 4 ? 1024 : 256; }
// Streaming-kernel instances: X(element type, columns per lane V, slots KB, load batches U).
// One lane owns V adjacent buckets and reads them with one V-element load per matrix row.
// For every (type, KB) the first entry is the planner's default; the others can be asked
// for with ATK_PLAN="V=..", and V=1 serves rows whose layout rules out vector loads.
// Wide lanes pay off only for KB = 1: with more slots the per-lane register queues
// (V*KB values and rows) cut the waves per CU, and narrower lanes are faster.
#define ATK_STAGE1_INSTANCES(X) \
    X(ATK_F32, 4, 1, 8)   X(ATK_F32, 2, 1, 8)   X(ATK_F32, 1, 1, 16)  \
    X(ATK_F32, 2, 2, 8)   X(ATK_F32, 4, 2, 4)   X(ATK_F32, 1, 2, 8)   \
    X(ATK_F32, 2, 4, 8)   X(ATK_F32, 4, 4, 4)   X(ATK_F32, 1, 4, 8)   \
    X(ATK_F32, 2, 8, 4)   X(ATK_F32, 4, 8, 2)   X(ATK_F32, 1, 8, 4)   \
    X(ATK_F32, 2, 16, 2)  X(ATK_F32, 1, 16, 2)                        \
    X(ATK_BF16, 8, 1, 8)  X(ATK_BF16, 4, 1, 8)  X(ATK_BF16, 1, 1, 16) \
    X(ATK_BF16, 4, 2, 8)  X(ATK_BF16, 8, 2, 4)  X(ATK_BF16, 2, 2, 8)  X(ATK_BF16, 1, 2, 8) \
    X(ATK_BF16, 2, 4, 8)  X(ATK_BF16, 4, 4, 8)  X(ATK_BF16, 8, 4, 2)  X(ATK_BF16, 1, 4, 8) \
    X(ATK_BF16, 2, 8, 4)  X(ATK_BF16, 4, 8, 2)  X(ATK_BF16, 1, 8, 4)  \
    X(ATK_BF16, 2, 16, 2) X(ATK_BF16, 1, 16, 2)

// Instances of the contiguous-assignment kernel: X(element type, elements per load V, slots KB,
// load batches U).  V is a full 16-byte load when the buckets allow it, else 1.
#define ATK_CONTIG_INSTANCES(X) \
    X(ATK_F32, 4, 1, 8)  X(ATK_F32, 4, 2, 4)  X(ATK_F32, 4, 4, 4)  X(ATK_F32, 4, 8, 2)  X(ATK_F32, 4, 16, 2)  \
    X(ATK_F32, 1, 1, 16) X(ATK_F32, 1, 2, 8)  X(ATK_F32, 1, 4, 8)  X(ATK_F32, 1, 8, 4)  X(ATK_F32, 1, 16, 2)  \
    X(ATK_BF16, 8, 1, 8) X(ATK_BF16, 8, 2, 4) X(ATK_BF16, 8, 4, 4) X(ATK_BF16, 8, 8, 2) X(ATK_BF16, 8, 16, 2) \
    X(ATK_BF16, 1, 1, 16) X(ATK_BF16, 1, 2, 8) X(ATK_BF16, 1, 4, 8) X(ATK_BF16, 1, 8, 4) X(ATK_BF16, 1, 16, 2)

// Columns per lane for (dtype, KB): the first listed instance whose V divides b, so that the
// V-element loads of a lane stay aligned from one matrix row to the next (and equals `want`,
// when that is not 0).  Rows that start off a V-element boundary (n not a multiple of V) are
// read from the aligned address before them.
inline int stage1_pick_v(int dtype, int KB, int want, int64_t b) {
#define ATK_X(ELT, VV, KK, UU) \
    if (dtype == ELT && KB == KK && (want == 0 || VV == want) && b % VV == 0) return VV;
    ATK_STAGE1_INSTANCES(ATK_X)
#undef ATK_X
    return want ? stage1_pick_v(dtype, KB, 0, b) : 1;
}
constexpr int kStage2MaxCand = 4096;      // composites held in LDS by the fused Stage 2
constexpr int kLdsBudget = 64 * 1024;     // static+dynamic LDS per workgroup we allow ourselves
constexpr int kLdsBudgetWholeRow = 160 * 1024;  // ... for exact_topk's one-workgroup-per-row kernel: all of a CU's LDS (gfx950)
constexpr int kNumCU = 256;               // MI355X
constexpr int kTicketStride = 32;          // words between row tickets: one 128-byte line each, so that
                                          // atomics of different rows do not queue up on one line
// Row splits whose lists the merging workgroup loads together (per lane), by slots per column.
constexpr int tail_split_batch(int KB) { return KB <= 2 ? 8 : (KB <= 4 ? 4 : 2); }
// Lanes side by side on one column in that merge: a power of two up to 64 such that all
// `cols` columns still fit the T lanes, and no more than there are batches of splits.
inline int tail_lanes_per_column(int64_t cols, int T, int KB, int64_t S) {
    int tpc = 1;
    while (tpc * 2 <= kWave && (int64_t)tpc * 2 * cols <= T && (int64_t)tpc * tail_split_batch(KB) < S) tpc <<= 1;
    return tpc;
}
constexpr int kEmptyT = 0x7fffffff;       // "no element yet" row marker of a register slot

// Launch-plan overrides for sweeps and tests: the ATK_PLAN environment variable, read once when the
// library is loaded, or whatever atk_set_plan_override() was last given.  0 / false = not set.
constexpr int kMultiSlots = 8;   // helpers + finisher on the lean kernel: mailbox words that a lane of the finisher fetches at once

struct PlanOverride {
    int T, S, V, P;   // threads per workgroup, row splits, columns per lane, lanes sharing a column group
    bool pk_off;      // PK=0: no packed bf16 queue words
    bool lm_off;      // LM=0: lanes that share a column merge through the LDS exchange, not by LDS atomic maximum
    int xs;           // exact_topk sampled threshold: 0 not set, 1 forced on (XS=1), -1 off (XS=0)
    int xc;           // exact_topk sweep chunk in elements
    int hf;           // two workgroups per row (helper + finisher): 0 not set, 1 forced on where legal (HF=1), -1 off (HF=0)
    int hq;           // the helper's share of the matrix rows in 64ths (HQ=..), 0 not set
    int ht;           // HT=<lanes>: workgroup size of the two-workgroups-per-row plans, 0 not set
    int sl;           // SL=<lanes>: lanes of a workgroup that stream (the rest only join Stage 2), 0 not set
    bool ln_off;      // LN=0: never the lean kernels
    int rf;           // RF=0: queues never pool their floors; RF=<n>: first after n load batches (0 not set)
    bool bo_off;      // BO=0: Stage 2's bins never take their range from the merge
    int mh;           // MH=0: no helpers + finisher plans for split rows (-1); MH=<h>: that many helpers where legal (0 not set)
};
const PlanOverride &plan_override();

// ------------------------------------------------------------------------------------
// Launch plan of approx_topk (host side, filled by make_plan()).
//
// A row of n elements is viewed as an L x b matrix (L = n/b rows, row-major): column j is
// bucket j (Appendix A.1, interleaved assignment), so Stage 1 is a column-wise top-k_b.
// A lane owns V adjacent columns (one 16-byte load) and walks down the matrix rows.
struct Plan {
    int dtype;        // ATK_F32 / ATK_BF16
    int V;            // columns per lane: 16 B / sizeof(element), or 1 for the scalar path
    int KB;           // register slots per column: k_b rounded up to a power of two
    int k_b;          // survivors per bucket
    int T;            // threads per workgroup
    int Gw;           // column groups (lanes side by side) per workgroup
    int P;            // row phases: lanes of one workgroup that share a column group
    int colblocks;    // workgroups side by side across the b columns
    int S;            // row splits: workgroups stacked down the L matrix rows
    int rows_per_split;
    int64_t G;        // column groups per row = b / V
    int64_t L;        // matrix rows = n / b
    int64_t m, n, k, b;
    bool stage2;      // b*k_b > k
    bool direct;      // every lane owns whole buckets: write results straight from registers
    bool use_scratch; // partial lists go through global scratch + a per-row ticket
    bool packed;      // bf16, k_b >= 3: 32-bit (key, row) queue words; needs rows_per_split + 2 < 32768
    int refresh;      // eight unpacked slots, lanes sharing columns: > 0 = the lanes of a column pool what they have seen after this many load batches (then after twice as many, ...) and raise their queues' floors to the k_b-th best of all
    bool lds_max;     // k_b = 1, no scratch, lanes share columns: they meet in LDS by atomic maximum
    bool bound_ok;    // lds_max with Stage 2: the merge yields a tight lower bound on the smallest candidate (see select_binned())
    bool lean;        // k_b = 1 on rows of whole aligned 16-byte vectors, one workgroup (or a pair) per row: the lean kernels
    int pair_rows;    // lean: > 0 = several workgroups per row (helpers + finisher), a helper takes this many matrix rows
    int helpers;      // > 0: the splits of a row (and column block) as that many helpers and a finisher (kLeanMulti); 0 with the pair kernels
    bool wave_merge;  // Gw < 64 and a power of two: lanes of a wavefront share columns, merged by shuffles
    int nparts;       // partial lists per column left for the LDS exchange
    int lds_xch_off, lds_cand_off;
    // contiguous assignment (floor(b*i/n)) only
    int tail_tpc;     // lanes per column in the last workgroup's merge of the row splits
    int assignment;   // ATK_INTERLEAVED / ATK_CONTIGUOUS
    int Gs;           // lanes side by side on one bucket (a power of two)
    int bblocks;      // workgroups side by side across the b buckets
    int chunks_per_split;  // V-element chunks of a bucket per row split
    int NB;           // short buckets (one load per lane): buckets a lane group takes in turn, else 0
    int64_t scratch_lists_bytes;   // composites
    int64_t scratch_ticket_bytes;  // one counter per row
    int lds_bytes;    // dynamic LDS of the launch
    int64_t grid;
};

int make_plan(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, Plan *plan);
int make_contig_plan(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, bool ptr16, Plan *plan);

// Enqueue the fused Stage 1 (+ merge, + Stage 2) kernel for `plan`.
// state: zeroed words (tickets); data: partial lists.
// trace: NULL, or (measurement build of the k_b = 1 kernels with 16-byte loads) a device buffer of
// grid * kTraceWaves * kTracePhases words that receives every wavefront's phase timestamps.
hipError_t launch_approx(const Plan &plan, const void *x, void *out_vals, int32_t *out_idx, void *state, void *data,
                         hipStream_t stream, void *trace = nullptr);
// The same for a plan of make_contig_plan().
hipError_t launch_approx_contig(const Plan &plan, const void *x, void *out_vals, int32_t *out_idx, void *state,
                                void *data, hipStream_t stream);

// The same for a plan with `lean` set (atk_lean_kernel.h).  state: the helper-to-finisher mailbox of a pair plan
// (plan.scratch_ticket_bytes, zero between calls), else unused.  trace: as for launch_approx.
hipError_t launch_approx_lean(const Plan &plan, const void *x, void *out_vals, int32_t *out_idx, void *state,
                              hipStream_t stream, void *trace = nullptr);

// ------------------------------------------------------------------------------------
// exact_topk plan
struct ExactPlan {
    int dtype;
    int64_t m, n, k;
    int64_t idx_n;          // column indices are below this (n, unless the rows are lists of (value, index) pairs)
    bool single_wg;         // whole row fits one workgroup's LDS
    int T;
    int lds_bytes;
    int chunks;             // workgroups per row of the global path
    int chunk_elems;        // elements of a row that one of them sweeps
    bool filter;            // small k: rows may finish through the copy-out buffer
    int filter_cap;         // ... of this many elements per row
    bool sample;            // very small k on big inputs: the copy-out threshold is first guessed from a sample of the row
    int64_t scratch_bytes;  // data pool
    int64_t state_bytes;    // zeroed-state pool
};
int make_exact_plan(int64_t m, int64_t n, int64_t k, int dtype, ExactPlan *plan);
// xi: NULL, or (device, m x n int32) the column index each element of x stands for: the rows are then
// lists of (value, index) pairs with distinct indices below plan.idx_n, and the order among equal
// values and out_idx follow those indices (Stage 2 over more candidates than fit one workgroup).
hipError_t launch_exact(const ExactPlan &plan, const void *x, const int32_t *xi, void *out_vals, int32_t *out_idx,
                        void *state, void *data, hipStream_t stream);

// ------------------------------------------------------------------------------------
// Device helpers.
#ifdef __HIPCC__

// Order-preserving map float bits -> unsigned key, with -0 mapped onto +0's key, so that
// integer order on keys equals IEEE order on values (NaN-free input).
__device__ __forceinline__ uint32_t ukey_of_bits(uint32_t bits) {
    uint32_t c = (bits == 0x80000000u) ? 0u : bits;
    uint32_t mask = (uint32_t)((int32_t)c >> 31) | 0x80000000u;
    return c ^ mask;
}
__device__ __forceinline__ uint32_t bits_of_ukey(uint32_t key) {
    return (key & 0x80000000u) ? (key ^ 0x80000000u) : ~key;
}

// Composite word: [63:32] value key, [31:1] 0x7fffffff - index, [0] "the element was -0".
// Larger composite <=> larger value, or equal value and lower index.  (key, index) pairs
// of one row are distinct, so bit 0 never decides an order; it only carries the sign of
// a zero to the output.  0 is never a valid composite (the key of -inf is 0x007fffff) and
// marks an empty slot.
__device__ __forceinline__ u64 make_composite(uint32_t bits, int32_t idx) {
    uint32_t key = ukey_of_bits(bits);
    uint32_t lo = ((0x7fffffffu - (uint32_t)idx) << 1) | (bits == 0x80000000u ? 1u : 0u);
    return ((u64)key << 32) | lo;
}
__device__ __forceinline__ int32_t composite_index(u64 c) {
    return (int32_t)(0x7fffffffu - ((uint32_t)c >> 1));
}
__device__ __forceinline__ uint32_t composite_bits(u64 c) {
    return ((uint32_t)c & 1u) ? 0x80000000u : bits_of_ukey((uint32_t)(c >> 32));
}

__device__ __forceinline__ u64 umax64(u64 a, u64 b) { return a > b ? a : b; }

__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int lane_mask) {
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    lo = (uint32_t)__shfl_xor((int)lo, lane_mask, kWave);
    hi = (uint32_t)__shfl_xor((int)hi, lane_mask, kWave);
    return ((u64)hi << 32) | lo;
}

// mine <- the KB largest of (mine U theirs); both sorted descending, result sorted descending.
template <int KB>
__device__ __forceinline__ void merge_topk(u64 (&mine)[KB], const u64 (&theirs)[KB]) {
#pragma unroll
    for (int j = 0; j < KB; ++j) mine[j] = umax64(mine[j], theirs[KB - 1 - j]);
    // mine is now bitonic and holds the KB largest: sort it descending
#pragma unroll
    for (int stride = KB / 2; stride >= 1; stride >>= 1) {
#pragma unroll
        for (int i = 0; i < KB; ++i) {
            if ((i & stride) == 0) {
                u64 a = mine[i], c = mine[i + stride];
                bool sw = c > a;
                mine[i] = sw ? c : a;
                mine[i + stride] = sw ? a : c;
            }
        }
    }
}

// Store the value part of an output element.
template <int ELT>
__device__ __forceinline__ void store_val(void *out_vals, int64_t pos, uint32_t bits32) {
    if (ELT == ATK_F32)
        ((uint32_t *)out_vals)[pos] = bits32;
    else
        ((uint16_t *)out_vals)[pos] = (uint16_t)(bits32 >> 16);
}

#endif  // __HIPCC__

}  // namespace atk
