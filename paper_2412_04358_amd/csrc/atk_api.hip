// C ABI of the library (include/approx_topk.h): argument checks, launch planning, the
// per-device scratch pool, and the measurement utilities.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <mutex>

#include "atk_common.h"
#include "atk_select.h"

namespace atk {

static thread_local int g_last_hip_error = 0;

static int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return ATK_ERR_HIP;
}

static int64_t pow2_ceil(int64_t v) {
    int64_t p = 1;
    while (p < v) p <<= 1;
    return p;
}

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ------------------------------------------------------------------------------------ checks
static int check_common(int64_t m, int64_t n, int64_t k, int dtype) {
    if (dtype != ATK_F32 && dtype != ATK_BF16) return ATK_ERR_DTYPE;
    if (m < 1 || n < 1 || k < 1 || k > n) return ATK_ERR_BAD_SHAPE;
    if (n >= (1ll << 31)) return ATK_ERR_BAD_SHAPE;  // int32 column indices
    if (m > (1ll << 40) / n || m > (1ll << 40) / k) return ATK_ERR_BAD_SHAPE;
    return ATK_OK;
}

// Section 2: b in {1..n}, k_b in {1..min(k, n/b)}, b*k_b >= k.
static int check_approx(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype) {
    int rc = check_common(m, n, k, dtype);
    if (rc != ATK_OK) return rc;
    if (b < 1 || b > n || k_b < 1) return ATK_ERR_BAD_PARAMS;
    if (k_b > k || k_b > n / b) return ATK_ERR_BAD_PARAMS;
    if (b * k_b < k) return ATK_ERR_BAD_PARAMS;
    if (k_b > ATK_MAX_KB) return ATK_ERR_UNSUPPORTED;
    return ATK_OK;
}

// ------------------------------------------------------------------------------------ plan override
// "T=128,S=4,V=2,...": tuning knobs for sweeps and tests; values the kernels cannot take are dropped here.
static PlanOverride parse_plan_override(const char *e) {
    PlanOverride o;
    memset(&o, 0, sizeof o);
    if (!e) return o;
    auto field = [&](const char *name) -> const char * {  // the text behind "name=" at the start of an item
        const size_t len = strlen(name);
        for (const char *q = e; (q = strstr(q, name)) != nullptr; q += len)
            if ((q == e || q[-1] == ',') && q[len] == '=') return q + len + 1;
        return nullptr;
    };
    if (const char *q = field("T")) {
        const int v = atoi(q);
        if (v == 64 || v == 128 || v == 256 || v == 512 || v == 1024) o.T = v;
    }
    if (const char *q = field("S")) {
        const int v = atoi(q);
        if (v >= 1 && v <= 4096) o.S = v;
    }
    if (const char *q = field("V")) {
        const int v = atoi(q);
        if (v == 1 || v == 2 || v == 4 || v == 8) o.V = v;
    }
    if (const char *q = field("P")) {
        const int v = atoi(q);
        if (v >= 1 && v <= 64 && (v & (v - 1)) == 0) o.P = v;
    }
    if (const char *q = field("PK")) o.pk_off = atoi(q) == 0;
    if (const char *q = field("LM")) o.lm_off = atoi(q) == 0;
    if (const char *q = field("LN")) o.ln_off = atoi(q) == 0;
    if (const char *q = field("XS")) o.xs = atoi(q) == 0 ? -1 : 1;
    if (const char *q = field("XC")) {
        const int v = atoi(q);
        if (v >= 1024 && v <= 16384 && (v & (v - 1)) == 0) o.xc = v;
    }
    if (const char *q = field("HF")) o.hf = atoi(q) == 0 ? -1 : 1;
    if (const char *q = field("HT")) o.ht = atoi(q);
    if (const char *q = field("RF")) o.rf = atoi(q) <= 0 ? -1 : atoi(q);
    if (const char *q = field("SL")) o.sl = atoi(q);
    if (const char *q = field("BO")) o.bo_off = atoi(q) == 0;
    if (const char *q = field("MH")) {
        const int v = atoi(q);
        o.mh = v <= 0 ? -1 : (v <= 255 ? v : 0);
    }
    if (const char *q = field("HQ")) {
        const int v = atoi(q);
        if (v >= 1 && v <= 63) o.hq = v;
    }
    return o;
}
static PlanOverride g_plan_override = parse_plan_override(getenv("ATK_PLAN"));  // read once, at load
const PlanOverride &plan_override() { return g_plan_override; }

// ------------------------------------------------------------------------------------ approx plan
static int make_plan_aligned(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, bool ptr16,
                             Plan *pl, bool allow_pair = true) {
    const int es = (dtype == ATK_F32) ? 4 : 2;
    Plan p;
    memset(&p, 0, sizeof p);
    p.dtype = dtype;
    p.m = m;
    p.n = n;
    p.k = k;
    p.b = b;
    p.k_b = (int)k_b;
    p.KB = (int)pow2_ceil(k_b);
    // columns per lane: the default instance for (dtype, KB), or the widest one within V_forced
    const PlanOverride &ov = plan_override();
    const int T_forced = ov.T, S_forced = ov.S, V_forced = ov.V;
    // (vector loads need a 16-byte aligned x and b a multiple of V)
    int v_want = !ptr16 ? 1 : V_forced;
    // bf16 queues of 8 and 16 slots over wide bucket layouts, on inputs that give the chip only a wavefront or
    // two per SIMD: one column per lane instead of two doubles the lanes, and the insertions, which bound
    // these shapes, spread over them (128 x 65536, b = 1024, k_b = 16: 29.1 -> 25.3 us; b = 2048, k_b = 8:
    // 13.7 -> 12.0 us; 64 rows, k_b = 16: 28.5 -> 22.4 us).  Past two (16 slots) or four (8 slots) wavefronts per
    // SIMD two columns per lane win again (256 rows, k_b = 16: 34.5 against 49.3 us), and so they do on fewer
    // lanes than one wavefront per SIMD, where the plan below puts several lanes on a column.
    if (!v_want && dtype == ATK_BF16 && p.KB >= 8 && b >= 1024 && m * b >= 256 * (int64_t)kNumCU &&
        m * b <= (p.KB >= 16 ? 512 : 1024) * (int64_t)kNumCU)
        v_want = 1;
    // f32 queues of 16 slots (fed sixteen matrix rows at a time, a long chain of dependent compare-exchanges) the same
    // way while two columns per lane would leave one wavefront per SIMD: 128 x 65536, b = 1024: 36.1 -> 27.0 us
    // (with more lanes than that two columns win: 128 x 2^20, b = 16384: 297 against 325 us)
    if (!v_want && dtype == ATK_F32 && p.KB >= 16 && b >= 1024 && m * b >= 256 * (int64_t)kNumCU && m * b <= 512 * (int64_t)kNumCU)
        v_want = 1;
    p.V = stage1_pick_v(dtype, p.KB, v_want, b);
    p.G = b / p.V;
    p.L = n / b;
    p.stage2 = b * k_b > k;

    // ---- workgroup size T and row splits S
    // Aim at about 16 vector loads per lane over the whole launch (in flight in batches), at least one workgroup per CU, and as few row splits as that allows: a split
    // costs a trip through memory at the end.  Narrow bucket layouts (fewer column groups
    // than lanes) take big workgroups, whose lanes merge through shuffles and LDS.
    const int t_max = max_threads_for_kb(p.KB);
    const int64_t n_vec = m * (n / p.V);
    int64_t want_threads = n_vec / 16;
    if (want_threads < 512 * (int64_t)kNumCU) want_threads = 512 * (int64_t)kNumCU;
    if (want_threads > 2048 * (int64_t)kNumCU) want_threads = 2048 * (int64_t)kNumCU;
    // with queues, a lane that sees more rows inserts less often, and every split less is a list less
    // through memory: half as many lanes measured faster (k_b = 2 on 128 x 2653751 bf16: 153 -> 136 us)
    if (p.KB >= 2 && want_threads > 1024 * (int64_t)kNumCU) want_threads = 1024 * (int64_t)kNumCU;
    // A running maximum costs a lane next to nothing, so k_b = 1 is bound by the memory system alone,
    // and that likes few, long streams: about one workgroup per CU measured fastest on long rows
    // (128 x 2^20, b = 64: 85.6 us with 1024 workgroups of 512 lanes, 80.1 with 256, 75.5 with 256
    // of 256 lanes), and every split less is a partial list less through memory.
    if (p.KB == 1) want_threads = 512 * (int64_t)kNumCU;
    const bool short_rule = p.KB == 1 && p.stage2 && !ov.lm_off && !ov.ln_off && ptr16 && p.V == 16 / es && n % b == 0 &&
                            (n * es) % 16 == 0 && 2 * m <= (int64_t)kNumCU && n <= 65536 && !S_forced;
    const bool lean_shape = ptr16 && p.V == 16 / es && n % b == 0 && (n * es) % 16 == 0;  // what the lean kernels ask of the input
    const bool multi_short = short_rule && allow_pair && ov.hf >= 0 && ov.mh >= 0 && m <= 32 && b <= 512 && n > 32768;
    // Without Stage 2 the workgroups of a row share out its columns in pieces of 128 bytes of a matrix row (below); a
    // row whose matrix rows are no longer than that (64 buckets in bf16, 32 in f32) cannot be shared out that way, and
    // two halves through scratch and a ticket cost more than the same pair of workgroups as helper and finisher
    // (128 x 65536 bf16, b = k = 64: 8.4 -> 7.5 us)
    const bool pair_out_rule = p.KB == 1 && !p.stage2 && allow_pair && ov.hf >= 0 && !ov.lm_off && !ov.ln_off && ptr16 &&
                               p.V == 16 / es && n % b == 0 && (n * es) % 16 == 0 && 2 * m <= (int64_t)kNumCU &&
                               n * es >= (128 << 10) && b * es <= 128 && !S_forced && !(dtype == ATK_BF16 && n <= 65536);
    // (bf16 rows of up to 65536 elements are better off in one workgroup of 512 lanes, all streaming: 128 x 65536, b = k = 64:
    // 6.9 us as a pair, 5.9 in one workgroup; 32 rows: 5.9 -> 5.4)
    const bool out_one_rule = p.KB == 1 && !p.stage2 && dtype == ATK_BF16 && ptr16 && p.V == 16 / es && n % b == 0 &&
                              (n * es) % 16 == 0 && n <= 65536 && b * es <= 128 && !S_forced && !ov.lm_off && !ov.ln_off;
    // rows short enough that a Stage 2 plan is better off in one workgroup per row than in two (below)
    const bool one_piece = n * (dtype == ATK_BF16 ? 4 : 1) <= 512 * 512;
    // Shapes on which two workgroups share a row as helper and finisher (atk_lean_kernel.h) instead of one workgroup, or
    // two halves meeting through scratch and a ticket: rows of whole aligned vectors with one slot per bucket, few
    // enough that every workgroup still has a CU of its own, long enough to be worth a second CU; past 512 buckets
    // Stage 2 outweighs what the second CU saves unless the row has 2^17 elements or more, or the batch is small
    // (65536-long rows, b = 1024: level at 128 rows; 32 rows: 9.4 us in one workgroup, 9.0 as a pair).
    const bool pair_rule = p.KB == 1 && p.stage2 && allow_pair && ov.hf >= 0 && !ov.lm_off && !ov.ln_off && ptr16 &&
                           p.V == 16 / es && n % b == 0 && (n * es) % 16 == 0 && 2 * m <= (int64_t)kNumCU &&
                           n * es >= (128 << 10) && b <= 1024 && (b <= 512 || n >= (1 << 17) || (m >= 8 && m <= 64));
    int T = 256;
    int64_t lanes_per_wg = 0;  // what a workgroup counts as when the splits are chosen (0: its size)
    if (p.G <= 256) {
        const int t_cols = (int)(ceil_div(p.G, kWave) * kWave);  // lanes that give every column group one lane
        if (m * t_cols * 2 >= want_threads) {
            // enough rows to fill the chip with one lane per column group: no merging at all
            T = t_cols;
        } else {
            T = t_max < 512 ? t_max : 512;
            while (T > 256 && m * T * 2 > want_threads) T >>= 1;  // keep at least two splits' worth of lanes
            // k_b = 1 in f32 with at least 32 loads per lane left: four wavefronts per CU stream faster
            // than eight (fewer open streams per memory channel); the number of workgroups stays.
            // bf16 lanes do twice the work per load and want the eight (43 against 55 us on 128 x 2^20).
            if (p.KB == 1 && T == 512 && dtype == ATK_F32 && !(p.stage2 && one_piece)) {
                const int64_t s512 = std::max<int64_t>(1, want_threads / (m * 512));
                if (p.L * p.G / (512 * s512) >= 32) { T = 256; lanes_per_wg = 512; }
            }
        }
    }
    // Stage 2 runs in this workgroup: it wants a lane for every two candidates (four at most, or it
    // falls back to the digit-by-digit selection), whatever the streaming part would be happy with
    if (p.stage2) {
        int t_s2 = (int)(ceil_div(ceil_div(b * k_b, 2), kWave) * kWave);
        if (t_s2 > 512) t_s2 = 512;
        // ... and a lane for every column group where one workgroup can still hold them all: narrow lanes (rows that are not
        // whole vectors: one column per lane) otherwise end up in two column blocks that meet through scratch and a ticket
        // (256 x 32000 bf16, k = 64, b = 501: 13.6 us in two column blocks of 256 lanes, 9.7 in one workgroup of 512)
        const int t_cols_s2 = (int)(ceil_div(p.G, kWave) * kWave);
        // (rows past 320 KB in batches that give every CU a workgroup of 256 stream faster in the two column blocks:
        // 128 x 128256 f32: 19.6 us, 23.6 in one workgroup of 512 per row)
        if (t_cols_s2 <= 512 && t_s2 < t_cols_s2 && (n * es <= (320 << 10) || 2 * m < (int64_t)kNumCU)) t_s2 = t_cols_s2;
        if (T < t_s2) T = t_s2;
    }
    // many column groups but few rows: smaller workgroups rather than row splits.  Not with Stage 2: there the
    // column blocks of a row have to meet in one workgroup again, through scratch and a ticket, and that workgroup
    // then selects from all candidates with few lanes (128 x 65536 f32, b = 2048: 21.0 us in two column blocks of 256
    // lanes, 12.0 in one workgroup of 512; k = 1000: 38.7 -> 16.0; bf16 b = 4096: 36.9 -> 18.7)
    if (p.G > 256 && !p.stage2)
        while (T > kWave && m * ceil_div(p.G, T) < (int64_t)kNumCU) T = (int)(ceil_div(T / 2, kWave) * kWave);  // whole wavefronts (T may be 384)
    if (T_forced) { T = T_forced; lanes_per_wg = 0; }
    if (T > t_max) T = t_max;

    // Long queues (k_b >= 5) on short buckets are bound by the chain of dependent selects of each
    // insertion: with one lane per column group and few column groups there are too few
    // independent chains per SIMD.  Then lanes share column groups inside the workgroup (P row
    // phases, merged once through LDS) until about one wavefront per SIMD is there (measured:
    // 14.3 -> 11.5 us at m = 32 on the 65536-long rows with k_b = 8; at m = 128 the merge costs more
    // than the extra lanes bring).
    int p_want = 1;
    if (p.KB >= 8 && p.G >= T && !T_forced)
        while (p_want < 4 && m * p.G * p_want < 64 * 4 * (int64_t)kNumCU && p.L >= 4 * p_want * 2) p_want <<= 1;
    // Queues without Stage 2 (b*k_b = k) on inputs that give the chip few lanes: more lanes of the workgroup share a column
    // group (merged once, in LDS) rather than row splits that meet through scratch - up to four wavefronts per SIMD where
    // every lane would own its column groups (two for k_b = 2, whose workgroups also share out the columns below), as
    // long as a lane keeps 16 matrix rows.  Eight slots and more cost a lane many insertions to fill its queues: only
    // on launches of under one wavefront per SIMD, down to 4*k_b rows per lane, also with fewer column groups than lanes
    // (then up to two wavefronts per SIMD).  Measured on 128 x 65536 f32, k = 4096: b = 1024, k_b = 4: 28.1 us in two splits,
    // 11.9 with four lanes a column group; b = 512, k_b = 8: 35.6 -> 19.4; b = 256, k_b = 16: 81.4 -> 44.4; k = 1024, b = 128,
    // k_b = 8: 46.1 -> 22.9; one row of 2^20, k = 4096, b = 1024, k_b = 4: 35.8 -> 8.9; k = 16384 on 128 rows (one lane per
    // column group fills the chip) stays as it is, and so do launches with more rows than that.
    // With Stage 2 behind them the same holds for eight slots and more from 2048 candidates on (128 x 65536 f32, k = 1024:
    // b = 128, k_b = 16: 106 -> 68 us; b = 512, k_b = 8: 151 -> 98; 8 x 2^18 bf16, b = 128, k_b = 16: 111 -> 71); with fewer
    // candidates the sweeps are mixed (8 x 2^18 f32, k = 256, b = 64, k_b = 16: 47 -> 66), and so they are in bf16 on rows past
    // 2^18 elements or past 256 buckets (128 x 65536, k = 1024, b = 512, k_b = 8: 96 -> 131), which stay as they were.
    const bool share_s2 = p.stage2 && p.KB >= 8 && b * k_b >= 2048 && (dtype == ATK_F32 || (n <= (1 << 18) && b <= 256));
    if (p.KB >= 2 && !T_forced && (p.stage2 ? share_s2 : (p.G >= T || p.KB >= 8))) {
        const int64_t min_rows = p.KB >= 8 ? 4 * p.KB : 16;
        const int64_t full = 256 * (int64_t)kNumCU;  // lanes of one wavefront per SIMD
        const int64_t target = p.KB <= 2 ? 2 * full : (p.G >= T ? 4 * full : 2 * full);
        auto lanes = [&](int pw) { return m * ceil_div(p.G, std::min<int64_t>(p.G, std::max(1, T / pw))) * T; };
        // A workgroup's piece of a matrix row gets shorter as lanes share column groups; pieces under 512 bytes (256 where
        // the insertions, not memory, bound the launch) stream badly once the input is more than the caches smooth over
        // (32 x 2^20 f32, k = 4096, b = 1024, k_b = 4: 53 us in row splits, 101 with sixteen lanes a column group and pieces of
        // 128 bytes); inputs of up to 8 MB take pieces down to 128 bytes (one row of 2^20: 35.8 -> 8.9 us).
        const int64_t piece_min = m * n * es <= (8 << 20) ? 128 : (p.KB >= 8 ? 256 : 512);
        const int64_t pw_max = std::max<int64_t>(1, (int64_t)T * p.V * es / piece_min);
        if (p.KB < 8 || lanes(1) < full) {
            int pw = 1;
            while (pw < 16 && 2 * pw <= pw_max && lanes(pw) < target && p.L / (2 * pw) >= min_rows) pw <<= 1;
            if (pw > p_want) p_want = pw;
        }
    }
    // Eight unpacked slots on long rows: sixteen lanes of the workgroup on a column (pieces of 128 bytes of a matrix
    // row per wavefront), which is what the pooled floors below need; the layout alone is faster too (128 x 2^20 f32,
    // k = 64, b = 128: 183 us with four lanes a column, 166 with sixteen, 151 with pooled floors; b = 256: 201 -> 154)
    // (with fewer than 128 workgroups before row splits the extra splits cost more: 16 x 2^20, b = 64: 50 -> 69 us)
    if (p.KB == 8 && dtype == ATK_F32 && !T_forced && T >= 256 && p.L >= 4096 && p.G >= T / 16 && p_want < 16 &&
        m * ceil_div(p.G, T / 16) >= 128)
        p_want = 16;
    const bool P_forced = ov.P != 0;
    if (P_forced) p_want = ov.P;

    // column groups side by side in a workgroup, row phases, LDS areas: for p_want lanes per column group
    int64_t lds = 0;
    auto layout = [&](int p_want) {
      for (;;) {
        p.Gw = (int)((p.G < T / p_want) ? p.G : T / p_want);
        p.P = T / p.Gw;
        if (p.P > p.L) p.P = (int)p.L;
        if (p.P < 1) p.P = 1;
        int t_used = (int)(ceil_div((int64_t)p.P * p.Gw, kWave) * kWave);
        if (t_used > T) t_used = T;
        p.T = t_used;
        p.wave_merge = p.P > 1 && p.Gw < kWave && (p.Gw & (p.Gw - 1)) == 0;
        p.nparts = p.wave_merge ? p.T / kWave : p.P;
        const int64_t lds_xch = (p.nparts > 1) ? (int64_t)p.nparts * std::min<int64_t>(b, (int64_t)p.Gw * p.V) * p.KB * 8 : 0;
        const int64_t lds_s2 = p.stage2 ? select_lds_bytes(b * k_b, (int)pow2_ceil(k)) : 0;
        if (p.stage2) {
            // candidates first; behind them the exchange area and, once that is dead, Stage 2's tables
            const int64_t cand_bytes = ceil_div(b * k_b * 8, 16) * 16;
            const int64_t tables = lds_s2 - b * k_b * 8;
            p.lds_cand_off = 16;
            p.lds_xch_off = (int)(16 + cand_bytes);
            lds = 16 + cand_bytes + (lds_xch > tables ? lds_xch : tables);
        } else {
            p.lds_xch_off = 16;
            p.lds_cand_off = (int)(16 + lds_xch);
            lds = 16 + lds_xch;
        }
        if (lds <= kLdsBudget || T <= kWave) break;
        T = (int)(ceil_div(T / 2, kWave) * kWave);
      }
      p.lds_bytes = (int)lds;
      T = p.T;
      p.colblocks = (int)ceil_div(p.G, p.Gw);
    };
    layout(p_want);
    if (p.stage2 && b * k_b > kStage2MaxCand) return ATK_ERR_UNSUPPORTED;
    if (lds > kLdsBudget) return ATK_ERR_UNSUPPORTED;

    // row splits for the layout just chosen
    auto row_splits = [&](bool strict_traffic = true) -> int64_t {
    int64_t base = m * p.colblocks;
    int64_t S = want_threads / (base * (lanes_per_wg ? lanes_per_wg : T));
    // every lane keeps at least 4 loads; a running maximum at least one full batch of 8 (one row of 2^20,
    // b = 64: 8.5 us with 128 splits of 4 loads per lane, 6.6 us with 64 of 8)
    int64_t s_rows = p.L / ((int64_t)p.P * (p.KB == 1 && !p.stage2 ? 8 : 4));  // (with Stage 2 more, shorter splits still measured faster)
    int64_t s_traffic = (p.L * es) / (32 * k_b);     // partial lists (written + read back) below half the bytes streamed
    // (a quarter for queues without Stage 2, whose lists are the whole output S times over: 128 x 2^18 f32, k = 16384,
    // b = 2048, k_b = 8: 145 us in two splits, 51 in one; 128 x 65536, k = 1024, b = 64, k_b = 16: 76.6 with 8, 42.1 with 4)
    if (p.KB >= 2 && !p.stage2 && strict_traffic) s_traffic /= 2;
    int64_t s_fill = ceil_div(kNumCU, base);         // splits that give every CU a workgroup
    if (S > s_traffic) S = s_traffic > s_fill ? s_traffic : (S < s_fill ? S : s_fill);  // filling the chip comes first
    if (S > s_rows) S = s_rows;
    // Two splits buy nothing once half the CUs have a big workgroup each (the memory system, not the
    // CU count, bounds a launch of this size), and cost the trip through scratch and the ticket
    // before Stage 2 can start: measured equal at b <= 512 and 1 us slower at b = 1024 on 128 x 65536.
    // Long rows are the other way round: there the second workgroup per row shortens the streaming
    // part by more than the trip costs (128 x 2^20 f32, b = 1024: 90.5 us in one piece, 84.2 in two;
    // the two are level at 2^18 elements in f32 and at 2^16 in bf16).
    // (Rows that a helper + finisher pair takes stay in one piece here: 128 x 2^20 f32, b = 1024: 83.6 us in two
    // halves, 76.9 as a pair; 2^19: 45.7 -> 41.1; bf16 2^18, b = 256: 19.3 -> 15.9.)
    if (S == 2 && p.stage2 && p.colblocks == 1 && ((base * T >= 256 * (int64_t)kNumCU && one_piece) || pair_rule)) S = 1;
    if (S == 2 && pair_out_rule && p.colblocks == 1) S = 1;
    if (S > 1 && out_one_rule && p.colblocks == 1) S = 1;
    // Short rows (up to 65536 elements) of a batch that leaves CUs idle: row splits through scratch and a ticket cost
    // more than they bring; one workgroup per row on the lean kernel, or a pair, is faster at every batch size (f32
    // n = 65536, k = 64: m = 1, b = 1024: 8.9 -> 6.6 us; m = 32: 11.1 -> 9.0; m = 64, b = 256: 9.7 -> 8.0; n = 32768:
    // 8.6 -> 6.2; bf16 m = 32, b = 512: 9.6 -> 7.5).  From 2^17 elements on the splits win (16 x 2^17: 9.3 against 10.6).
    // ... except that up to 32 such rows of more than 32768 elements with at most 512 buckets are better off still as three
    // helpers and a finisher on the lean kernel (below; f32 n = 65536: m = 1, b = 128: 7.1 us in one workgroup, 6.6 as a
    // pair, 5.6 in four; m = 32, b = 256: 7.7 -> 6.9; seven helpers are slower again from 256 buckets on)
    if (S > 1 && short_rule && p.colblocks == 1) S = (multi_short && S >= 4) ? 4 : 1;
    // The same on the general kernel (rows that are not whole aligned vectors, or b does not divide n): one slot per
    // bucket up to 65536 elements (f32 n = 50000: one row, b = 1024: 9.4 -> 6.5 us; 32 rows, b = 2048: 15.0 -> 11.7; 128
    // rows, b = 64: 9.2 -> 7.7), queues of several slots up to 16384 (512 x 16384 f32, b = 8, k_b = 8: 24.8 -> 20;
    // 128 x 16384 bf16, b = 32, k_b = 2: 7.5 -> 6.5); longer rows with queues are better off split (128 x 65536,
    // b = 8, k_b = 8: four splits are the fastest)
    if (S > 1 && p.KB == 1 && n <= 65536 && !lean_shape) S = 1;
    // (eight slots and more on fewer rows than half the CUs are bound by their insertions and want the lanes:
    // 8 x 16384 f32, b = 8, k_b = 8: 15.2 us in one workgroup, 11.3 in eight)
    if (S > 1 && p.KB >= 2 && n <= 16384 && (p.KB < 8 || n <= 4096 || 2 * m >= (int64_t)kNumCU)) S = 1;
    // Queues in front of Stage 2 on short rows: four splits per row give the last workgroup four lists per column to
    // fetch and merge before it can select; two measured faster once the rows alone fill half the chip (128 x 65536
    // f32: k = 512, b = 1024, k_b = 2: 24.0 -> 18.6 us; b = 512, k_b = 4: 25.1 -> 21.9; k = 64, b = 64, k_b = 8: 32.6 -> 29.3)
    if (S == 4 && p.stage2 && p.KB >= 2 && base * T >= 256 * (int64_t)kNumCU && n * es <= (256 << 10)) S = 2;
    {
        // The workgroup that draws the last ticket merges S lists per column, SU splits per batch
        // of loads, tpc lanes per column: keep that serial tail to about four batches.
        const int64_t tail_cols = p.stage2 ? b : std::min<int64_t>(b, (int64_t)p.Gw * p.V);
        auto batches = [&](int64_t s) {
            const int64_t tpc = tail_lanes_per_column(tail_cols, T, p.KB, s);
            return ceil_div(tail_cols, T / tpc) * ceil_div(s, tpc * tail_split_batch(p.KB));
        };
        while (S > 1 && batches(S) > 4) S = (S + 1) / 2;
        // Queues of eight and sixteen slots on few, long rows: there the insertions are what takes the time, and a lane
        // with a thousand matrix rows to itself costs more than the longer tail (one row of 2^20, b = 256, k_b = 16:
        // 411 us with 4 splits, 144 with 32; 16 rows of 2^18: 138 -> 102 with 8), so split down to about 128 matrix
        // rows per lane while that stays below one workgroup per CU
        // ... on rows of up to 2^18 elements no more splits than give the launch two wavefronts per SIMD: beyond that the
        // lists - S per column, k_b entries each, all through one workgroup at the end - cost more than the lanes bring
        // (128 x 65536 f32, k = 256, b = 32, k_b = 16: 67.3 us with 8 splits, 42 with 4; 512 x 32768, b = 16: 69.7 with 2, 50 with 1)
        // (inputs past 128 MB are bound by memory again and want the lanes: 512 x 2^18, b = 8, k_b = 8: 109 us in two splits, 137 in one)
        if (p.KB >= 8 && n <= (1 << 18) && m * n * es <= (1ll << 27)) {
            const int64_t s_lanes = std::max<int64_t>(1, 512 * (int64_t)kNumCU / (base * T));
            if (S > s_lanes) S = s_lanes;
        }
        if (p.KB >= 8) {
            int64_t s_long = p.L / ((int64_t)p.P * 128);
            if (s_long > 32) s_long = 32;
            if (s_long > s_rows) s_long = s_rows;
            while (s_long > S && base * s_long > (int64_t)kNumCU) s_long >>= 1;
            if (S < s_long) S = s_long;
        }
    }
    return S;
    };
    int64_t S = row_splits();
    // Many rows with few column groups came out above with workgroups of one or two wavefronts (a lane per column group
    // fills the chip) and may still get row splits on top - through scratch and a ticket, between workgroups of 64
    // lanes.  Bigger workgroups whose lanes share the columns do the same without memory in between (2048 x 16384 bf16,
    // k = 256, b = 64, k_b = 4: 35.0 -> 21 us; 2048 x 4096 f32, b = 32, k_b = 2: 11.6 -> 9.0; b = 8, k_b = 8: 27.2 -> 20)
    // (and so do 512 lanes instead of two workgroups of 256 with queues: 512 x 50000 f32, k = 1024, b = 256, k_b = 4:
    // 32.3 -> 23 us)
    // (what counts below 256 lanes is whether the lanes asked for are there, not whether the splits survived their caps)
    // (queues of eight slots and more are bound by insertions, and their splits' caps say how many lanes they want)
    // (... while a lane of the bigger workgroup still has sixteen matrix rows: 512 x 1024, k = 1024, b = 256, k_b = 4 has four a column)
    while (((T < 256 && (p.KB >= 8 ? S >= 2
                                   : (S >= 2 || (want_threads / (m * p.colblocks * (lanes_per_wg ? lanes_per_wg : T)) >= 2 &&
                                                 p.L / (2 * (int64_t)p.P) >= 16)))) ||
            (S >= 2 && T < 512 && S == 2 && p.KB >= 2)) && 2 * T <= t_max && !T_forced && !P_forced && !S_forced) {
        const int t_before = T;
        T *= 2;
        layout(p_want);
        if (lds > kLdsBudget) return ATK_ERR_UNSUPPORTED;
        S = row_splits();
        if (T <= t_before) break;  // (rows too short to give more lanes something to do)
    }
    // With Stage 2 the workgroups of a row meet in one of them whichever way the row is shared out; column blocks leave
    // that workgroup one candidate per column to fetch, row splits a list per split to merge first.  So few rows - up
    // to an eighth of the CUs' worth of workgroups - that would be split by rows, or fill under half the chip, share
    // out their columns instead (more lanes per column group, narrower workgroups) while that stays within one workgroup
    // per CU, 8 matrix rows per lane and pieces of 256 bytes of a matrix row; rows that the helpers + finisher plans
    // take (below) are left to them.  Measured (f32): 4 x 2^22, k = 64, b = 4096: 139 -> 25 us; one row of 2^20, b = 1024: 14.1 -> 11.6;
    // 8 x 2^20: 16.0 -> 13.7; one row of 2^24, b = 128: 34.0 -> 22.7; 32 x 128256, k = 256, b = 2048: 16.3 -> 13.2; 8 x 151936,
    // k = 256, b = 512, k_b = 2: 15.3 -> 10.2; 128 rows keep their plans (128 x 2^18, b = 2048: 27.7 us, 32 and more with column blocks).
    // (Not for matrix rows that do not start on 128-byte lines - pieces would straddle lines, read once by each of two
    // workgroups: 32 x 2^22, b = 500: 81 -> 119 us; a plan that needs no scratch as it is - one workgroup per row - only on
    // rows of 2 MB and more: 64 x 65536 bf16, k = 256, b = 2048: 9.7 us in one workgroup, 12.8 in column blocks; pieces of 512
    // bytes at least once the input is more than the caches smooth over.)
    if (p.stage2 && p.KB <= 4 && !T_forced && !P_forced && !S_forced && m * p.colblocks * 8 <= (int64_t)kNumCU &&
        (b * es) % 128 == 0 && (S >= 2 || (m * p.colblocks * 2 < (int64_t)kNumCU && n * es >= (2 << 20)))) {
        const bool to_helpers = p.KB == 1 && lean_shape && allow_pair && ov.hf >= 0 && ov.mh >= 0 && !ov.lm_off && !ov.ln_off &&
                                T <= 512 && p.colblocks == 1 && S >= 2 && (S - 1) * (int64_t)p.Gw * p.V <= (int64_t)kMultiSlots * T;
        if (!to_helpers) {
            int pw = std::max(1, T / std::max(1, p.Gw));  // lanes on a column group now
            const int pw0 = pw;
            auto blocks = [&](int q) { return ceil_div(p.G, std::min<int64_t>(p.G, std::max(1, T / q))); };
            while (pw < 16 && m * blocks(2 * pw) <= (int64_t)kNumCU && p.L / (2 * pw) >= 8 &&
                   (int64_t)(T / (2 * pw)) * p.V * es >= (m * n * es > (8 << 20) ? 512 : 256))
                pw <<= 1;
            if (pw > pw0 && blocks(pw) > p.colblocks) {
                layout(pw);
                if (lds > kLdsBudget) return ATK_ERR_UNSUPPORTED;
                S = row_splits();
            }
        }
    }
    // Without Stage 2 nothing ties the columns of a row together, and a workgroup that owns whole
    // buckets needs no hand-over at all: as long as rows would be split, and a workgroup's piece of
    // a matrix row stays 128 bytes or more, halve the workgroup's column groups instead (measured on
    // 128 x 65536 f32, b = 64: 9.3 -> 8.2 us; one row of 2^20: 10.8 -> 6.6 us).
    // Only for rows that start on 128-byte lines: pieces that straddle lines are read twice, once by each
    // of the two workgroups (n = 100003: 15.2 -> 17.5 us).
    // Queues of two slots take it the same way (128 x 65536, b = 128, k_b = 2: 11.8 -> 9.3 us); with four
    // slots the lanes that the row splits would have added are worth more as soon as rows get longer
    // (2^18: 32.6 us with the splits, 38.9 without; 2^20: 100 against 119), so only up to 256 KB per row
    // (128 x 65536, b = 256, k_b = 4: 15.8 -> 12.1 us).
    if ((p.KB <= 2 || (p.KB == 4 && n * es <= (256 << 10))) && !p.stage2 && p.P > 1 && !P_forced && !S_forced &&
        (n * es) % 128 == 0) {
        int gw = p.Gw;
        // (how far the columns are shared out goes by the splits that the looser bound on the lists' traffic allows)
        int64_t s = std::max(S, row_splits(false)), cb = p.colblocks;
        // ... and as long as the launch has fewer workgroups than the chip has CUs (rows that allow no
        // more splits: 64 x 128256 bf16, b = 256 came out with 128 workgroups)
        while ((s >= 2 || m * cb * s < (int64_t)kNumCU) && (gw & 1) == 0 && (int64_t)(gw / 2) * p.V * es >= 128 &&
               p.G % (gw / 2) == 0) {
            gw >>= 1;
            cb <<= 1;
            s = s >= 2 ? s >> 1 : 1;
        }
        if (gw != p.Gw) {
            // f32: the narrower workgroup also does better with four wavefronts than with eight (few rows of
            // 65536: 7.3 -> 6.0 us at m = 32; level at m = 128); it still counts as 512 lanes for the splits
            if (dtype == ATK_F32 && T == 512 && !T_forced) {
                T = 256;
                lanes_per_wg = 512;
            }
            layout(T / gw);
            if (lds > kLdsBudget) return ATK_ERR_UNSUPPORTED;
            S = row_splits();
        }
    }
    // One slot per bucket on rows of whole aligned vectors, where the plan so far splits rows: the splits of a row (and
    // column block) run as helpers and a finisher on the lean kernel (atk_lean_kernel.h, kLeanMulti) instead of meeting
    // through partial lists, a fence and a ticket.  Every workgroup but the last takes the same whole number of row
    // phases' worth of matrix rows, the last one - the finisher - what is left, at least one row per phase.
    int helpers = 0;
    int64_t helper_rows = 0;
    const bool multi_ok = p.KB == 1 && allow_pair && ov.hf >= 0 && ov.mh >= 0 && !ov.lm_off && !ov.ln_off && ptr16 &&
                          p.V == 16 / es && n % b == 0 && (n * es) % 16 == 0 && !S_forced && T <= 512 &&
                          (!p.stage2 || p.colblocks == 1);
    // Queues of two to four slots without Stage 2: the workgroup that draws the last ticket merges S lists of (its
    // columns) x k_b entries, so the splits that pay grow with the square root of the row's length over that, and beyond 32
    // the tickets and the fetch of that many lists cost more than shorter streams save whatever the lists' size - unless
    // a split would then stream more than 128 KB, which few workgroups cannot pull fast enough (f32, k = 1024, b = 256,
    // k_b = 4: 8 x 2^17: 18.0 us with 32 splits, 12.3 with 8; 8 x 2^18: 19.1 -> 15.1 with 16; k = 64, b = 32, k_b = 2, one
    // row of 2^20: 15.7 with 256 splits, 11.2 with 32, but 2^22: 17.6 with 256, 25.5 with 32)
    if (p.KB >= 2 && p.KB <= 4 && !p.stage2 && !S_forced) {
        const int64_t cols = std::min<int64_t>(b, (int64_t)p.Gw * p.V);
        int64_t s_tail = (int64_t)(0.75 * std::sqrt((double)n / (double)(cols * k_b)));
        if (s_tail > 32) s_tail = 32;
        const int64_t s_stream = n * es / (128 << 10);
        if (s_tail < s_stream) s_tail = s_stream;
        if (s_tail < 1) s_tail = 1;
        if (S > s_tail) S = s_tail;
        // (a launch just over one workgroup per CU runs as two rounds: 32 x 2^18, k = 1024, b = 256, k_b = 4: 22.6 us
        // with 12 or 16 splits, 18.2 with 8)
        const int64_t per = m * p.colblocks;
        if (per * S > (int64_t)kNumCU && per * S < 2 * (int64_t)kNumCU && per <= (int64_t)kNumCU) S = (int64_t)kNumCU / per;
    }
    if (multi_ok && ov.mh > 0) S = ov.mh + 1;  // (sweeps and tests; clamped like any other count below)
    if (S_forced) S = S_forced;
    if (S > p.L / p.P) S = p.L / p.P;
    if (S < 1) S = 1;
    int64_t rps = ceil_div(p.L, S);
    rps = ceil_div(rps, p.P) * p.P;
    S = ceil_div(p.L, rps);
    if (multi_ok && S > 1 && (S - 1) * (int64_t)p.Gw * p.V <= (int64_t)kMultiSlots * T) {
        int64_t lh = ceil_div(p.L, S * p.P) * p.P;
        if (p.L - (S - 1) * lh < p.P) lh = p.L / (S * p.P) * p.P;
        if (lh >= p.P && p.L - (S - 1) * lh >= p.P) {
            helpers = (int)S - 1;
            helper_rows = lh;
            S = 1;
            rps = ceil_div(p.L, p.P) * p.P;
        }
    }
    p.S = (int)S;
    p.rows_per_split = (int)rps;

    p.packed = dtype == ATK_BF16 && p.KB >= 4 && p.rows_per_split + 2 < 32768 && !ov.pk_off;
    // Eight unpacked slots with many lanes of the workgroup on a column, each with many matrix rows: what a lane has
    // seen alone is a poor bound on what still matters (after t rows one element in t/8 still enters its queue, and
    // with 128 lane-columns per wavefront some lane always needs the insertion), so the lanes of a column pool their
    // queues - after 8 load batches, then 16, 32, ... - and raise their floors to the eighth best of all.  Measured on
    // 128 x 2^20 f32, k_b = 8: b = 8 (64 lanes a column) 162 -> 116 us, b = 16 (32 lanes) 163 -> 129, b = 32 (16 lanes)
    // 164 -> 151; with 8 lanes a column or fewer, or under 256 rows a lane, the pooling costs more than it saves.
    p.refresh = 0;
    if (p.KB == 8 && !p.packed && n % p.V == 0 && ov.rf >= 0 && p.P > 1 &&
        (ov.rf > 0 || (p.P >= 16 && p.rows_per_split / p.P >= 256)))
        p.refresh = ov.rf > 0 ? ov.rf : 8;
    p.tail_tpc = tail_lanes_per_column(p.stage2 ? b : std::min<int64_t>(b, (int64_t)p.Gw * p.V), p.T, p.KB, p.S);
    p.direct = (p.P == 1 && p.S == 1 && !p.stage2 && helpers == 0);
    p.use_scratch = (p.S > 1) || (p.stage2 && p.colblocks > 1);
    if (p.use_scratch && p.stage2) {
        // the candidates are gathered by the last workgroup of the row, after its exchange area
        // is dead, so the two share LDS (without splits emit() fills one while the other is read)
        const int64_t lds_xch = (p.nparts > 1) ? (int64_t)p.nparts * std::min<int64_t>(b, (int64_t)p.Gw * p.V) * p.KB * 8 : 0;
        const int64_t lds_s2 = select_lds_bytes(b * k_b, (int)pow2_ceil(k));
        p.lds_cand_off = 16;
        p.lds_xch_off = 16;
        p.lds_bytes = (int)(16 + (lds_xch > lds_s2 ? lds_xch : lds_s2));
    }

    // One slot per bucket and no hand-over through memory: the lanes meet in LDS by atomic maximum, in the
    // candidate array itself (no exchange area); Stage 2's tables sit behind it.
    p.lds_max = p.KB == 1 && !p.use_scratch && !p.direct && !ov.lm_off;
    if (p.lds_max) {
        const int64_t wcols = std::min<int64_t>(b, (int64_t)p.Gw * p.V);
        p.lds_cand_off = 16;
        p.lds_xch_off = 16;
        p.lds_bytes = (int)(16 + (p.stage2 ? select_lds_bytes(b, (int)pow2_ceil(k)) : ceil_div(wcols * 8, 16) * 16));
    }
    // one ticket per row with Stage 2, else one per (row, column block)
    p.scratch_ticket_bytes = p.use_scratch ? m * (p.stage2 ? 1 : p.colblocks) * kTicketStride * 4 : 0;
    p.scratch_lists_bytes = p.use_scratch ? m * p.S * b * k_b * 8 : 0;
    p.grid = m * p.S * p.colblocks;
    if (p.grid >= (1ll << 31)) return ATK_ERR_UNSUPPORTED;
    // Stage 2's short form takes its bins' lower end from the merge: tight when some wavefront covers every column
    // (its minimum bounds the smallest candidate), else only as tight as the smallest value any lane holds -
    // good enough once every lane has seen a few dozen rows
    // (A lane that has seen few rows holds a negative maximum now and then - one lane-column in 2^rows on centred data -
    // and a bound at or below zero stretches the bins over every exponent there is: all candidates land in a few bins
    // and the selection falls back to digit by digit.  With a wavefront's cover bound it takes such a lane in every
    // wavefront; measured with 8 rows per lane: bf16 128 x 32768, b = 256: 10.7 us, 6.5 with the range taken from the
    // merged candidates instead; f32 128 x 8192, b = 128: 7.5 -> 5.2; level from 16 rows per lane.)
    p.bound_ok = p.lds_max && p.stage2 && ((p.Gw <= kWave && p.L / p.P >= 16) || p.L / p.P >= 24) && !ov.bo_off;
    // Rows of whole, aligned 16-byte vectors with one slot per bucket and one workgroup per row or column
    // block: the lean kernels (same mapping, nothing else in the kernel).
    p.lean = p.lds_max && ptr16 && p.V == 16 / es && n % b == 0 && (n * es) % 16 == 0 && p.S == 1 && p.T <= 512 && !ov.ln_off;
    p.pair_rows = 0;
    p.helpers = 0;
    if (helpers > 0) {
        if (!p.lean) return ATK_ERR_UNSUPPORTED;  // never: multi_ok holds what the lean kernels ask for
        p.pair_rows = (int)helper_rows;
        p.helpers = helpers;
        p.grid = m * p.colblocks * (helpers + 1);
        if (p.grid >= (1ll << 31)) return ATK_ERR_UNSUPPORTED;
        // the mailboxes: per (row, column block) one per helper, a composite per column of the block, zero between calls
        p.scratch_ticket_bytes = m * p.colblocks * helpers * (int64_t)p.Gw * p.V * 8;
        p.bound_ok = p.stage2 && helper_rows >= 16 && !ov.bo_off;  // (the first helper's mailbox is a bound, a column's maximum over that many rows)
    }
    if (p.lean && p.stage2 && ov.sl && ov.sl >= p.Gw && ov.sl <= p.T) p.P = ov.sl / p.Gw;  // SL=<lanes that stream> (sweeps)
    if (p.lean && helpers == 0 && p.colblocks == 1 && allow_pair && ov.hf >= 0 && (p.stage2 ? (ov.hf > 0 || pair_rule) : pair_out_rule)) {
        // Two workgroups per row (helper + finisher, see atk_lean_kernel.h) while that still leaves every workgroup a CU of
        // its own, on rows long enough to be worth a second CU.  What the memory system likes is four streaming
        // wavefronts per CU on all CUs (128 x 65536 f32: 256 workgroups of 256 lanes have their rows in 1.1 us before
        // 128 of 512 do, and 256 of 512 are slower than either), so the pair streams with 256 lanes per workgroup: up to
        // 256 buckets in workgroups of 256 lanes with the rows split in half (b = 128: 9.9 -> 9.1 us, b = 256: 10.0 ->
        // 9.4 us), up to 512 buckets in workgroups of 512 lanes (Stage 2 wants a lane per candidate) of which 256 stream,
        // (10.2 -> 9.6 us).  The two take half the matrix rows each: the finisher has Stage 2 to run, but a helper
        // with less than half measured slower all the same (b = 512: 9.97 us at 30/64 or 34/64, 9.62 at half; bf16
        // 8.87 against 8.00).  bf16 lanes do twice the work per load, and on rows from 2^18 elements all 512 stream
        // (2^20, b = 256: 48.4 us with 256, 42.6 with 512; 2^17: 10.4 against 10.9).
        int t_pair = b <= 256 ? 256 : 512, lanes = 256, share = 32;
        if (dtype == ATK_BF16 && n >= (1 << 18)) t_pair = lanes = 512;
        if (ov.ht && ov.ht % kWave == 0 && ov.ht <= 512) t_pair = ov.ht;
        if (ov.sl) lanes = ov.sl;
        if (ov.hq) share = ov.hq;
        if (lanes > t_pair) lanes = t_pair;
        if (t_pair >= p.Gw && lanes >= p.Gw) {
            const int P = lanes / p.Gw;
            const int64_t unit = P;
            const int64_t lh = p.L * share / 64 / unit * unit;
            if (lh > 0 && p.L - lh >= unit && b <= (int64_t)kBkSlots * t_pair && 2 * m < (1ll << 31)) {
                p.T = t_pair;
                p.P = P;
                p.pair_rows = (int)lh;
                p.grid = 2 * m;
                p.scratch_ticket_bytes = m * b * 8;  // the mailbox: one composite per bucket, zero between calls
                p.bound_ok = lh >= 16 && !ov.bo_off;  // (the mailbox is the bound: a column's maximum over that many rows)
            }
        }
    }
    *pl = p;
    return ATK_OK;
}

// ------------------------------------------------------------------------------------ contiguous plan
// Gs lanes per bucket, chosen so that a lane has about 8 loads while the launch still has
// enough lanes for the chip; buckets longer than a workgroup can chew are also split.
int make_contig_plan(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, bool ptr16, Plan *pl) {
    const int es = (dtype == ATK_F32) ? 4 : 2;
    Plan p;
    memset(&p, 0, sizeof p);
    p.assignment = ATK_CONTIGUOUS;
    p.dtype = dtype;
    p.m = m;
    p.n = n;
    p.k = k;
    p.b = b;
    p.k_b = (int)k_b;
    p.KB = (int)pow2_ceil(k_b);
    p.L = n / b;
    p.stage2 = b * k_b > k;
    const int vfull = 16 / es;
    p.V = (ptr16 && n % b == 0 && p.L % vfull == 0) ? vfull : 1;
    const int T_forced = plan_override().T, S_forced = plan_override().S, V_forced = plan_override().V;
    if (V_forced == 1) p.V = 1;
    const int t_max = max_threads_for_kb(p.KB);
    const int64_t chunks = ceil_div(n, b) / p.V;  // of the longest bucket (V > 1: of every bucket)
    const int64_t want_lanes = 512 * (int64_t)kNumCU;
    if (chunks <= kWave) {
        // Short buckets: as many lanes per bucket as it has loads (rounded up to a power of two),
        // so that a wavefront reads one contiguous stretch, and NB buckets per lane group in turn.
        int64_t Gs = pow2_ceil(chunks);
        int T = T_forced ? T_forced : (p.stage2 ? 512 : 256);  // (measured: Stage 2 likes the bigger workgroup)
        if (T > t_max) T = t_max;
        const int64_t need = ceil_div(b * Gs, kWave) * kWave;  // lanes that cover one row's buckets
        if (need < T) T = (int)need;
        const int bpw = T / (int)Gs;
        int64_t NB = (m * b * Gs) / (2 * want_lanes);
        if (NB > 8) NB = 8;
        if (NB > ceil_div(b, bpw)) NB = ceil_div(b, bpw);
        if (NB < 1) NB = 1;
        p.Gs = (int)Gs;
        p.T = T;
        p.NB = (int)NB;
        p.bblocks = (int)ceil_div(b, bpw * NB);
        p.S = 1;
        p.chunks_per_split = (int)chunks;
        p.use_scratch = p.stage2 && p.bblocks > 1;
        p.tail_tpc = 1;
        if (p.stage2 && b * k_b > kStage2MaxCand) return ATK_ERR_UNSUPPORTED;
        const int64_t lds_s2 = p.stage2 ? select_lds_bytes(b * k_b, (int)pow2_ceil(k)) : 0;
        p.lds_xch_off = 16;
        p.lds_cand_off = 16;
        p.lds_bytes = (int)(16 + lds_s2);
        if (p.lds_bytes > kLdsBudget) return ATK_ERR_UNSUPPORTED;
        p.scratch_ticket_bytes = p.use_scratch ? m * kTicketStride * 4 : 0;
        p.scratch_lists_bytes = p.use_scratch ? m * b * k_b * 8 : 0;
        p.grid = m * p.bblocks;
        if (p.grid >= (1ll << 31)) return ATK_ERR_UNSUPPORTED;
        *pl = p;
        return ATK_OK;
    }
    int64_t Gs = 1;
    while (Gs * 2 <= t_max && Gs * 16 <= chunks) Gs <<= 1;                          // about 8..16 loads per lane
    while (Gs * 2 <= t_max && Gs * 2 <= chunks && m * b * Gs < want_lanes) Gs <<= 1;  // more lanes, down to one load each
    if (T_forced && Gs > T_forced) Gs = T_forced;
    if (Gs > kWave && Gs < 256 && !T_forced) Gs = (chunks >= 256 && t_max >= 256) ? 256 : kWave;
    int T;
    if (Gs > kWave) {
        T = (int)Gs;  // a whole workgroup per bucket
    } else {
        T = T_forced ? T_forced : 256;
        if (T > t_max) T = t_max;
        const int64_t need = ceil_div(b * Gs, kWave) * kWave;  // lanes that cover one row's buckets
        if (need < T) T = (int)need;
    }
    p.Gs = (int)Gs;
    p.T = T;
    const int bpw = T / p.Gs;
    p.bblocks = (int)ceil_div(b, bpw);
    int64_t S = 1;
    if (p.Gs == T) {
        S = want_lanes / (m * b * T);
        const int64_t s_loads = chunks / ((int64_t)T * 4);  // every lane keeps at least 4 loads
        if (S > s_loads) S = s_loads;
    }
    if (S_forced && p.Gs == T) S = S_forced;
    if (S > chunks) S = chunks;
    if (S < 1) S = 1;
    int64_t cps = ceil_div(chunks, S);
    S = ceil_div(chunks, cps);
    p.S = (int)S;
    p.chunks_per_split = (int)cps;
    p.use_scratch = (S > 1) || (p.stage2 && p.bblocks > 1);
    p.tail_tpc = tail_lanes_per_column(p.stage2 ? b : std::min<int64_t>(b, bpw), T, p.KB, S);
    p.direct = false;
    if (p.stage2 && b * k_b > kStage2MaxCand) return ATK_ERR_UNSUPPORTED;
    const int64_t lds_xch = (p.Gs > kWave) ? (int64_t)(T / kWave) * p.KB * 8 : 0;
    const int64_t lds_s2 = p.stage2 ? select_lds_bytes(b * k_b, (int)pow2_ceil(k)) : 0;
    p.lds_xch_off = 16;
    p.lds_cand_off = (int)(16 + lds_xch);
    p.lds_bytes = (int)(16 + lds_xch + lds_s2);
    if (p.lds_bytes > kLdsBudget) return ATK_ERR_UNSUPPORTED;
    p.scratch_ticket_bytes = p.use_scratch ? m * (p.stage2 ? 1 : p.bblocks) * kTicketStride * 4 : 0;
    p.scratch_lists_bytes = p.use_scratch ? m * p.S * b * k_b * 8 : 0;
    p.grid = m * p.S * p.bblocks;
    if (p.grid >= (1ll << 31)) return ATK_ERR_UNSUPPORTED;
    *pl = p;
    return ATK_OK;
}

int make_plan(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, Plan *pl) {
    return make_plan_aligned(m, n, k, b, k_b, dtype, true, pl);
}

// ------------------------------------------------------------------------------------ scratch pool
// Two grow-only allocations per device: `state` (tickets and other words that every kernel
// leaves zeroed, so that the next call can rely on zeros) and `data` (partial lists and
// other buffers that carry nothing from call to call).  Both are zero-filled when
// (re)allocated.  They are kept apart so that one call's data can never alias what a later
// call, with other sizes, takes for zeroed state.
static std::mutex g_pool_mu;
enum { kPoolState = 0, kPoolData = 1 };
static void *g_pool_ptr[64][2];
static size_t g_pool_bytes[64][2];
static hipStream_t g_pool_stream[64];  // the stream of the last call that took a pool on the device
static bool g_pool_stream_set[64];

// The pools are per device, not per stream: work queued on one stream may still be using them when a call arrives
// on another.  Such a call first waits, on the host, for the stream of the call before it (calls that stay on one
// stream never wait: their kernels are ordered by the stream).
static hipError_t get_pool(int which, size_t bytes, void **out, hipStream_t stream) {
    *out = nullptr;
    if (bytes == 0) return hipSuccess;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_pool_mu);
    if (g_pool_stream_set[dev] && g_pool_stream[dev] != stream) {
        if (hipStreamSynchronize(g_pool_stream[dev]) != hipSuccess) {  // (the stream may be gone by now)
            (void)hipGetLastError();
            e = hipDeviceSynchronize();
            if (e != hipSuccess) return e;
        }
    }
    g_pool_stream[dev] = stream;
    g_pool_stream_set[dev] = true;
    if (g_pool_bytes[dev][which] < bytes) {
        if (g_pool_ptr[dev][which]) {
            e = hipFree(g_pool_ptr[dev][which]);  // waits for work that may still use it
            g_pool_ptr[dev][which] = nullptr;
            g_pool_bytes[dev][which] = 0;
            if (e != hipSuccess) return e;
        }
        size_t want = bytes + bytes / 4;
        if (which == kPoolState && want < 64 * 1024) want = 64 * 1024;
        void *p = nullptr;
        e = hipMalloc(&p, want);
        if (e != hipSuccess) return e;
        e = hipMemset(p, 0, want);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) {
            (void)hipFree(p);
            return e;
        }
        g_pool_ptr[dev][which] = p;
        g_pool_bytes[dev][which] = want;
    }
    *out = g_pool_ptr[dev][which];
    return hipSuccess;
}

// ------------------------------------------------------------------------------------ fixed scratch
// Scratch of the allocation-free entry point: one array per device that the library runs on, part of the
// code object, so it is there (zero-filled) when the module is loaded and stays until the process ends.
// The first ATK_NOALLOC_STATE_BYTES hold the tickets, the rest the partial lists.
static __device__ __align__(256) unsigned char scratch[ATK_NOALLOC_SCRATCH_BYTES];
// The array's name is a host-side stand-in, not a device address: the address on each device comes from
// hipGetSymbolAddress, once per device, with that device current, and only that pointer is used afterwards.
static void *g_fixed_scratch[64];
static hipError_t fixed_scratch(void **out) {
    *out = nullptr;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_pool_mu);
    if (!g_fixed_scratch[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_fixed_scratch[dev] = p;
    }
    *out = g_fixed_scratch[dev];
    return hipSuccess;
}

// zero fill (a kernel, not a memset: a caller may be capturing the stream into a graph)
__global__ void __launch_bounds__(256) fill_zero_kernel(uint4 *p, int64_t n_vec) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_vec) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// ------------------------------------------------------------------------------------ utilities
__global__ void __launch_bounds__(256) read_ceiling_kernel(const uint4 *x, int64_t n_vec, int64_t slab, u64 *sink) {
    // every workgroup streams one contiguous slab, eight 16-byte loads per lane in flight
    const int64_t lo = (int64_t)blockIdx.x * slab, hi = lo + slab < n_vec ? lo + slab : n_vec;
    int64_t i = lo + threadIdx.x;
    uint32_t acc = 0;
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    const v4u *px = (const v4u *)x;
    for (; i + 7 * 256 < hi; i += 8 * 256) {
        v4u v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(px + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < hi; i += 256) {
        v4u v = __builtin_nontemporal_load(px + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc ^= __shfl_xor(acc, off, 64);
    // one word per wave, no contended atomics: sink holds gridDim.x * 4 words
    if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = acc;
}

// plain copy of n_vec 16-byte words: known read and write volume, used to scale hardware counters
__global__ void __launch_bounds__(256) copy_kernel(const uint4 *src, uint4 *dst, int64_t n_vec) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

__global__ void sleep_kernel(int64_t ticks, u64 *unused) {
    // wall_clock64() counts at a fixed 100 MHz; the loop ends after `ticks` of it.
    const u64 start = wall_clock64();
    while ((int64_t)(wall_clock64() - start) < ticks) __builtin_amdgcn_s_sleep(32);
    (void)unused;
}

}  // namespace atk

using namespace atk;

// ====================================================================================== C ABI
extern "C" {

const char *atk_strerror(int code) {
    switch (code) {
        case ATK_OK: return "ok";
        case ATK_ERR_NULL_PTR: return "a required pointer is NULL";
        case ATK_ERR_BAD_SHAPE: return "m, n or k out of range (need m,n,k >= 1, k <= n, n < 2^31)";
        case ATK_ERR_BAD_PARAMS: return "b, k_b must satisfy 1 <= b <= n, 1 <= k_b <= min(k, n/b), b*k_b >= k";
        case ATK_ERR_UNSUPPORTED: return "parameters are legal for the method but not supported by this library";
        case ATK_ERR_DTYPE: return "dtype must be ATK_F32 (0) or ATK_BF16 (1)";
        case ATK_ERR_HIP: return "a HIP runtime call failed";
        case ATK_ERR_ALIGN: return "a pointer is not aligned to its element size";
        case ATK_ERR_WORKSPACE: return "the call needs more scratch than the allocation-free entry point holds (ATK_NOALLOC_SCRATCH_BYTES)";
    }
    return "unknown error code";
}

int atk_last_hip_error(void) { return g_last_hip_error; }

// ---- the whole call: Stage 1 (+ fused Stage 2), or Stage 1 into scratch followed by the long-row
// exact selection over the candidates when there are more of them than one workgroup holds
struct FullPlan {
    Plan s1;
    bool two_step;
    ExactPlan ex;            // two_step: selection over the b*k_b candidates of (a block of) the rows
    int64_t cand_vals_off;   // byte offsets into the data pool
    int64_t cand_idx_off;
    int64_t ex_data_off;
    int64_t ex_state_off;    // byte offset into the state pool
    int64_t state_bytes, data_bytes;
};
static const int64_t kExactRowsPerPass = 65535;  // long rows are the y dimension of their grids
static int64_t align256(int64_t v) { return (v + 255) / 256 * 256; }

// Plan of exact_topk over m rows: `first` is the plan of the first block of rows (all rows when the
// rows go one per workgroup), and the pool sizes cover every block.  The last block has fewer rows and
// is planned on its own by run_exact(): with fewer rows it may take paths the full blocks do not (the
// copy-out buffer, a finer sweep), so its needs are not bounded by the first block's.
static int make_exact_plans(int64_t m, int64_t n, int64_t k, int dtype, ExactPlan *first, int64_t *state_bytes,
                            int64_t *data_bytes) {
    int rc = make_exact_plan(m > kExactRowsPerPass ? kExactRowsPerPass : m, n, k, dtype, first);
    if (rc == ATK_OK && first->single_wg) rc = make_exact_plan(m, n, k, dtype, first);
    if (rc != ATK_OK) return rc;
    *state_bytes = first->state_bytes;
    *data_bytes = first->scratch_bytes;
    if (!first->single_wg && m > kExactRowsPerPass && m % kExactRowsPerPass) {
        ExactPlan last;
        rc = make_exact_plan(m % kExactRowsPerPass, n, k, dtype, &last);
        if (rc != ATK_OK) return rc;
        *state_bytes = std::max(*state_bytes, last.state_bytes);
        *data_bytes = std::max(*data_bytes, last.scratch_bytes);
    }
    return ATK_OK;
}

static int make_full_plan(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, int assignment,
                          bool ptr16, FullPlan *fp, bool allow_pair = true) {
    if (assignment != ATK_INTERLEAVED && assignment != ATK_CONTIGUOUS) return ATK_ERR_BAD_PARAMS;
    const int es = (dtype == ATK_F32) ? 4 : 2;
    const int64_t nc = b * k_b;
    fp->two_step = nc > k && nc > kStage2MaxCand;
    const int64_t k1 = fp->two_step ? nc : k;  // two steps: Stage 1 writes all its candidates, bucket by bucket
    int rc = (assignment == ATK_CONTIGUOUS) ? make_contig_plan(m, n, k1, b, k_b, dtype, ptr16, &fp->s1)
                                            : make_plan_aligned(m, n, k1, b, k_b, dtype, ptr16, &fp->s1, allow_pair);
    if (rc != ATK_OK) return rc;
    fp->state_bytes = fp->s1.scratch_ticket_bytes;
    fp->data_bytes = fp->s1.scratch_lists_bytes;
    if (!fp->two_step) return ATK_OK;
    int64_t ex_state = 0, ex_data = 0;
    rc = make_exact_plans(m, nc, k, dtype, &fp->ex, &ex_state, &ex_data);
    if (rc != ATK_OK) return rc;
    fp->ex.idx_n = n;
    fp->cand_vals_off = align256(fp->s1.scratch_lists_bytes);
    fp->cand_idx_off = fp->cand_vals_off + align256(m * nc * es);
    fp->ex_data_off = fp->cand_idx_off + align256(m * nc * 4);
    fp->ex_state_off = align256(fp->s1.scratch_ticket_bytes);
    fp->data_bytes = fp->ex_data_off + ex_data;
    fp->state_bytes = fp->ex_state_off + ex_state;
    return ATK_OK;
}

// exact selection over the rows of x (values) / xi (their indices, or NULL), in blocks of rows
// state_cap, data_cap: bytes of the two scratch areas (make_exact_plans() sized them for every block)
static int run_exact(const ExactPlan &first, const void *x, const int32_t *xi, int64_t m, int64_t n, int64_t k, int dtype,
                     void *out_vals, int32_t *out_idx, void *state, int64_t state_cap, void *data, int64_t data_cap,
                     hipStream_t stream) {
    const int es = (dtype == ATK_F32) ? 4 : 2;
    if (first.single_wg) {  // one workgroup per row, rows along x: no limit on m
        hipError_t e = launch_exact(first, x, xi, out_vals, out_idx, state, data, stream);
        return e == hipSuccess ? ATK_OK : hip_fail(e);
    }
    for (int64_t r0 = 0; r0 < m; r0 += kExactRowsPerPass) {
        ExactPlan pl = first;
        if (m - r0 < pl.m) {
            int rc = make_exact_plan(m - r0, n, k, dtype, &pl);
            if (rc != ATK_OK) return rc;
            pl.idx_n = first.idx_n;
        }
        if (pl.state_bytes > state_cap || pl.scratch_bytes > data_cap) return ATK_ERR_UNSUPPORTED;  // never: a planning mistake must not become a stray write
        hipError_t e = launch_exact(pl, (const unsigned char *)x + r0 * n * es, xi ? xi + r0 * n : nullptr,
                                    (unsigned char *)out_vals + r0 * k * es, out_idx + r0 * k, state, data, stream);
        if (e != hipSuccess) return hip_fail(e);
    }
    return ATK_OK;
}

static int run_approx(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, int assignment,
                      void *out_vals, int32_t *out_idx, void *stream, void *trace = nullptr, int64_t trace_bytes = 0) {
    if (!x || !out_vals || !out_idx) return ATK_ERR_NULL_PTR;
    int rc = check_approx(m, n, k, b, k_b, dtype);
    if (rc != ATK_OK) return rc;
    if (assignment != ATK_INTERLEAVED && assignment != ATK_CONTIGUOUS) return ATK_ERR_BAD_PARAMS;
    const int es = (dtype == ATK_F32) ? 4 : 2;
    if (((uintptr_t)x | (uintptr_t)out_vals) & (uintptr_t)(es - 1)) return ATK_ERR_ALIGN;
    if ((uintptr_t)out_idx & 3u) return ATK_ERR_ALIGN;
    FullPlan fp;
    rc = make_full_plan(m, n, k, b, k_b, dtype, assignment, ((uintptr_t)x & 15u) == 0, &fp);
    if (rc != ATK_OK) return rc;
    if (trace) {  // measurement build: the lean kernels alone, and room for every wavefront's timestamps
        if (fp.two_step || assignment != ATK_INTERLEAVED || !fp.s1.lean) return ATK_ERR_UNSUPPORTED;
        if (trace_bytes < fp.s1.grid * kTraceWaves * kTracePhases * 8 || fp.s1.T > kTraceWaves * kWave) return ATK_ERR_BAD_SHAPE;
    }
    void *state = nullptr, *data = nullptr;
    hipError_t e = get_pool(kPoolState, (size_t)fp.state_bytes, &state, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    e = get_pool(kPoolData, (size_t)fp.data_bytes, &data, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    void *s1_vals = out_vals;
    int32_t *s1_idx = out_idx;
    if (fp.two_step) {
        s1_vals = (unsigned char *)data + fp.cand_vals_off;
        s1_idx = (int32_t *)((unsigned char *)data + fp.cand_idx_off);
    }
    if (assignment == ATK_CONTIGUOUS)
        e = launch_approx_contig(fp.s1, x, s1_vals, s1_idx, state, data, (hipStream_t)stream);
    else if (fp.s1.lean)
        e = launch_approx_lean(fp.s1, x, s1_vals, s1_idx, state, (hipStream_t)stream, trace);
    else
        e = launch_approx(fp.s1, x, s1_vals, s1_idx, state, data, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    if (!fp.two_step) return ATK_OK;
    return run_exact(fp.ex, s1_vals, s1_idx, m, b * k_b, k, dtype, out_vals, out_idx,
                     (unsigned char *)state + fp.ex_state_off, fp.state_bytes - fp.ex_state_off,
                     (unsigned char *)data + fp.ex_data_off, fp.data_bytes - fp.ex_data_off, (hipStream_t)stream);
}

int atk_check_approx(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype) {
    int rc = check_approx(m, n, k, b, k_b, dtype);
    if (rc != ATK_OK) return rc;
    FullPlan fp;
    return make_full_plan(m, n, k, b, k_b, dtype, ATK_INTERLEAVED, true, &fp);
}

int atk_check_exact(int64_t m, int64_t n, int64_t k, int dtype) {
    int rc = check_common(m, n, k, dtype);
    if (rc != ATK_OK) return rc;
    ExactPlan pl;
    int64_t state_bytes = 0, data_bytes = 0;
    return make_exact_plans(m, n, k, dtype, &pl, &state_bytes, &data_bytes);
}

int atk_set_plan_override(const char *spec) {
    g_plan_override = parse_plan_override(spec);
    return ATK_OK;
}

int64_t atk_stage2_max_candidates(void) { return kStage2MaxCand; }

int64_t atk_workspace_bytes_assign(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, int assignment) {
    int rc = check_approx(m, n, k, b, k_b, dtype);
    if (rc != ATK_OK) return rc;
    FullPlan fp;
    rc = make_full_plan(m, n, k, b, k_b, dtype, assignment, true, &fp);
    if (rc != ATK_OK) return rc;
    return fp.state_bytes + fp.data_bytes;
}

int64_t atk_workspace_bytes(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype) {
    return atk_workspace_bytes_assign(m, n, k, b, k_b, dtype, ATK_INTERLEAVED);
}

int64_t atk_exact_workspace_bytes(int64_t m, int64_t n, int64_t k, int dtype) {
    int rc = check_common(m, n, k, dtype);
    if (rc != ATK_OK) return rc;
    ExactPlan pl;
    int64_t state_bytes = 0, data_bytes = 0;
    rc = make_exact_plans(m, n, k, dtype, &pl, &state_bytes, &data_bytes);
    if (rc != ATK_OK) return rc;
    return state_bytes + data_bytes;
}

int atk_exact_workspace_parts(int64_t m, int64_t n, int64_t k, int dtype, int64_t *state_bytes, int64_t *data_bytes) {
    if (!state_bytes || !data_bytes) return ATK_ERR_NULL_PTR;
    int rc = check_common(m, n, k, dtype);
    if (rc != ATK_OK) return rc;
    ExactPlan pl;
    return make_exact_plans(m, n, k, dtype, &pl, state_bytes, data_bytes);
}

int atk_plan_describe_assign(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, int assignment,
                             char *buf, int64_t buflen) {
    if (!buf || buflen < 1) return ATK_ERR_NULL_PTR;
    int rc = check_approx(m, n, k, b, k_b, dtype);
    if (rc != ATK_OK) return rc;
    FullPlan fp;
    rc = make_full_plan(m, n, k, b, k_b, dtype, assignment, true, &fp);
    if (rc != ATK_OK) return rc;
    const Plan &pl = fp.s1;
    // two steps: Stage 2 is the long-row exact selection over the candidates Stage 1 left in scratch
    const int stage2 = fp.two_step ? 2 : (int)pl.stage2;
    if (assignment == ATK_CONTIGUOUS)
        snprintf(buf, (size_t)buflen,
                 "contiguous V=%d KB=%d T=%d Gs=%d NB=%d bblocks=%d S=%d chunks_per_split=%d grid=%lld stage2=%d "
                 "scratch=%d lds=%d scratch_bytes=%lld",
                 pl.V, pl.KB, pl.T, pl.Gs, pl.NB, pl.bblocks, pl.S, pl.chunks_per_split, (long long)pl.grid, stage2,
                 (int)pl.use_scratch, pl.lds_bytes, (long long)(fp.state_bytes + fp.data_bytes));
    else
        snprintf(buf, (size_t)buflen,
                 "V=%d KB=%d T=%d Gw=%d P=%d colblocks=%d S=%d rows_per_split=%d grid=%lld stage2=%d direct=%d "
                 "scratch=%d wave_merge=%d nparts=%d lds=%d scratch_bytes=%lld packed=%d lean=%d pair_rows=%d refresh=%d helpers=%d",
                 pl.V, pl.KB, pl.T, pl.Gw, pl.P, pl.colblocks, pl.S, pl.rows_per_split, (long long)pl.grid, stage2,
                 (int)pl.direct, (int)pl.use_scratch, (int)pl.wave_merge, pl.nparts, pl.lds_bytes,
                 (long long)(fp.state_bytes + fp.data_bytes), (int)pl.packed, (int)pl.lean, pl.pair_rows, pl.refresh, pl.helpers);
    return ATK_OK;
}

int atk_plan_describe(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, char *buf,
                      int64_t buflen) {
    return atk_plan_describe_assign(m, n, k, b, k_b, dtype, ATK_INTERLEAVED, buf, buflen);
}

int approx_topk_assign(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype,
                       int assignment, void *out_vals, int32_t *out_idx, void *stream) {
    return run_approx(x, m, n, k, b, k_b, dtype, assignment, out_vals, out_idx, stream);
}

int approx_topk(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype,
                void *out_vals, int32_t *out_idx, void *stream) {
    return run_approx(x, m, n, k, b, k_b, dtype, ATK_INTERLEAVED, out_vals, out_idx, stream);
}

int approx_topk_noalloc(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype,
                        void *out_vals, int32_t *out_idx, void *stream) {
    if (!x || !out_vals || !out_idx) return ATK_ERR_NULL_PTR;
    int rc = check_approx(m, n, k, b, k_b, dtype);
    if (rc != ATK_OK) return rc;
    const int es = (dtype == ATK_F32) ? 4 : 2;
    if (((uintptr_t)x | (uintptr_t)out_vals) & (uintptr_t)(es - 1)) return ATK_ERR_ALIGN;
    if ((uintptr_t)out_idx & 3u) return ATK_ERR_ALIGN;
    FullPlan fp;
    // (no pair plans here: their mailbox has to be zero between calls, and this entry point shares its array)
    rc = make_full_plan(m, n, k, b, k_b, dtype, ATK_INTERLEAVED, ((uintptr_t)x & 15u) == 0, &fp, false);
    if (rc != ATK_OK) return rc;
    if (fp.two_step) return ATK_ERR_UNSUPPORTED;  // Stage 2 over more candidates than one workgroup holds: approx_topk only
    if (fp.state_bytes > ATK_NOALLOC_STATE_BYTES || fp.data_bytes > ATK_NOALLOC_SCRATCH_BYTES - ATK_NOALLOC_STATE_BYTES)
        return ATK_ERR_WORKSPACE;
    unsigned char *base = nullptr;
    if (fp.s1.use_scratch) {
        void *p = nullptr;
        const hipError_t e = fixed_scratch(&p);
        if (e != hipSuccess) return hip_fail(e);
        base = (unsigned char *)p;
        // The array keeps what the last call left.  Every launch leaves its tickets at zero, but a launch
        // that was cut short would not have: the tickets of this call are cleared first.
        const int64_t n_vec = (fp.state_bytes + 15) / 16;
        hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)ceil_div(n_vec, 256)), dim3(256), 0, (hipStream_t)stream,
                           (uint4 *)base, n_vec);
        const hipError_t ez = hipGetLastError();
        if (ez != hipSuccess) return hip_fail(ez);
    }
    const hipError_t e = fp.s1.lean ? launch_approx_lean(fp.s1, x, out_vals, out_idx, nullptr, (hipStream_t)stream)
                                    : launch_approx(fp.s1, x, out_vals, out_idx, base,
                                                    base ? base + ATK_NOALLOC_STATE_BYTES : nullptr, (hipStream_t)stream);
    return e == hipSuccess ? ATK_OK : hip_fail(e);
}

int exact_topk(const void *x, int64_t m, int64_t n, int64_t k, int dtype, void *out_vals, int32_t *out_idx,
               void *stream) {
    if (!x || !out_vals || !out_idx) return ATK_ERR_NULL_PTR;
    int rc = check_common(m, n, k, dtype);
    if (rc != ATK_OK) return rc;
    const int es = (dtype == ATK_F32) ? 4 : 2;
    if (((uintptr_t)x | (uintptr_t)out_vals) & (uintptr_t)(es - 1)) return ATK_ERR_ALIGN;
    if ((uintptr_t)out_idx & 3u) return ATK_ERR_ALIGN;
    ExactPlan pl;
    int64_t state_bytes = 0, data_bytes = 0;
    rc = make_exact_plans(m, n, k, dtype, &pl, &state_bytes, &data_bytes);
    if (rc != ATK_OK) return rc;
    void *state = nullptr, *data = nullptr;
    hipError_t e = get_pool(kPoolState, (size_t)state_bytes, &state, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    e = get_pool(kPoolData, (size_t)data_bytes, &data, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    return run_exact(pl, x, nullptr, m, n, k, dtype, out_vals, out_idx, state, state_bytes, data, data_bytes,
                     (hipStream_t)stream);
}

int64_t atk_trace_bytes(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype) {
    int rc = check_approx(m, n, k, b, k_b, dtype);
    if (rc != ATK_OK) return rc;
    FullPlan fp;
    rc = make_full_plan(m, n, k, b, k_b, dtype, ATK_INTERLEAVED, true, &fp);
    if (rc != ATK_OK) return rc;
    return fp.s1.grid * kTraceWaves * kTracePhases * 8;
}

int atk_trace_approx(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, void *out_vals,
                     int32_t *out_idx, void *trace, int64_t trace_bytes, void *stream) {
    if (!trace) return ATK_ERR_NULL_PTR;
    if ((uintptr_t)trace & 7u) return ATK_ERR_ALIGN;
    return run_approx(x, m, n, k, b, k_b, dtype, ATK_INTERLEAVED, out_vals, out_idx, stream, trace, trace_bytes);
}

int atk_read_ceiling(const void *x, int64_t bytes, void *sink, void *stream) {
    if (!x || !sink) return ATK_ERR_NULL_PTR;
    if (bytes < 16 || (bytes & 15) || ((uintptr_t)x & 15u) || ((uintptr_t)sink & 7u)) return ATK_ERR_ALIGN;
    const int64_t n_vec = bytes / 16;
    int64_t wgs = (n_vec + 256 * 8 - 1) / (256 * 8);
    if (wgs > 2 * kNumCU) wgs = 2 * kNumCU;  // measured best from 32 MB to 512 MB: two workgroups of four wavefronts per CU
    if (wgs > ATK_CEILING_SINK_BYTES / 32) wgs = ATK_CEILING_SINK_BYTES / 32;
    const int64_t slab = (n_vec + wgs - 1) / wgs;
    hipLaunchKernelGGL(read_ceiling_kernel, dim3((unsigned)wgs), dim3(256), 0, (hipStream_t)stream, (const uint4 *)x,
                       n_vec, slab, (u64 *)sink);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    return ATK_OK;
}

int atk_copy(void *dst, const void *src, int64_t bytes, void *stream) {
    if (!dst || !src) return ATK_ERR_NULL_PTR;
    if (bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15u) || ((uintptr_t)dst & 15u)) return ATK_ERR_ALIGN;
    const int64_t n_vec = bytes / 16;
    int64_t wgs = (n_vec + 256 * 4 - 1) / (256 * 4);
    if (wgs > kNumCU * 16) wgs = kNumCU * 16;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)wgs), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src,
                       (uint4 *)dst, n_vec);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    return ATK_OK;
}

int atk_sleep(int64_t microseconds, void *stream) {
    if (microseconds < 0 || microseconds > 1000000) return ATK_ERR_BAD_SHAPE;
    hipLaunchKernelGGL(sleep_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, microseconds * 100, (u64 *)nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    return ATK_OK;
}

}  // extern "C"
