// Host-only helpers for choosing (b, k_b): the recall model of Appendix C (Eq. 1) and a
// runtime estimate in the shape of Appendix D's cost composition,
//   cost(approx) = cost(Stage 1 over b buckets) + [b*k_b > k] * cost(Stage 2 over b*k_b candidates),
// with the terms taken from timings of this library's kernels on an MI355X instead of the
// paper's operation counts.  Section 3 / Appendix E describe the trade-off this makes
// executable: for k << n raise b (more candidates, then Stage 2), for k ~ n raise k_b with
// b*k_b = k.  No HIP call is made here.
#include <algorithm>
#include <cmath>
#include <cstdint>

#include "atk_common.h"

namespace atk {

// Eq. 1 rewritten per bucket: with X ~ Binomial(k, 1/b) top-k elements in a bucket, min(X, k_b)
// of them are returned, and E[recall] = (b/k) E[min(X, k_b)].  Only the k_b lowest terms of
// the distribution are needed: E[min(X, k_b)] = k_b - sum_{z < k_b} (k_b - z) Pr(X = z).
static double eq1_recall(int64_t k, int64_t b, int64_t k_b) {
    if (b <= 1) return 1.0;
    const double lp = -std::log((double)b), lq = std::log1p(-1.0 / (double)b);
    double deficit = 0.0;
    for (int64_t z = 0; z < k_b && z <= k; ++z) {
        const double lc = std::lgamma((double)k + 1.0) - std::lgamma((double)z + 1.0) - std::lgamma((double)(k - z) + 1.0);
        deficit += (double)(k_b - z) * std::exp(lc + (double)z * lp + (double)(k - z) * lq);
    }
    double r = (double)b / (double)k * ((double)k_b - deficit);
    return r > 1.0 ? 1.0 : (r < 0.0 ? 0.0 : r);
}

// Microseconds of one approx_topk call, from measurements of this library on one MI355X:
// a fixed launch + ramp cost, the bytes at the streaming rate a launch of that size reaches
// (the bytes read times a factor for the register queues of k_b > 1), the hand-over between
// workgroups when rows are split, and Stage 2.  Small launches are bound by the chain of
// hand-overs instead (workgroup merge, ticket, merge of the splits, Stage 2): a floor.
static double estimate_us(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype) {
    const double es = (dtype == ATK_F32) ? 4.0 : 2.0;
    const double rd = (double)m * (double)n * es, wr = (double)m * (double)k * (es + 4.0), bytes = rd + wr;
    int KB = 1;
    while (KB < k_b) KB <<= 1;
    // streaming rate grows with the size of the launch.  f32 running maxima: 5.8 TB/s at 32 MB,
    // 7.1 TB/s at 0.5 GB; queues and bf16 (twice the elements per byte): 5.5 and 6.4 TB/s
    const bool lean = KB == 1 && dtype == ATK_F32;
    double rate = (lean ? 7.2e6 : 6.5e6) * bytes / (bytes + (lean ? 8.0e6 : 6.0e6));  // bytes per microsecond
    if (rate < 0.5e6) rate = 0.5e6;
    // (sixteen slots: f32 rows go through the sorting-network scan, bf16 rows hold twice the elements per byte)
    // (eight slots on long buckets: few elements still enter a queue once the lanes of a column have pooled their floors)
    const double queue = KB <= 1 ? 1.0 : KB == 2 ? 1.07 : KB == 4 ? 1.3 : KB == 8 ? (n / b >= 4096 ? 1.7 : 2.7) : (dtype == ATK_F32 && n / b < 4096 ? 3.9 : 6.9);
    double us = 1.5 + (rd * queue + wr) / rate;
    const bool stage2 = b * k_b > k;
    const double cand = (double)(b * k_b);
    // Rows are split over workgroups when whole rows, in workgroups of one lane per column group
    // (64 lanes at least), leave CUs idle; a lane keeps four loads at least.
    const double groups = (double)b / (double)stage1_pick_v(dtype, KB, 0, b);
    double splits = 256.0 / ((double)m * std::max(1.0, groups / 64.0));
    splits = std::min(splits, std::min((double)n / 8192.0, (double)(n / b) / 4.0));
    // without Stage 2 (and with small queues) the workgroups of a row first share out its columns, in
    // 128-byte pieces of the matrix rows, which costs no hand-over
    if (!stage2 && KB <= 2 && ((double)n * es) == std::floor((double)n * es / 128.0) * 128.0) {
        double pieces = (double)b * es / 128.0;
        while (pieces >= 2.0 && splits >= 2.0) {
            pieces /= 2.0;
            splits /= 2.0;
        }
    }
    if (stage2 && splits > 16.0) splits = 16.0;
    if (splits > 128.0) splits = 128.0;
    const bool split = splits >= 2.0;
    if (split || stage2) us += 2.0;
    if (stage2) us += 0.3 + 0.001 * cand;
    // Stage 2 behind queues: the candidates of a row come together through the general kernel's exchange, and from
    // 2048 candidates on they are selected digit by digit (128 x 65536 f32, k = 512: b = 1024, k_b = 2 takes 24 us where
    // b = 1024, k_b = 1 with half the candidates takes 11)
    if (stage2 && KB >= 2) us += 0.005 * cand;
    // more than four candidates per lane of the selecting workgroup: digit by digit (k = 512, b = 4096: 32 us)
    if (stage2 && cand > 2048.0) us += 0.004 * cand;
    // more candidates than one workgroup holds: Stage 1 leaves them in scratch and exact_topk's kernels select from
    // the pairs (further launches; one workgroup per row in LDS up to 160 KB, sweeps beyond)
    if (stage2 && b * k_b > atk_stage2_max_candidates()) us += 35.0 + 0.02 * (double)k + (double)m * cand * 24.0 / 5.0e6;
    // more rows than CUs: the selections of the rows that share a CU queue up behind each other (measured 2 us
    // a row at 1024 candidates, k = 256; 3 us at k = 512)
    if (stage2 && m > 256) us += (double)m / 256.0 * (0.001 * cand + 0.004 * (double)k);
    double floor_us = 4.0;
    // lanes share column groups and merge inside the workgroup when the rows alone cannot fill the chip
    if ((double)m * groups < 16384.0) floor_us = 6.0 + bytes / 16.0e6;
    if (split && !(stage2 && m >= 128)) floor_us = 6.5 + bytes / 12.0e6 + (stage2 ? 1.5 + 0.001 * cand : 0.0);
    if (us < floor_us) us = floor_us;
    // long queues whose lists go through scratch: the last workgroup's merges of 8- and 16-slot lists (8 x 2^18 f32,
    // k = 64, b = 16, k_b = 8: 25 us where the bytes and the floor say 10)
    if (split && KB >= 8) us += KB >= 16 ? 25.0 : 15.0;
    // few rows: many splits per row, merged by the workgroup that finishes the row
    if (split && splits > 2.0) us += 0.04 * splits * (stage2 ? std::max(1.0, cand / 256.0) : 1.0);
    return us;
}

}  // namespace atk

using namespace atk;

extern "C" {

double atk_expected_recall(int64_t k, int64_t b, int64_t k_b) {
    if (k < 1 || b < 1 || k_b < 1 || k_b > k || b * k_b < k) return -1.0;
    return eq1_recall(k, b, k_b);
}

double atk_worst_case_recall(int64_t n, int64_t k, int64_t b, int64_t k_b) {
    // Eq. 2 of Appendix C: the true top-k packed into as few buckets as possible - floor(b*k/n) buckets filled
    // with top-k elements, of which k_b each come back, and k mod (n/b) of them in one more bucket
    if (n < 1 || k < 1 || k > n || b < 1 || b > n || n % b != 0 || k_b < 1 || k_b > k || k_b > n / b || b * k_b < k) return -1.0;
    const int64_t len = n / b;
    const int64_t full = k / len, rest = k % len;  // floor(b*k/n) = floor(k / (n/b))
    const double r = (double)(full * k_b + std::min<int64_t>(k_b, rest)) / (double)k;
    return r > 1.0 ? 1.0 : r;
}

double atk_estimate_us(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype) {
    if (atk_check_approx(m, n, k, b, k_b, dtype) != ATK_OK) return -1.0;
    return estimate_us(m, n, k, b, k_b, dtype);
}

int atk_advise(int64_t m, int64_t n, int64_t k, int dtype, double min_recall, int64_t *b_out, int64_t *k_b_out,
               double *recall_out, double *us_out) {
    if (!b_out || !k_b_out) return ATK_ERR_NULL_PTR;
    int rc = atk_check_exact(m, n, k, dtype);
    if (rc != ATK_OK) return rc;
    if (!(min_recall > 0.0) || min_recall > 1.0) return ATK_ERR_BAD_PARAMS;
    const int64_t lane = (dtype == ATK_F32) ? 4 : 8;
    bool have = false, have_ok = false;
    int64_t best_b = 0, best_kb = 0;
    double best_recall = 0.0, best_us = 0.0;
    for (int64_t k_b = 1; k_b <= ATK_MAX_KB && k_b <= k; k_b <<= 1) {
        for (int64_t ratio = 1; ratio <= 64; ratio <<= 1) {
            int64_t b = (ratio * k + k_b - 1) / k_b;
            if (ratio > 1 && b % lane) b += lane - b % lane;  // whole vector loads per lane
            if (atk_check_approx(m, n, k, b, k_b, dtype) != ATK_OK) break;  // b grows with ratio: k_b > n/b from here on
            const double rec = eq1_recall(k, b, k_b), us = estimate_us(m, n, k, b, k_b, dtype);
            const bool ok = rec >= min_recall;
            bool take;
            if (!have)
                take = true;
            else if (ok != have_ok)
                take = ok;
            else if (ok)
                take = us < best_us || (us == best_us && rec > best_recall);
            else
                take = rec > best_recall;
            if (take) {
                have = true;
                have_ok = ok;
                best_b = b;
                best_kb = k_b;
                best_recall = rec;
                best_us = us;
            }
            if (rec >= 1.0) break;
        }
    }
    if (!have) return ATK_ERR_UNSUPPORTED;
    *b_out = best_b;
    *k_b_out = best_kb;
    if (recall_out) *recall_out = best_recall;
    if (us_out) *us_out = best_us;
    return have_ok ? ATK_OK : ATK_ADVISE_BELOW_TARGET;
}

}  // extern "C"
