// The lean kernels' launches with one workgroup per row or column block, or a helper + finisher pair (see
// atk_lean_kernel.h for the kernel).
#include "atk_lean_kernel.h"

namespace atk {

hipError_t launch_approx_lean(const Plan &pl, const void *x, void *out_vals, int32_t *out_idx, void *state, hipStream_t stream,
                              void *trace) {
    if (!pl.lean || pl.T > 512 || pl.T % kWave) return hipErrorInvalidValue;
    LeanParams prm;
    memset(&prm, 0, sizeof prm);
    prm.x = x;
    prm.out_vals = out_vals;
    prm.out_idx = out_idx;
    prm.mail = (u64 *)state;
    prm.n = pl.n;
    prm.b = (int)pl.b;
    prm.L = (int)pl.L;
    prm.G = (int)pl.G;
    prm.Gw = pl.Gw;
    prm.P = pl.P;
    prm.colblocks = pl.colblocks;
    prm.gw_shift = log2_exact_lean(pl.Gw);
    prm.cb_shift = log2_exact_lean(pl.colblocks);
    prm.k = (int)pl.k;
    prm.idx_bits = 1;
    while (((int64_t)1 << prm.idx_bits) < pl.n) ++prm.idx_bits;
    prm.m = (int)pl.m;
    prm.Lh = pl.pair_rows;
    prm.H = pl.helpers;
    prm.spin_limit = 1 << 20;  // about a second of polling
    prm.bound_ok = pl.bound_ok;
    prm.trace = (u64 *)trace;
    const int mode = pl.helpers > 0 ? kLeanMulti : pl.pair_rows > 0 ? kLeanPair : (!pl.stage2 ? kLeanOut : kLeanSelect);
    if ((mode == kLeanPair || mode == kLeanMulti) && !state) return hipErrorInvalidValue;
    if (mode == kLeanMulti) return launch_lean_multi(pl, prm, stream);
#define ATK_LEAN(ELT)                                                              \
    switch (mode) {                                                                \
        case kLeanOut: return launch_lean_mode<ELT, kLeanOut>(pl, prm, stream);    \
        case kLeanSelect: return launch_lean_mode<ELT, kLeanSelect>(pl, prm, stream); \
        default: return launch_lean_mode<ELT, kLeanPair>(pl, prm, stream);         \
    }
    if (pl.dtype == ATK_F32) {
        ATK_LEAN(ATK_F32)
    }
    ATK_LEAN(ATK_BF16)
#undef ATK_LEAN
}

}  // namespace atk
