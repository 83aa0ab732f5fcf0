// exact_topk: the exact comparison point (Section 1; RadixSelect of Appendix D.2).
// Small rows: one workgroup per row, the row's composites live in LDS and go through the
// same radix select + ordering as Stage 2.
#include "atk_common.h"
#include "atk_select.h"

namespace atk {

static int64_t pow2_ceil64(int64_t v) {
    int64_t p = 1;
    while (p < v) p <<= 1;
    return p;
}

int make_exact_plan(int64_t m, int64_t n, int64_t k, int dtype, ExactPlan *pl) {
    ExactPlan p;
    p.dtype = dtype;
    p.m = m;
    p.n = n;
    p.k = k;
    p.T = kMaxThreads;
    p.chunks = 1;
    p.scratch_bytes = 0;
    p.state_bytes = 0;
    int64_t lds = select_lds_bytes(n, (int)pow2_ceil64(k < (1 << 20) ? k : (1 << 20)));
    p.single_wg = lds <= kLdsBudget;
    if (!p.single_wg) return ATK_ERR_UNSUPPORTED;
    if (m >= (1ll << 31)) return ATK_ERR_UNSUPPORTED;
    p.lds_bytes = (int)lds;
    *pl = p;
    return ATK_OK;
}

template <int ELT>
__global__ void __launch_bounds__(kMaxThreads) exact_small_kernel(const void *x, int n, int k, void *out_vals,
                                                                  int32_t *out_idx) {
    extern __shared__ __align__(16) unsigned char smem[];
    u64 *cand = (u64 *)smem;
    const int r = blockIdx.x;
    const int T = blockDim.x;
    auto load_bits = [&](int i) -> uint32_t {
        if (ELT == ATK_F32) return ((const uint32_t *)x)[(int64_t)r * n + i];
        return ((uint32_t)((const uint16_t *)x)[(int64_t)r * n + i]) << 16;
    };
    int i = threadIdx.x;
    for (; i + 3 * T < n; i += 4 * T) {  // four loads in flight
        uint32_t b0 = load_bits(i), b1 = load_bits(i + T), b2 = load_bits(i + 2 * T), b3 = load_bits(i + 3 * T);
        cand[i] = make_composite(b0, i);
        cand[i + T] = make_composite(b1, i + T);
        cand[i + 2 * T] = make_composite(b2, i + 2 * T);
        cand[i + 3 * T] = make_composite(b3, i + 3 * T);
    }
    for (; i < n; i += T) cand[i] = make_composite(load_bits(i), i);
    __syncthreads();
    select_write<ELT>(cand, n, k, out_vals, out_idx, (int64_t)r);
}

hipError_t launch_exact(const ExactPlan &pl, const void *x, void *out_vals, int32_t *out_idx, void *state,
                        void *data, hipStream_t stream) {
    (void)state;
    (void)data;
    if (pl.dtype == ATK_F32)
        hipLaunchKernelGGL(exact_small_kernel<ATK_F32>, dim3((unsigned)pl.m), dim3(pl.T), (size_t)pl.lds_bytes, stream, x,
                           (int)pl.n, (int)pl.k, out_vals, out_idx);
    else
        hipLaunchKernelGGL(exact_small_kernel<ATK_BF16>, dim3((unsigned)pl.m), dim3(pl.T), (size_t)pl.lds_bytes, stream, x,
                           (int)pl.n, (int)pl.k, out_vals, out_idx);
    return hipGetLastError();
}

}  // namespace atk
