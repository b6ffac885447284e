// Offline re-layout of a Monarch layer's first factor so that the layer can consume an activation
// that an upstream Monarch layer left in BLOCKED output order (paper Section 4, optimisation 3: the
// final permutation of a Monarch layer is dropped and folded into the static weight that consumes
// its output). With b blocks, the upstream layer stores feature j*b + k at position k*(n/b) + j.
// Input block l of this layer covers canonical features l*p + jj*b + k (jj < p/b, k < b), which in
// blocked order are b runs of p/b consecutive elements: run k starts at k*(n/b) + l*(p/b). Ordering
// the contraction index run by run, a' = k*(p/b) + jj, makes every run a contiguous read:
//     Rp[l][c][k*(p/b) + jj] = R[l][c][jj*b + k].
#include "blr_common.h"

namespace blr {
namespace {

template <typename TS>
__global__ __launch_bounds__(256) void permute_first_factor_kernel(const TS* __restrict__ R, TS* __restrict__ Rp,
                                                                   int64_t rows, int p, int b) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= rows * p) return;
    const int ap = (int)(e % p);                        // a' = k*(p/b) + jj
    const int64_t row = e / p;                          // (l, c) flattened
    const int seg = p / b, k = ap / seg, jj = ap % seg;
    Rp[e] = R[row * p + (int64_t)jj * b + k];
}

}  // namespace

hipError_t launch_monarch_permute_first_factor(const void* R, void* Rp, int n_in, int nblocks, int r, DType dt, hipStream_t s) {
    const int p = n_in / nblocks;
    const int64_t rows = (int64_t)nblocks * r, total = rows * p;
    if (total <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dt == DType::F32)
        hipLaunchKernelGGL(permute_first_factor_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)R, (float*)Rp, rows, p, nblocks);
    else
        hipLaunchKernelGGL(permute_first_factor_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t*)R, (bf16_t*)Rp, rows, p, nblocks);
    return hipGetLastError();
}

}  // namespace blr
