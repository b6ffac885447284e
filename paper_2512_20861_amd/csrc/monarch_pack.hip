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

// First factor of `members` Monarch layers of one shape that share their input, as the first factor of
// one layer with members * b output blocks: Rg[l][rho*(members*b) + m*b + k][:] = Rs[m][l][rho*b + k][:].
template <typename TS>
__global__ __launch_bounds__(256) void group_first_factor_kernel(const TS* __restrict__ Rs, TS* __restrict__ Rg,
                                                                 int members, int b, int rp, int p, int64_t total) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int a = (int)(e % p);
    int64_t row = e / p;                                // (l, rho, m, k) flattened
    const int k = (int)(row % b); row /= b;
    const int m = (int)(row % members); row /= members;
    const int rho = (int)(row % rp);
    const int64_t l = row / rp;
    Rg[e] = Rs[((((int64_t)m * b + l) * rp + rho) * b + k) * p + a];
}

// Blocked -> interleaved output order of a Monarch layer with b2 = 2^shift output blocks (paper Section 2.1:
// the final stride permutation P): Y[t][j*b2 + k] = Yb[t][k*q + j]. A workgroup takes one token and
// a segment of js values of j through LDS: rows k of the segment arrive as 16-byte pieces and leave
// as 16-byte pieces of the interleaved order, both fully coalesced. LDS rows are padded by 8 elements
// so that the 2-byte reads of neighbouring lanes (same k, neighbouring j; or rows 8 apart) fall into
// different banks.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void interleave_rows_kernel(const bf16_t* __restrict__ Yb, bf16_t* __restrict__ Y,
                                                              int64_t T, int q, int b2, int shift, int js, int nseg, int tpw) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* rows = (bf16_t*)smem;
    const int tid = threadIdx.x;
    const int seg = blockIdx.x % nseg;
    const int64_t t0 = (int64_t)(blockIdx.x / nseg) * tpw;      // tpw tokens per workgroup (1 unless nseg == 1)
    const int nt = T - t0 < tpw ? (int)(T - t0) : tpw;
    const int j0 = seg * js, jn = q - j0 < js ? q - j0 : js, ls = js + 8;
    const int64_t n_out = (int64_t)q * b2;
    const bf16_t* src = Yb + t0 * n_out + j0;
    const int vpr = jn >> 3, nv = vpr * b2;             // 16-byte pieces per row k, and per token
    const int total = nv * nt;
    for (int v0 = 0; v0 < total; v0 += 4 * 256) {
        u32x4 r[4];
        int at[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int v = v0 + u * 256 + tid;
            at[u] = -1;
            if (v < total) {
                const int tk = v / vpr, jv = v - tk * vpr;      // tk = token * b2 + k
                const int tl = tk >> shift, k = tk & (b2 - 1);
                r[u] = *(const u32x4*)(src + tl * n_out + (int64_t)k * q + 8 * jv);
                at[u] = tk * ls + 8 * jv;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (at[u] >= 0) *(u32x4*)(rows + at[u]) = r[u];
    }
    __syncthreads();
    bf16_t* dst = Y + t0 * n_out + (int64_t)j0 * b2;
    for (int v = tid; v < total; v += 256) {
        const int tl = v / nv;
        const int o = (v - tl * nv) << 3;               // first of 8 consecutive outputs of the segment
        const bf16_t* rt = rows + tl * b2 * ls;
        unsigned e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) e[i] = rt[((o + i) & (b2 - 1)) * ls + ((o + i) >> shift)];
        u32x4 w;
        w.x = e[0] | (e[1] << 16); w.y = e[2] | (e[3] << 16); w.z = e[4] | (e[5] << 16); w.w = e[6] | (e[7] << 16);
        *(u32x4*)(dst + tl * n_out + o) = w;
    }
}

// segment length: the whole row of one k if it fits 32 KB of LDS together with the other k
inline int interleave_segment(int q, int b2) {
    int js = (32 * 1024 / 2 / b2 - 8) / 16 * 16;
    return js < q ? js : q;
}

}  // namespace

bool monarch_interleave_supported(int64_t T, int n_out, int b2) {
    if (b2 < 2 || b2 > 64 || (b2 & (b2 - 1)) || n_out % b2) return false;
    const int q = n_out / b2;
    return q % 8 == 0 && interleave_segment(q, b2) >= 16 && T * ((q + interleave_segment(q, b2) - 1) / interleave_segment(q, b2)) < (1ll << 31);
}

hipError_t launch_monarch_interleave(const void* Yb, void* Y, int64_t T, int n_out, int b2, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    const int q = n_out / b2, js = interleave_segment(q, b2), nseg = (q + js - 1) / js;
    int shift = 0;
    while ((1 << shift) < b2) ++shift;
    // short rows: several tokens per workgroup, about 16 KB of them
    const int row_lds = b2 * (js + 8) * 2;
    int tpw = nseg == 1 ? 16 * 1024 / row_lds : 1;
    if (tpw < 1) tpw = 1;
    const int64_t groups = (T + tpw - 1) / tpw;
    hipLaunchKernelGGL(interleave_rows_kernel, dim3((unsigned)(groups * nseg)), dim3(256), (size_t)tpw * row_lds, s,
                       (const bf16_t*)Yb, (bf16_t*)Y, T, q, b2, shift, js, nseg, tpw);
    return hipGetLastError();
}

hipError_t launch_monarch_group_first_factor(const void* Rs, void* Rg, int n_in, int nblocks, int r, int members, DType dt, hipStream_t s) {
    const int p = n_in / nblocks, rp = r / nblocks;
    const int64_t total = (int64_t)members * nblocks * r * p;
    if (total <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dt == DType::F32)
        hipLaunchKernelGGL(group_first_factor_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)Rs, (float*)Rg, members, nblocks, rp, p, total);
    else
        hipLaunchKernelGGL(group_first_factor_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t*)Rs, (bf16_t*)Rg, members, nblocks, rp, p, total);
    return hipGetLastError();
}

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
