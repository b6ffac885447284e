// One-time re-layout of the static BLAST factors (bf16):
//   Vt[j][rho][c] = V[j][c][rho]      contraction index of stage 1 made contiguous
//   Sp[rho][i][j] = S[i][j][rho]      one zero-padded 16x16 coupling tile per rank index
#include "blr_common.h"

namespace blr {
namespace {

__global__ __launch_bounds__(256) void pack_v_kernel(const bf16_t* V, bf16_t* Vt, int q, int r) {
    __shared__ bf16_t tile[32][34];
    const int j = blockIdx.z;
    const int rho0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const bf16_t* Vj = V + (int64_t)j * q * r;
    bf16_t* Vtj = Vt + (int64_t)j * q * r;
    for (int cc = ty; cc < 32; cc += 8) {
        const int c = c0 + cc, rho = rho0 + tx;
        tile[cc][tx] = (c < q && rho < r) ? Vj[(int64_t)c * r + rho] : (bf16_t)0;
    }
    __syncthreads();
    for (int rr = ty; rr < 32; rr += 8) {
        const int rho = rho0 + rr, c = c0 + tx;
        if (rho < r && c < q) Vtj[(int64_t)rho * q + c] = tile[tx][rr];
    }
}

// Vt re-laid for the fused stage 1 + coupling kernel when q is not a multiple of the layer's chunk (64 or
// 128 columns): row (j, rho) holds the k chunks of GLOBAL input columns that block j touches, chunk c of
// the row = columns chunk (cb + c) .. + chunk - 1 with cb = floor(j q / chunk); positions outside
// [j q, (j+1) q) are zero. The kernel can then walk X in whole aligned cache lines, whatever q is.
__global__ __launch_bounds__(256) void pack_va_kernel(const bf16_t* __restrict__ V, bf16_t* __restrict__ Va, int q, int r, int qp, int chunk, int64_t total) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int x = (int)(e % qp);
    const int rho = (int)((e / qp) % r);
    const int j = (int)(e / ((int64_t)qp * r));
    const int64_t gcol = (((int64_t)j * q) / chunk) * chunk + x;     // global input column
    const int64_t c = gcol - (int64_t)j * q;
    Va[e] = (c >= 0 && c < q) ? V[((int64_t)j * q + c) * r + rho] : (bf16_t)0;
}

// perm: the form the single-kernel path reads. Slot j' = (j % 8)*2 + j/8 holds input block j, and the
// tiles are in the fragment order of v_mfma_f32_16x16x16_bf16 with two rank indices per 16 bytes:
//   Sq[rho/2][lane][rho%2][v] = S'[rho][i = lane%16][slot 4 (lane/16) + v]
// so that a lane fetches the B operands of two rank indices with one 16-byte load.
__global__ __launch_bounds__(256) void pack_s_kernel(const bf16_t* S, bf16_t* Sp, int b, int r, int perm) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)r * 256) return;
    const int slot = (int)(e & 15), i = (int)((e >> 4) & 15);
    const int j = perm ? (slot >> 1) + (slot & 1) * 8 : slot;
    const int rho = (int)(e >> 8);
    const int64_t dst = perm ? (((int64_t)(rho >> 1) * 64 + (slot >> 2) * 16 + i) * 8 + (rho & 1) * 4 + (slot & 3)) : e;
    Sp[dst] = (i < b && j < b) ? S[((int64_t)i * b + j) * r + rho] : (bf16_t)0;
}

// V in the fragment order of v_mfma_f32_32x32x16_bf16 (see blr_common.h), zero-filled past q and r
__global__ __launch_bounds__(256) void pack_vf_kernel(const bf16_t* V, bf16_t* Vf, int q, int r, int ntl, int nks, int64_t total) {
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    const int e = (int)(id & 7), lane = (int)((id >> 3) & 63);
    int64_t t = id >> 9;
    const int ks = (int)(t % nks); t /= nks;
    const int nt = (int)(t % ntl);
    const int j = (int)(t / ntl);
    const int rho = nt * 32 + (lane & 31), k = ks * 16 + (lane >> 5) * 8 + e;
    Vf[id] = (rho < r && k < q) ? V[((int64_t)j * q + k) * r + rho] : (bf16_t)0;
}

// U in the fragment order of v_mfma_f32_16x16x32_bf16, zero-filled past r
__global__ __launch_bounds__(256) void pack_uf_kernel(const bf16_t* U, bf16_t* Uf, int p, int r, int npt, int nks, int64_t total) {
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    const int e = (int)(id & 7), lane = (int)((id >> 3) & 63);
    int64_t t = id >> 9;
    const int ks = (int)(t % nks); t /= nks;
    const int nt = (int)(t % npt);
    const int i = (int)(t / npt);
    const int a = nt * 16 + (lane & 15), rho = ks * 32 + (lane >> 4) * 8 + e;
    Uf[id] = (rho < r) ? U[((int64_t)i * p + a) * r + rho] : (bf16_t)0;
}

__global__ __launch_bounds__(256) void copy_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int64_t n) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e < n) dst[e] = src[e];
}

// Stand-alone coupling for FEW tokens: A[t][i][rho] = sum_j S[i][j][rho] * Z[t][j][rho] from the
// canonical S[b][b][r] (rank index contiguous). One thread per (token, output block, PAIR of rank
// indices): 2 b independent 4-byte loads (all in flight at once), one 4-byte store; consecutive lanes
// take consecutive pairs, so a wavefront reads and writes contiguous runs. The fine grain is for
// parallelism: with one token the whole of S (b b r elements) is read once, and 8 rank indices per
// thread left it to 5 workgroups (8 us); pairs spread it over 20. B > 0: compile-time block count.
template <int B>
__global__ __launch_bounds__(256) void coupling_small_kernel(const bf16_t* __restrict__ Z, const bf16_t* __restrict__ S,
                                                             bf16_t* __restrict__ A, int64_t total, int b_rt, int r2) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int b = B > 0 ? B : b_rt;
    const int c = (int)(e % r2);
    const int i = (int)((e / r2) % b);
    const int64_t t = e / ((int64_t)r2 * b);
    const uint32_t* z = (const uint32_t*)Z + t * b * r2 + c;          // Z[t][0][2c], stride r2 words per block
    const uint32_t* sp = (const uint32_t*)S + (int64_t)i * b * r2 + c;   // S[i][0][2c]
    float acc0 = 0.f, acc1 = 0.f;
    if (B > 0) {
        uint32_t zv[B > 0 ? B : 1], sv[B > 0 ? B : 1];
#pragma unroll
        for (int j = 0; j < B; ++j) { zv[j] = z[(int64_t)j * r2]; sv[j] = sp[(int64_t)j * r2]; }
#pragma unroll
        for (int j = 0; j < B; ++j) {
            acc0 = fmaf(__uint_as_float(sv[j] << 16), __uint_as_float(zv[j] << 16), acc0);
            acc1 = fmaf(__uint_as_float(sv[j] & 0xFFFF0000u), __uint_as_float(zv[j] & 0xFFFF0000u), acc1);
        }
    } else {
        for (int j = 0; j < b; ++j) {
            const uint32_t zw = z[(int64_t)j * r2], sw = sp[(int64_t)j * r2];
            acc0 = fmaf(__uint_as_float(sw << 16), __uint_as_float(zw << 16), acc0);
            acc1 = fmaf(__uint_as_float(sw & 0xFFFF0000u), __uint_as_float(zw & 0xFFFF0000u), acc1);
        }
    }
    ((uint32_t*)A)[(t * b + i) * r2 + c] = pack2_bf16(acc0, acc1);
}

}  // namespace

hipError_t launch_coupling_small(const void* Z, const void* S, void* A, int64_t T, int b, int r, hipStream_t s) {
    const int64_t total = T * b * (r / 2);              // r is a multiple of 8
    if (total <= 0) return hipSuccess;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (b == 16)
        hipLaunchKernelGGL(coupling_small_kernel<16>, grid, dim3(256), 0, s, (const bf16_t*)Z, (const bf16_t*)S, (bf16_t*)A, total, b, r / 2);
    else
        hipLaunchKernelGGL(coupling_small_kernel<0>, grid, dim3(256), 0, s, (const bf16_t*)Z, (const bf16_t*)S, (bf16_t*)A, total, b, r / 2);
    return hipGetLastError();
}

hipError_t launch_blast_pack(const void* U, const void* S, const void* V, void* Sp, void* Sc, void* Vt, void* Va, void* Vf, void* Uf,
                             int n_in, int n_out, int b, int r, hipStream_t s) {
    const int q = n_in / b, p = n_out / b;
    if (Sc) {                                           // canonical S, for the few-token coupling
        const int64_t total = (int64_t)b * b * r;
        hipLaunchKernelGGL(copy_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t*)S, (bf16_t*)Sc, total);
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
    }
    hipLaunchKernelGGL(pack_s_kernel, dim3((unsigned)r), dim3(256), 0, s, (const bf16_t*)S, (bf16_t*)Sp, b, r, Vf ? 1 : 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (Vt) {
        dim3 gv((unsigned)((r + 31) / 32), (unsigned)((q + 31) / 32), (unsigned)b);
        hipLaunchKernelGGL(pack_v_kernel, gv, dim3(256), 0, s, (const bf16_t*)V, (bf16_t*)Vt, q, r);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (Va) {
        const int chunk = blast_chunk(n_in, b), qp = blast_va_row(q, chunk);
        const int64_t total = (int64_t)b * r * qp;
        hipLaunchKernelGGL(pack_va_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t*)V, (bf16_t*)Va, q, r, qp, chunk, total);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (Vf) {
        const int ntl = (r + 31) / 32, nks = (q + 15) / 16;
        const int64_t total = (int64_t)b * ntl * nks * 512;
        hipLaunchKernelGGL(pack_vf_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const bf16_t*)V, (bf16_t*)Vf, q, r, ntl, nks, total);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (Uf) {
        const int npt = p / 16, nks = (r + 31) / 32;
        const int64_t total = (int64_t)b * npt * nks * 512;
        hipLaunchKernelGGL(pack_uf_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const bf16_t*)U, (bf16_t*)Uf, p, r, npt, nks, total);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace blr
