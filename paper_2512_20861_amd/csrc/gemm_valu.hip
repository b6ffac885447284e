// Portable scalar-ALU kernels: correct for every shape and stride, fp32 accumulation.
// They are the whole fp32 path and the fallback of the bf16 path where the MFMA kernels'
// alignment contract does not hold.
#include "blr_common.h"

namespace blr {
namespace {

template <typename TS> __device__ inline float load_as_float(const TS* p);
template <> __device__ inline float load_as_float<float>(const float* p) { return *p; }
template <> __device__ inline float load_as_float<bf16_t>(const bf16_t* p) { return bf16_to_float(*p); }
template <typename TS> __device__ inline void store_from_float(TS* p, float v);
template <> __device__ inline void store_from_float<float>(float* p, float v) { *p = v; }
template <> __device__ inline void store_from_float<bf16_t>(bf16_t* p, float v) { *p = float_to_bf16(v); }

constexpr int VBM = 64, VBN = 64, VBK = 16;

// 64x64 output tile per workgroup, 4x4 outputs per thread, operands staged in LDS as fp32.
template <typename TS>
__global__ __launch_bounds__(256) void gemm_valu_kernel(GemmDesc d) {
    __shared__ float As[VBK][VBM + 4];
    __shared__ float Bs[VBK][VBN + 4];
    const int tid = threadIdx.x;
    const int g = blockIdx.z;
    const int64_t m0 = (int64_t)blockIdx.x * VBM;
    const int n0 = blockIdx.y * VBN;
    const TS* A = (const TS*)d.A + (int64_t)g * d.a_gs;
    const TS* B = (const TS*)d.B + (int64_t)g * d.b_gs;
    TS* C = (TS*)d.C;
    const int tx = tid & 15, ty = tid >> 4;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < d.K; k0 += VBK) {
#pragma unroll
        for (int e = tid; e < VBM * VBK; e += 256) {
            const int row = e / VBK, kk = e % VBK;
            const int64_t m = m0 + row;
            const int k = k0 + kk;
            float a = 0.f, b = 0.f;
            if (m < d.M && k < d.K) a = load_as_float(A + m * d.a_rs + (d.a_seg ? (int64_t)(k / d.a_seg) * d.a_seg_stride + k % d.a_seg : k));
            const int n = n0 + row;
            if (n < d.N && k < d.K) {
                const int64_t nr = d.b_div ? (int64_t)(n % d.b_div) * d.b_mul + n / d.b_div : n;
                b = load_as_float(B + nr * d.b_rs + (int64_t)k * d.b_ks);
            }
            As[kk][row] = a;
            Bs[kk][row] = b;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < VBK; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + ty * 4 + i;
        if (m >= d.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= d.N) continue;
            const int64_t col = (int64_t)g * d.c_gs + (int64_t)(n / d.c_div) * d.c_hi + (int64_t)(n % d.c_div) * d.c_lo;
            store_from_float(C + m * d.c_rs + col, acc[i][j]);
        }
    }
}

// one thread per (t, i, rho)
template <typename TS>
__global__ __launch_bounds__(256) void coupling_valu_kernel(const TS* Z, const TS* S, TS* A, int64_t T, int b, int r) {
    const int64_t total = T * b * r;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int rho = (int)(e % r);
        const int i = (int)((e / r) % b);
        const int64_t t = e / ((int64_t)r * b);
        float acc = 0.f;
        for (int j = 0; j < b; ++j)
            acc = fmaf(load_as_float(S + ((int64_t)i * b + j) * r + rho),
                       load_as_float(Z + (t * b + j) * r + rho), acc);
        store_from_float(A + e, acc);
    }
}

}  // namespace

hipError_t launch_gemm_valu(const GemmDesc& d, DType dt, hipStream_t s) {
    if (d.M <= 0 || d.N <= 0 || d.G <= 0) return hipSuccess;
    dim3 grid((unsigned)((d.M + VBM - 1) / VBM), (unsigned)((d.N + VBN - 1) / VBN), (unsigned)d.G);
    if (dt == DType::F32)
        hipLaunchKernelGGL(gemm_valu_kernel<float>, grid, dim3(256), 0, s, d);
    else
        hipLaunchKernelGGL(gemm_valu_kernel<bf16_t>, grid, dim3(256), 0, s, d);
    return hipGetLastError();
}

hipError_t launch_coupling_valu(const void* Z, const void* S, void* A, int64_t T, int b, int r, DType dt, hipStream_t s) {
    const int64_t total = T * b * r;
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536 * 16) blocks = 65536 * 16;
    if (dt == DType::F32)
        hipLaunchKernelGGL(coupling_valu_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s,
                           (const float*)Z, (const float*)S, (float*)A, T, b, r);
    else
        hipLaunchKernelGGL(coupling_valu_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, s,
                           (const bf16_t*)Z, (const bf16_t*)S, (bf16_t*)A, T, b, r);
    return hipGetLastError();
}

}  // namespace blr
