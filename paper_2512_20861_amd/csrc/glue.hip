// Row-wise and elementwise glue between the BLR linears of a decoder-layer chain (paper Section 5
// replaces the projections and the MLP of Llama decoder layers with BLR linears; what sits between
// them here is a weightless RMS normalisation, the residual additions, the mean of the q/k/v
// branches and the SiLU gate of the MLP). bf16 or fp32 storage, fp32 arithmetic, 16-byte accesses
// where the row length and the pointers allow. All of it is HBM-bound streaming work.
#include "../../include/blr.h"
#include "blr_common.h"

namespace blr {
namespace {

template <typename TS> struct Vec;                       // 16 bytes of storage type TS <-> floats
template <> struct Vec<float> {
    static constexpr int N = 4;
    static __device__ inline void load(const float* p, float (&v)[4]) { const float4 t = *(const float4*)p; v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; }
    static __device__ inline void store(float* p, const float (&v)[4]) { *(float4*)p = make_float4(v[0], v[1], v[2], v[3]); }
    static __device__ inline float load1(const float* p) { return *p; }
    static __device__ inline void store1(float* p, float v) { *p = v; }
    static __device__ inline float round(float v) { return v; }
};
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    static __device__ inline void load(const bf16_t* p, float (&v)[8]) {
        const uint4 t = *(const uint4*)p;
        const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { v[2 * i] = __uint_as_float(w[i] << 16); v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
    }
    static __device__ inline void store(bf16_t* p, const float (&v)[8]) {
        *(uint4*)p = make_uint4(pack2_bf16(v[0], v[1]), pack2_bf16(v[2], v[3]), pack2_bf16(v[4], v[5]), pack2_bf16(v[6], v[7]));
    }
    static __device__ inline float load1(const bf16_t* p) { return bf16_to_float(*p); }
    static __device__ inline void store1(bf16_t* p, float v) { *p = float_to_bf16(v); }
    static __device__ inline float round(float v) { return bf16_to_float(float_to_bf16(v)); }
};

__device__ inline float silu(float x) { return x / (1.f + __expf(-x)); }

// One workgroup per row: optional residual addition H += Y (stored back, rounded to the storage type),
// then N = H / sqrt(mean(H^2) + eps) from the stored values. The second sweep re-reads the row, which
// the first sweep left in L2. VEC: d is a multiple of the vector width and all pointers are 16-byte aligned.
template <typename TS, bool VEC>
__global__ __launch_bounds__(256) void add_rmsnorm_kernel(TS* __restrict__ H, const TS* __restrict__ Y, TS* __restrict__ Nout,
                                                          int d, float eps) {
    using V = Vec<TS>;
    __shared__ float red[4];
    const int tid = threadIdx.x;
    TS* h = H + (int64_t)blockIdx.x * d;
    const TS* y = Y ? Y + (int64_t)blockIdx.x * d : nullptr;
    float ss = 0.f;
    if (VEC) {
        for (int c = tid * V::N; c < d; c += 256 * V::N) {
            float a[V::N];
            V::load(h + c, a);
            if (y) {
                float b[V::N];
                V::load(y + c, b);
#pragma unroll
                for (int i = 0; i < V::N; ++i) a[i] = V::round(a[i] + b[i]);
                V::store(h + c, a);
            }
#pragma unroll
            for (int i = 0; i < V::N; ++i) ss += a[i] * a[i];
        }
    } else {
        for (int c = tid; c < d; c += 256) {
            float a = V::load1(h + c);
            if (y) { a = V::round(a + V::load1(y + c)); V::store1(h + c, a); }
            ss += a * a;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();                                     // (each thread re-reads only what it wrote itself)
    if (!Nout) return;
    const float scale = rsqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
    TS* n = Nout + (int64_t)blockIdx.x * d;
    if (VEC) {
        for (int c = tid * V::N; c < d; c += 256 * V::N) {
            float a[V::N];
            V::load(h + c, a);
#pragma unroll
            for (int i = 0; i < V::N; ++i) a[i] *= scale;
            V::store(n + c, a);
        }
    } else {
        for (int c = tid; c < d; c += 256) V::store1(n + c, V::load1(h + c) * scale);
    }
}

// OP 0: O = (A + B + C) * scale;  OP 1: O = silu(A) * B;  OP 2: O = A + B  (O may alias A)
template <typename TS, int OP, bool VEC>
__global__ __launch_bounds__(256) void elementwise_kernel(const TS* A, const TS* B, const TS* C, TS* O, int64_t n, float scale) {
    using V = Vec<TS>;
    const int64_t stride = (int64_t)gridDim.x * 256;
    if (VEC) {
        for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v * V::N < n; v += stride) {
            float a[V::N], b[V::N], c[V::N];
            V::load(A + v * V::N, a);
            V::load(B + v * V::N, b);
            if (OP == 0) V::load(C + v * V::N, c);
#pragma unroll
            for (int i = 0; i < V::N; ++i) a[i] = OP == 0 ? (a[i] + b[i] + c[i]) * scale : OP == 1 ? silu(a[i]) * b[i] : a[i] + b[i];
            V::store(O + v * V::N, a);
        }
    } else {
        for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += stride) {
            const float a = V::load1(A + e), b = V::load1(B + e);
            V::store1(O + e, OP == 0 ? (a + b + V::load1(C + e)) * scale : OP == 1 ? silu(a) * b : a + b);
        }
    }
}

// The same operations on inputs whose rows are `ld` elements apart (column slices of a wider tensor, e.g.
// the outputs of several layers computed by one call side by side); the output rows are contiguous.
// One workgroup row per token row (grid-stride over rows), no index divisions.
template <typename TS, int OP, bool VEC>
__global__ __launch_bounds__(256) void elementwise_rows_kernel(const TS* A, const TS* B, const TS* C, TS* O, int64_t T, int d, int64_t ld, float scale) {
    using V = Vec<TS>;
    for (int64_t t = blockIdx.y; t < T; t += gridDim.y) {
        const TS *a_row = A + t * ld, *b_row = B + t * ld, *c_row = OP == 0 ? C + t * ld : nullptr;
        TS* o_row = O + t * (int64_t)d;
        if (VEC) {
            for (int v = blockIdx.x * 256 + threadIdx.x; v * V::N < d; v += gridDim.x * 256) {
                float a[V::N], b[V::N], c[V::N];
                V::load(a_row + v * V::N, a);
                V::load(b_row + v * V::N, b);
                if (OP == 0) V::load(c_row + v * V::N, c);
#pragma unroll
                for (int i = 0; i < V::N; ++i) a[i] = OP == 0 ? (a[i] + b[i] + c[i]) * scale : silu(a[i]) * b[i];
                V::store(o_row + v * V::N, a);
            }
        } else {
            for (int e = blockIdx.x * 256 + threadIdx.x; e < d; e += gridDim.x * 256) {
                const float a = V::load1(a_row + e), b = V::load1(b_row + e);
                V::store1(o_row + e, OP == 0 ? (a + b + V::load1(c_row + e)) * scale : silu(a) * b);
            }
        }
    }
}

inline bool al16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

template <typename TS>
hipError_t run_add_rmsnorm(void* H, const void* Y, void* N, int64_t T, int d, float eps, hipStream_t s) {
    const bool vec = d % Vec<TS>::N == 0 && al16(H) && al16(Y) && al16(N);
    if (vec) hipLaunchKernelGGL((add_rmsnorm_kernel<TS, true>), dim3((unsigned)T), dim3(256), 0, s, (TS*)H, (const TS*)Y, (TS*)N, d, eps);
    else hipLaunchKernelGGL((add_rmsnorm_kernel<TS, false>), dim3((unsigned)T), dim3(256), 0, s, (TS*)H, (const TS*)Y, (TS*)N, d, eps);
    return hipGetLastError();
}

template <typename TS, int OP>
hipError_t run_elementwise(const void* A, const void* B, const void* C, void* O, int64_t n, float scale, hipStream_t s) {
    const bool vec = n % Vec<TS>::N == 0 && al16(A) && al16(B) && al16(C) && al16(O);
    const int64_t items = vec ? n / Vec<TS>::N : n;
    int64_t blocks = (items + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;           // grid-stride beyond 16 workgroups per compute unit
    if (vec) hipLaunchKernelGGL((elementwise_kernel<TS, OP, true>), dim3((unsigned)blocks), dim3(256), 0, s, (const TS*)A, (const TS*)B, (const TS*)C, (TS*)O, n, scale);
    else hipLaunchKernelGGL((elementwise_kernel<TS, OP, false>), dim3((unsigned)blocks), dim3(256), 0, s, (const TS*)A, (const TS*)B, (const TS*)C, (TS*)O, n, scale);
    return hipGetLastError();
}

template <typename TS, int OP>
hipError_t run_elementwise_rows(const void* A, const void* B, const void* C, void* O, int64_t T, int d, int64_t ld, float scale, hipStream_t s) {
    const bool vec = d % Vec<TS>::N == 0 && ld % Vec<TS>::N == 0 && al16(A) && al16(B) && (OP != 0 || al16(C)) && al16(O);
    const int items = vec ? d / Vec<TS>::N : d;
    int bx = (items + 255) / 256;
    if (bx > 64) bx = 64;
    const dim3 grid((unsigned)bx, (unsigned)(T < 65535 ? T : 65535));
    if (vec) hipLaunchKernelGGL((elementwise_rows_kernel<TS, OP, true>), grid, dim3(256), 0, s, (const TS*)A, (const TS*)B, (const TS*)C, (TS*)O, T, d, ld, scale);
    else hipLaunchKernelGGL((elementwise_rows_kernel<TS, OP, false>), grid, dim3(256), 0, s, (const TS*)A, (const TS*)B, (const TS*)C, (TS*)O, T, d, ld, scale);
    return hipGetLastError();
}

inline blr_status status_of(hipError_t e) { return e == hipSuccess ? BLR_OK : BLR_ERR_LAUNCH; }
inline bool dims_ok(int64_t T, int d, blr_dtype dt) { return T >= 0 && d > 0 && T < (1ll << 31) && (dt == BLR_F32 || dt == BLR_BF16); }

}  // namespace
}  // namespace blr

using namespace blr;

extern "C" {

blr_status blr_rmsnorm(const void* H, void* N, int64_t T, int d, float eps, blr_dtype dt, blr_stream stream) {
    if (!dims_ok(T, d, dt) || !(eps >= 0.f)) return BLR_ERR_INVALID_ARG;
    if (T == 0) return BLR_OK;
    if (!H || !N || H == N) return BLR_ERR_INVALID_ARG;
    // the kernel only writes H when a residual is given
    return status_of(dt == BLR_BF16 ? run_add_rmsnorm<bf16_t>((void*)H, nullptr, N, T, d, eps, (hipStream_t)stream)
                                    : run_add_rmsnorm<float>((void*)H, nullptr, N, T, d, eps, (hipStream_t)stream));
}

blr_status blr_residual_add_rmsnorm(void* H, const void* Y, void* N, int64_t T, int d, float eps, blr_dtype dt, blr_stream stream) {
    if (!dims_ok(T, d, dt) || !(eps >= 0.f)) return BLR_ERR_INVALID_ARG;
    if (T == 0) return BLR_OK;
    if (!H || !Y || H == Y || H == N || Y == N) return BLR_ERR_INVALID_ARG;
    return status_of(dt == BLR_BF16 ? run_add_rmsnorm<bf16_t>(H, Y, N, T, d, eps, (hipStream_t)stream)
                                    : run_add_rmsnorm<float>(H, Y, N, T, d, eps, (hipStream_t)stream));
}

blr_status blr_sum3_scaled(const void* Q, const void* K, const void* V, void* A, int64_t T, int d, float scale, blr_dtype dt, blr_stream stream) {
    if (!dims_ok(T, d, dt)) return BLR_ERR_INVALID_ARG;
    if (T == 0) return BLR_OK;
    if (!Q || !K || !V || !A) return BLR_ERR_INVALID_ARG;
    return status_of(dt == BLR_BF16 ? run_elementwise<bf16_t, 0>(Q, K, V, A, T * d, scale, (hipStream_t)stream)
                                    : run_elementwise<float, 0>(Q, K, V, A, T * d, scale, (hipStream_t)stream));
}

blr_status blr_silu_mul(const void* G, const void* U, void* M, int64_t T, int d, blr_dtype dt, blr_stream stream) {
    if (!dims_ok(T, d, dt)) return BLR_ERR_INVALID_ARG;
    if (T == 0) return BLR_OK;
    if (!G || !U || !M) return BLR_ERR_INVALID_ARG;
    return status_of(dt == BLR_BF16 ? run_elementwise<bf16_t, 1>(G, U, nullptr, M, T * d, 1.f, (hipStream_t)stream)
                                    : run_elementwise<float, 1>(G, U, nullptr, M, T * d, 1.f, (hipStream_t)stream));
}

blr_status blr_sum3_scaled_ld(const void* Q, const void* K, const void* V, void* A, int64_t T, int d, int64_t ld, float scale,
                              blr_dtype dt, blr_stream stream) {
    if (!dims_ok(T, d, dt) || ld < d) return BLR_ERR_INVALID_ARG;
    if (T == 0) return BLR_OK;
    if (!Q || !K || !V || !A) return BLR_ERR_INVALID_ARG;
    return status_of(dt == BLR_BF16 ? run_elementwise_rows<bf16_t, 0>(Q, K, V, A, T, d, ld, scale, (hipStream_t)stream)
                                    : run_elementwise_rows<float, 0>(Q, K, V, A, T, d, ld, scale, (hipStream_t)stream));
}

blr_status blr_silu_mul_ld(const void* G, const void* U, void* M, int64_t T, int d, int64_t ld, blr_dtype dt, blr_stream stream) {
    if (!dims_ok(T, d, dt) || ld < d) return BLR_ERR_INVALID_ARG;
    if (T == 0) return BLR_OK;
    if (!G || !U || !M) return BLR_ERR_INVALID_ARG;
    return status_of(dt == BLR_BF16 ? run_elementwise_rows<bf16_t, 1>(G, U, nullptr, M, T, d, ld, 1.f, (hipStream_t)stream)
                                    : run_elementwise_rows<float, 1>(G, U, nullptr, M, T, d, ld, 1.f, (hipStream_t)stream));
}

}  // extern "C"
