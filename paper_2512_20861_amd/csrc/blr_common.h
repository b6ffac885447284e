// Internal declarations shared by the kernel translation units and the C-ABI front end.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <initializer_list>
#include <mutex>
#include <utility>

namespace blr {

// compile-time loop: f(std::integral_constant<int, 0>{}) ... f(std::integral_constant<int, N-1>{})
template <class F, int... I>
__host__ __device__ inline void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__host__ __device__ inline void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

typedef unsigned short bf16_t;  // bfloat16 bit pattern

// Raises the dynamic-LDS limit of the given kernels exactly once per process, also when several host
// threads make their first call at the same time; every caller gets the outcome of that one attempt.
struct LdsLimitOnce {
    std::once_flag flag;
    hipError_t err = hipSuccess;
    hipError_t set(std::initializer_list<const void*> kernels, int bytes) {
        std::call_once(flag, [&] {
            for (const void* k : kernels) {
                err = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
                if (err != hipSuccess) return;
            }
        });
        return err;
    }
};

// Workgroup id -> logical work item id such that each XCD (the hardware deals workgroup ids round-robin
// over the 8 XCDs) works on a contiguous range of logical ids: neighbours in logical order share an L2.
__device__ inline int xcd_contiguous(int bid, int nblk) {
    const int q8 = nblk >> 3, rem = nblk & 7;
    const int xcd = bid & 7, slot = bid >> 3;
    return xcd * q8 + (xcd < rem ? xcd : rem) + slot;
}

__host__ __device__ inline float bf16_to_float(bf16_t v) {
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)v << 16;
    return c.f;
}
// round to nearest even (inputs are finite); on the device this is the hardware conversion
__host__ __device__ inline bf16_t float_to_bf16(float f) {
#if defined(__HIP_DEVICE_COMPILE__)
    const __bf16 h = (__bf16)f;
    return __builtin_bit_cast(bf16_t, h);
#else
    union { uint32_t u; float f; } c;
    c.f = f;
    uint32_t u = c.u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
#endif
}
// two floats -> two bf16 in one 32-bit word (lo in the low half): one v_cvt_pk_bf16_f32
__device__ inline uint32_t pack2_bf16(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    const bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}

// pointer casts for __builtin_amdgcn_global_load_lds (global -> LDS without staging registers:
// lane l of the wavefront deposits its 16 bytes at the wavefront-uniform LDS address + 16 l)
#define BLR_GPTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define BLR_LPTR(p) ((void __attribute__((address_space(3)))*)(p))

// value select (a ternary on two uint4 lvalues would select an address and force them into memory)
__device__ inline uint4 keep_if(bool ok, uint4 v) {
    return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
}

// A batched "NT" product with index maps, general enough for every contraction of the path:
//   C(g, m, n) = sum_k A(g, m, k) * B(g, n, k),  g < G, m < M, n < N, k < K
// element addresses (in elements of the storage type):
//   A(g,m,k) = A + g*a_gs + m*a_rs + k
//   B(g,n,k) = B + g*b_gs + brow(n)*b_rs + k*b_ks,  brow(n) = (n % b_div)*b_mul + n / b_div   (row gather)
//   C(g,m,n) = C + m*c_rs + g*c_gs + (n / c_div)*c_hi + (n % c_div)*c_lo                       (column scatter)
// b_div = N, b_mul = 1... is written as b_div = 0 meaning brow(n) = n.
struct GemmDesc {
    const void* A; int64_t a_gs; int64_t a_rs;
    int a_seg; int64_t a_seg_stride;   // a_seg > 0: contraction index k of A lives at (k / a_seg) * a_seg_stride + k % a_seg
    const void* B; int64_t b_gs; int64_t b_rs; int64_t b_ks; int b_div; int b_mul;
    void* C; int64_t c_rs; int64_t c_gs; int c_div; int64_t c_hi; int64_t c_lo;
    int64_t M; int N; int K; int G;
    float* split_scratch; size_t split_scratch_bytes;   // optional: room for fp32 partial tiles of a split contraction
    int c_fp8;                         // C is stored as 8-bit floats (E4M3, round to nearest even, clamped to +-448): one byte per
                                       // element, strides and offsets of C then count bytes; tile kernels of launch_gemm_mfma only
};

enum class DType { F32 = 0, BF16 = 1 };

// portable scalar-ALU kernels (any shape, any stride, fp32 accumulation)
hipError_t launch_gemm_valu(const GemmDesc& d, DType dt, hipStream_t s);
// A[t][i][rho] = sum_j S[i][j][rho] * Z[t][j][rho], Z and A are [T][b][r]
hipError_t launch_coupling_valu(const void* Z, const void* S, void* A, int64_t T, int b, int r, DType dt, hipStream_t s);

// first Monarch factor re-ordered for an input in blocked order: Rp[l][c][k*(p/b)+jj] = R[l][c][jj*b+k]
hipError_t launch_monarch_permute_first_factor(const void* R, void* Rp, int n_in, int nblocks, int r, DType dt, hipStream_t s);
// first factors of `members` layers that share their input, stacked [members][b][r][p] -> one layer with members*b output blocks
hipError_t launch_monarch_group_first_factor(const void* Rs, void* Rg, int n_in, int nblocks, int r, int members, DType dt, hipStream_t s);
// blocked -> interleaved output order of a bf16 Monarch result, Y[t][j*b2 + k] = Yb[t][k*(n_out/b2) + j]
// (b2 a power of two up to 64, 8 | n_out/b2)
bool monarch_interleave_supported(int64_t T, int n_out, int b2);
hipError_t launch_monarch_interleave(const void* Yb, void* Y, int64_t T, int n_out, int b2, hipStream_t s);

// bf16 MFMA kernels; `mfma_gemm_supported` states the alignment contract
bool mfma_gemm_supported(const GemmDesc& d);
hipError_t launch_gemm_mfma(const GemmDesc& d, hipStream_t s);
// scratch bytes with which launch_gemm_mfma may split the contraction index of an (M, N, K, G) product
// over several workgroups per tile (0: it would not split)
size_t gemm_split_scratch_bytes(int64_t M, int N, int K, int G);
// can C of this product be written as 8-bit floats (16 consecutive columns = 16 contiguous, aligned bytes)?
bool gemm_fp8_store_supported(const GemmDesc& d);
// few tokens (M <= 32): weight-streaming kernel, split-K inside the workgroup; same alignment contract
bool skinny_gemm_supported(const GemmDesc& d);
hipError_t launch_gemm_skinny(const GemmDesc& d, bool cvec, hipStream_t s);
// the same kernel over tiles of 32 tokens (the weights are streamed once per tile): for products with
// too few 64 x 64 tiles to fill the chip and a long contraction index
bool skinny_gemm_tiled_supported(const GemmDesc& d);

// Monarch (b1 input blocks, b2 output blocks, per-block rank rp; low-rank is b1 = b2 = 1) in one kernel
// for narrow layers: the intermediate stays on chip. Needs 16 | rp, 32 | n_in/b1, 32 | b1 rp and a token
// tile plus intermediate that fit LDS.
bool monarch_fused_supported(int64_t T, int n_in, int n_out, int b1, int b2, int rp);
int monarch_fused_lds_bytes(int64_t T, int n_in, int n_out, int b1, int b2, int rp);   // of a supported call
hipError_t launch_monarch_fused(const void* X, const void* R, const void* L, void* Y, int64_t T, int n_in, int n_out,
                                int b1, int b2, int rp, bool out_blocked, hipStream_t s);

// BLAST: fused stage 1 + coupling on MFMA. X[T][n_in], Vt[b][r][q], Sp[r][16][16] -> A[T][b][r] (bf16)
bool blast_fused_supported(int64_t T, int n_in, int b, int r);
int64_t blast_fused_tiles(int64_t T, int r);                 // workgroups the fused stage 1 + coupling kernel would launch
hipError_t launch_blast_stage12(const void* X, const void* Vt, const void* Sp, void* A,
                                int64_t T, int n_in, int b, int r, hipStream_t s);
// BLAST: stand-alone coupling on MFMA, Z[T][b][r] -> A[T][b][r] (bf16), S tiles from Sp[r][16][16]; needs r % 8 == 0, b <= 16
hipError_t launch_blast_coupling(const void* Z, const void* Sp, void* A, int64_t T, int b, int r, hipStream_t s, bool z_fp8 = false);

// BLAST: whole layer in one kernel for small ranks. Vf / Uf are V and U in MFMA-fragment order:
//   Vf[j][nt][ks][lane][e] = V[j][ks*16 + (lane/32)*8 + e][nt*32 + lane%32]      (zero past q, r)
//   Uf[i][nt][ks][lane][e] = U[i][nt*16 + lane%16][ks*32 + (lane/16)*8 + e]      (zero past r)
bool blast_full_fusion_shape_ok(int n_in, int n_out, int b, int r);
bool blast_full_fusion_supported(int64_t T, int n_in, int n_out, int b, int r);
size_t blast_vf_bytes(int n_in, int b, int r);
size_t blast_uf_bytes(int n_out, int b, int r);
hipError_t launch_blast_full(const void* X, const void* Sp, const void* Vf, const void* Uf, void* Y,
                             int64_t T, int n_in, int n_out, int b, int r, hipStream_t s);

// BLAST: whole layer in one kernel for few, wide blocks (q = n_in/b <= 256, r <= 256, 32 | q, 32 | r): a workgroup owns
// 32 tokens, one output block and a range of its outputs; the coupling is accumulated in registers.
// Vt[b][r][q] (contraction index contiguous), canonical S[b][b][r], U[b][p][r].
bool blast_narrow_supported(int64_t T, int n_in, int n_out, int b, int r);
int64_t blast_narrow_workgroups(int64_t T, int n_out, int b);
int blast_narrow_lds_bytes(int64_t T, int n_in, int n_out, int b, int r);   // of a supported call
hipError_t launch_blast_narrow(const void* X, const void* Vt, const void* S, const void* U, void* Y,
                               int64_t T, int n_in, int n_out, int b, int r, hipStream_t s);

// stand-alone coupling reading the packed tiles Sp[r][16][16] (bf16)
hipError_t launch_coupling_small(const void* Z, const void* S, void* A, int64_t T, int b, int r, hipStream_t s);   // few tokens; canonical S

// BLAST weight re-layout (bf16): Sp always; Vt (row-major transpose) if non-null; Vf and Uf if non-null
// the fused stage 1 + coupling kernel walks the contraction index in chunks aligned to this many GLOBAL input
// columns: 128 when the input blocks are whole numbers of such chunks (no padded boundary chunks; measured
// 4 % faster than 64 on 4096 x 4096, b = 16), else 64 (with q = 688 the deeper chunks' extra padding costs 1.5 %)
inline int blast_chunk(int n_in, int b) { return (n_in / b) % 128 == 0 ? 128 : 64; }
// elements per (j, rho) row of the chunk-aligned copy of Vt: the chunks of `chunk` columns a block of q columns can touch
inline int blast_va_row(int q, int chunk) { return q % chunk ? ((q + chunk - 1) / chunk + 1) * chunk : q; }
hipError_t launch_blast_pack(const void* U, const void* S, const void* V, void* Sp, void* Sc, void* Vt, void* Va, void* Vf, void* Uf,
                             int n_in, int n_out, int b, int r, hipStream_t s);

}  // namespace blr
