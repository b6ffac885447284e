// bf16 MFMA batched "NT" GEMM for gfx950 with index maps on the B rows and the C columns.
//
// Workgroup = 256 threads = 4 wavefronts in a 2x2 arrangement over a BM x BN output tile; each
// wavefront owns (BM/2) x (BN/2) as a grid of 32x32 v_mfma_f32_32x32x16_bf16 tiles with fp32
// accumulators. Operand tiles (BM x BK of A, BN x BK of B, both with the contraction index
// contiguous) go global -> registers -> LDS with 16-byte accesses, double-buffered, one barrier
// per BK step. LDS rows are padded by 16 bytes so that the 16-byte fragment reads of the lanes
// of a wavefront fall into distinct banks.
#include "blr_common.h"

namespace blr {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

template <int BM, int BN, int BK>
struct TileCfg {
    static constexpr int CPR = BK / 8;              // 16-byte chunks per tile row
    static constexpr int RPP = 256 / CPR;           // tile rows covered by one pass of the workgroup
    static constexpr int NA = BM / RPP;             // passes for the A tile
    static constexpr int NB = BN / RPP;             // passes for the B tile
    static constexpr int STR = BK * 2 + 16;         // LDS row stride in bytes
    static constexpr int A_BYTES = BM * STR;
    static constexpr int B_BYTES = BN * STR;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE;
    static constexpr int WTM = BM / 2, WTN = BN / 2;
    static constexpr int MI = WTM / 32, NI = WTN / 32;
    static_assert(NA >= 1 && NB >= 1 && MI >= 1 && NI >= 1, "tile too small");
};

template <int BM, int BN, int BK, int D>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmDesc d, int tiles_m) {
    using C = TileCfg<BM, BN, BK>;
    static_assert(D % 2 == 0, "the ring slot parity must equal the LDS stage parity");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int g = blockIdx.y;
    const int tile_m = blockIdx.x % tiles_m;
    const int tile_n = blockIdx.x / tiles_m;
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;

    const bf16_t* Ag = (const bf16_t*)d.A + (int64_t)g * d.a_gs;
    const bf16_t* Bg = (const bf16_t*)d.B + (int64_t)g * d.b_gs;

    const int lrow = tid / C::CPR, lchunk = tid % C::CPR;
    const bf16_t* ap[C::NA];
    const bf16_t* bp[C::NB];
#pragma unroll
    for (int i = 0; i < C::NA; ++i) {
        int64_t m = m0 + lrow + i * C::RPP;
        if (m > d.M - 1) m = d.M - 1;               // rows past the end re-read the last row; never stored
        ap[i] = Ag + m * d.a_rs;
    }
#pragma unroll
    for (int i = 0; i < C::NB; ++i) {
        int n = n0 + lrow + i * C::RPP;
        if (n > d.N - 1) n = d.N - 1;
        const int64_t nr = d.b_div ? (int64_t)(n % d.b_div) * d.b_mul + n / d.b_div : n;
        bp[i] = Bg + nr * d.b_rs;
    }

    // Register ring: the global loads of steps s+1 .. s+D are in flight while step s is computed from
    // LDS, so HBM/L2 latency is covered by D steps of MFMA work. Slots are indexed statically (the
    // main loop is unrolled by D) and every load is unconditional (addresses are clamped, chunks past
    // K are zeroed when they are written to LDS), so each wait counts only the loads older than the
    // slot it needs instead of draining the queue.
    const int nk = (d.K + BK - 1) / BK;
    uint4 ra[D][C::NA], rb[D][C::NB];
    auto gload = [&](auto SLOT, int kt) {
        constexpr int slot = decltype(SLOT)::value;
        if (kt > nk - 1) kt = nk - 1;               // steps past the end repeat the last one; never consumed
        int k = kt * BK + lchunk * 8;
        if (k > d.K - 8) k = d.K - 8;               // K is a multiple of 8
#pragma unroll
        for (int i = 0; i < C::NA; ++i) ra[slot][i] = *(const uint4*)(ap[i] + k);
#pragma unroll
        for (int i = 0; i < C::NB; ++i) rb[slot][i] = *(const uint4*)(bp[i] + k);
    };
    auto sstore = [&](auto SLOT, int kt) {
        constexpr int slot = decltype(SLOT)::value;
        constexpr int stage = slot & 1;             // D is even: slot parity == step parity
        unsigned char* base = smem + stage * C::STAGE;
        const bool ok = (kt * BK + lchunk * 8) < d.K;
#pragma unroll
        for (int i = 0; i < C::NA; ++i) *(uint4*)(base + (lrow + i * C::RPP) * C::STR + lchunk * 16) = keep_if(ok, ra[slot][i]);
#pragma unroll
        for (int i = 0; i < C::NB; ++i) *(uint4*)(base + C::A_BYTES + (lrow + i * C::RPP) * C::STR + lchunk * 16) = keep_if(ok, rb[slot][i]);
    };

    f32x16 acc[C::MI][C::NI];
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int frag_off = (lane & 31) * C::STR + (lane >> 5) * 16;
    auto step = [&](auto U, int kt) {               // u = kt % D, a compile-time constant
        constexpr int u = decltype(U)::value;
        const unsigned char* As = smem + (u & 1) * C::STAGE + (wm * C::WTM) * C::STR + frag_off;
        const unsigned char* Bs = smem + (u & 1) * C::STAGE + C::A_BYTES + (wn * C::WTN) * C::STR + frag_off;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[C::MI], bfr[C::NI];
#pragma unroll
            for (int i = 0; i < C::MI; ++i) af[i] = *(const bf16x8*)(As + i * 32 * C::STR + ks * 32);
#pragma unroll
            for (int j = 0; j < C::NI; ++j) bfr[j] = *(const bf16x8*)(Bs + j * 32 * C::STR + ks * 32);
#pragma unroll
            for (int i = 0; i < C::MI; ++i)
#pragma unroll
                for (int j = 0; j < C::NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        sstore(std::integral_constant<int, (u + 1) % D>{}, kt + 1);   // past the last step this writes the unused stage
        gload(std::integral_constant<int, (u + 1) % D>{}, kt + 1 + D);
        __syncthreads();
    };

    static_for<D>([&](auto U) { gload(U, decltype(U)::value); });
    sstore(std::integral_constant<int, 0>{}, 0);
    gload(std::integral_constant<int, 0>{}, D);
    __syncthreads();
    int kt0 = 0;
    for (; kt0 + D <= nk; kt0 += D) static_for<D>([&](auto U) { step(U, kt0 + decltype(U)::value); });
    static_for<D - 1>([&](auto U) { if (kt0 + decltype(U)::value < nk) step(U, kt0 + decltype(U)::value); });

    // epilogue: accumulator element e of a 32x32 tile is row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
    bf16_t* Cp = (bf16_t*)d.C;
#pragma unroll
    for (int j = 0; j < C::NI; ++j) {
        const int n = n0 + wn * C::WTN + j * 32 + (lane & 31);
        if (n >= d.N) continue;
        const int64_t col = (int64_t)g * d.c_gs + (int64_t)(n / d.c_div) * d.c_hi + (int64_t)(n % d.c_div) * d.c_lo;
#pragma unroll
        for (int i = 0; i < C::MI; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t m = m0 + wm * C::WTM + i * 32 + 8 * (e / 4) + 4 * (lane >> 5) + (e % 4);
                if (m < d.M) Cp[m * d.c_rs + col] = float_to_bf16(acc[i][j][e]);
            }
        }
    }
}

template <int BM, int BN, int BK, int D>
hipError_t launch_cfg(const GemmDesc& d, hipStream_t s) {
    using C = TileCfg<BM, BN, BK>;
    static bool attr_set = false;   // benign if set twice
    auto kern = gemm_mfma_kernel<BM, BN, BK, D>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (int)((d.M + BM - 1) / BM);
    const int tiles_n = (d.N + BN - 1) / BN;
    dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)d.G);
    hipLaunchKernelGGL(kern, grid, dim3(256), C::LDS_BYTES, s, d, tiles_m);
    return hipGetLastError();
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

bool mfma_gemm_supported(const GemmDesc& d) {
    return d.b_ks == 1 && d.K % 8 == 0 && d.a_rs % 8 == 0 && d.a_gs % 8 == 0 && d.b_rs % 8 == 0 &&
           d.b_gs % 8 == 0 && aligned16(d.A) && aligned16(d.B) && d.M > 0 && d.N > 0 && d.K > 0 &&
           (int64_t)((d.M + 63) / 64) * ((d.N + 63) / 64) < (1ll << 30) && d.G <= 65535;
}

hipError_t launch_gemm_mfma(const GemmDesc& d, hipStream_t s) {
    const bool k64 = (d.K % 64 == 0);
    if (d.M > 64 && d.N > 64) return k64 ? launch_cfg<128, 128, 64, 2>(d, s) : launch_cfg<128, 128, 32, 4>(d, s);
    if (d.M > 64)             return k64 ? launch_cfg<128, 64, 64, 2>(d, s) : launch_cfg<128, 64, 32, 4>(d, s);
    if (d.N > 64)             return k64 ? launch_cfg<64, 128, 64, 2>(d, s) : launch_cfg<64, 128, 32, 4>(d, s);
    return k64 ? launch_cfg<64, 64, 64, 4>(d, s) : launch_cfg<64, 64, 32, 4>(d, s);
}

}  // namespace blr
