// bf16 MFMA batched "NT" GEMM for gfx950 with index maps on the B rows and the C columns.
//
// A workgroup of WGM x WGN wavefronts owns a BM x BN output tile; each wavefront owns
// (BM/WGM) x (BN/WGN) as a grid of 32x32 v_mfma_f32_32x32x16_bf16 tiles with fp32 accumulators.
// Operand tiles (BM x BK of A, BN x BK of B, both with the contraction index contiguous) go
// global -> registers -> LDS with 16-byte accesses, LDS double-buffered, one barrier per BK step,
// with a register ring of D steps of global loads in flight. LDS rows are padded by 16 bytes so
// that the 16-byte fragment reads of a wavefront fall into distinct banks.
// The weight tile is the FIRST MFMA operand: an accumulator lane then holds four consecutive
// output columns of one token, which go to an LDS copy of the C tile as 8-byte writes and from
// there to global memory as 16-byte row-contiguous stores (or element-wise through the column map
// when the map scatters).
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin over the 8 XCDs) owns a
// contiguous range of tiles, walked in groups of 8 row-tiles per column-tile, so the operand
// panels an XCD touches at one time fit its own L2.
#include "blr_common.h"

namespace blr {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

template <int BM, int BN, int BK, int WGM, int WGN>
struct TileCfg {
    static constexpr int THREADS = 64 * WGM * WGN;
    static constexpr int CPR = BK / 8;              // 16-byte chunks per tile row
    static constexpr int RPP = THREADS / CPR;       // tile rows covered by one pass of the workgroup
    static constexpr int NA = BM / RPP;             // passes for the A tile
    static constexpr int NB = BN / RPP;             // passes for the B tile
    static constexpr int STR = BK * 2 + 16;         // LDS row stride in bytes
    static constexpr int A_BYTES = BM * STR;
    static constexpr int B_BYTES = BN * STR;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int CSTR = BN * 2 + 16;        // row stride of the staged C tile
    static constexpr int C_BYTES = BM * CSTR;
    static constexpr int LDS_BYTES = 2 * STAGE > C_BYTES ? 2 * STAGE : C_BYTES;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int MI = WTM / 32, NI = WTN / 32;
    static_assert(NA >= 1 && NB >= 1 && MI >= 1 && NI >= 1, "tile too small");
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile rows must be a multiple of one load pass");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

__device__ inline int xcd_contiguous(int bid, int nblk) {
    const int q8 = nblk >> 3, rem = nblk & 7;
    const int xcd = bid & 7, slot = bid >> 3;
    return xcd * q8 + (xcd < rem ? xcd : rem) + slot;
}

template <int BM, int BN, int BK, int WGM, int WGN, int D>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_mfma_kernel(GemmDesc d, int tiles_m, int tiles_n, int cvec, int gfast) {
    using C = TileCfg<BM, BN, BK, WGM, WGN>;
    static_assert(D % 2 == 0, "the ring slot parity must equal the LDS stage parity");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    // tile and batch index of this workgroup. With a scattering column map (gfast) the batch index
    // varies fastest, so the G workgroups that interleave their columns into the same cache lines
    // run side by side on one XCD and their partial-line writes merge in its L2.
    constexpr int GM = 8;
    int g, logical;
    if (gfast) {
        const int lg = xcd_contiguous(blockIdx.x, tiles_m * tiles_n * d.G);
        g = lg % d.G;
        logical = lg / d.G;
    } else {
        g = blockIdx.y;
        logical = xcd_contiguous(blockIdx.x, tiles_m * tiles_n);
    }
    const int group_size = GM * tiles_n;
    const int first_m = (logical / group_size) * GM;
    const int gm = tiles_m - first_m < GM ? tiles_m - first_m : GM;
    const int in_group = logical % group_size;
    const int tile_m = first_m + in_group % gm;
    const int tile_n = in_group / gm;
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
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
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

    // epilogue. Every step ends with a barrier, so the operand stages are dead here and the C tile may
    // overwrite them. With the weight fragment as first operand, accumulator element e of tile (i, j)
    // is output column j*32 + 8*(e/4) + 4*(lane/32) + e%4 of token i*32 + lane%32.
    unsigned char* Cs = smem;
    {
        const int mrow = wm * C::WTM + (lane & 31);
        const int ncol = wn * C::WTN + 4 * (lane >> 5);
#pragma unroll
        for (int i = 0; i < C::MI; ++i)
#pragma unroll
            for (int j = 0; j < C::NI; ++j)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *(uint2*)(Cs + (mrow + i * 32) * C::CSTR + (ncol + j * 32 + 8 * q4) * 2) =
                        make_uint2(pack2_bf16(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1]),
                                   pack2_bf16(acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]));
    }
    __syncthreads();
    bf16_t* Cp = (bf16_t*)d.C;
    if (cvec) {
        // groups of 8 consecutive columns map to 8 consecutive, 16-byte aligned elements of C
        constexpr int CPRC = BN / 8;
        for (int id = tid; id < BM * CPRC; id += C::THREADS) {
            const int row = id / CPRC, cc = id % CPRC;
            const int64_t m = m0 + row;
            const int n = n0 + cc * 8;
            if (m < d.M && n < d.N) {
                const int64_t col = (int64_t)g * d.c_gs + (int64_t)(n / d.c_div) * d.c_hi + (int64_t)(n % d.c_div) * d.c_lo;
                *(uint4*)(Cp + m * d.c_rs + col) = *(const uint4*)(Cs + row * C::CSTR + cc * 16);
            }
        }
    } else {
        for (int id = tid; id < BM * BN; id += C::THREADS) {
            const int row = id / BN, nn = id % BN;
            const int64_t m = m0 + row;
            const int n = n0 + nn;
            if (m < d.M && n < d.N) {
                const int64_t col = (int64_t)g * d.c_gs + (int64_t)(n / d.c_div) * d.c_hi + (int64_t)(n % d.c_div) * d.c_lo;
                Cp[m * d.c_rs + col] = *(const bf16_t*)(Cs + row * C::CSTR + nn * 2);
            }
        }
    }
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// can 8 consecutive (8-aligned) tile columns be stored as one 16-byte vector?
inline bool c_map_vectorizes(const GemmDesc& d) {
    if (!aligned16(d.C) || d.c_rs % 8 || d.N % 8 || d.c_gs % 8) return false;
    if (d.c_div == 1) return d.c_hi == 1;
    return d.c_div % 8 == 0 && d.c_lo == 1 && d.c_hi % 8 == 0;
}

template <int BM, int BN, int BK, int WGM, int WGN, int D>
hipError_t launch_cfg(const GemmDesc& d, hipStream_t s) {
    using C = TileCfg<BM, BN, BK, WGM, WGN>;
    static bool attr_set = false;   // benign if set twice
    auto kern = gemm_mfma_kernel<BM, BN, BK, WGM, WGN, D>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (int)((d.M + BM - 1) / BM);
    const int tiles_n = (d.N + BN - 1) / BN;
    const bool vec = c_map_vectorizes(d);
    const bool gfast = !vec && d.G > 1 && (int64_t)tiles_m * tiles_n * d.G < (1ll << 31);
    dim3 grid(gfast ? (unsigned)(tiles_m * tiles_n * d.G) : (unsigned)(tiles_m * tiles_n), gfast ? 1u : (unsigned)d.G);
    hipLaunchKernelGGL(kern, grid, dim3(C::THREADS), C::LDS_BYTES, s, d, tiles_m, tiles_n, vec ? 1 : 0, gfast ? 1 : 0);
    return hipGetLastError();
}

}  // namespace

bool mfma_gemm_supported(const GemmDesc& d) {
    return d.b_ks == 1 && d.K % 8 == 0 && d.a_rs % 8 == 0 && d.a_gs % 8 == 0 && d.b_rs % 8 == 0 &&
           d.b_gs % 8 == 0 && aligned16(d.A) && aligned16(d.B) && d.M > 0 && d.N > 0 && d.K > 0 &&
           (int64_t)((d.M + 63) / 64) * ((d.N + 63) / 64) < (1ll << 30) && d.G <= 65535;
}

hipError_t launch_gemm_mfma(const GemmDesc& d, hipStream_t s) {
    constexpr int kSmallK = 256;     // short contractions: 128 x 128 tiles, two workgroups per CU overlap prologue and epilogue
    const bool k64 = (d.K % 64 == 0);
    // large problems: 256 x 256 tiles on 8 wavefronts (half the LDS and L2 traffic per FLOP of 128 x 128)
    if (d.M > 128 && d.N > 128 && d.K > kSmallK && (int64_t)((d.M + 255) / 256) * ((d.N + 255) / 256) * d.G >= 256)
        return k64 ? launch_cfg<256, 256, 64, 2, 4, 2>(d, s) : launch_cfg<256, 256, 32, 2, 4, 2>(d, s);
    if (d.M > 64 && d.N > 64) return k64 ? launch_cfg<128, 128, 64, 2, 2, 2>(d, s) : launch_cfg<128, 128, 32, 2, 2, 4>(d, s);
    if (d.M > 64)             return k64 ? launch_cfg<128, 64, 64, 2, 2, 2>(d, s) : launch_cfg<128, 64, 32, 2, 2, 4>(d, s);
    if (d.N > 64)             return k64 ? launch_cfg<64, 128, 64, 2, 2, 2>(d, s) : launch_cfg<64, 128, 32, 2, 2, 4>(d, s);
    return k64 ? launch_cfg<64, 64, 64, 2, 2, 4>(d, s) : launch_cfg<64, 64, 32, 2, 2, 4>(d, s);
}

}  // namespace blr
