// bf16 MFMA batched "NT" GEMM for FEW tokens (M <= 32): the weight-streaming regime, HBM-bound. Also
// used tile by tile (32 tokens per workgroup, grid.y) for products with small weights, few 64 x 64
// tiles and a long contraction index, where the weights then come from L2.
//
// With few tokens the product is a stream of the weights through the chip, so the tiling is turned
// around: a workgroup owns 16 weight rows (output columns) and ALL tokens, and its four wavefronts
// split the contraction index between them (split-K inside the workgroup, summed through LDS in a
// fixed order, so results do not depend on timing). Every weight element is fetched from HBM exactly
// once, straight into v_mfma_f32_16x16x32_bf16 fragments (one 16-byte load per lane and k32 step,
// several steps in flight per wavefront to cover HBM latency); the token fragments come from L2.
// Many small workgroups (N/16 per batch entry) put every compute unit to work on the stream, which
// the square tiles of the large-problem kernel cannot do when there is only one row of tiles.
// The weight fragment is the first MFMA operand, as in the large kernel: an accumulator lane holds
// four consecutive output columns of one token. Same index maps on B rows and C columns.
#include "blr_common.h"

namespace blr {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int SK_BN = 16;             // weight rows per workgroup
constexpr int SK_WAVES = 4;           // wavefronts = K splits per workgroup

// MT: 16-token tiles (M <= 16 MT); D: k32 steps of loads in flight per wavefront
template <int MT, int D>
__global__ __launch_bounds__(64 * SK_WAVES) void gemm_skinny_kernel(GemmDesc d, int tiles_n, int cvec) {
    __shared__ __attribute__((aligned(16))) float part[SK_WAVES][MT * 16][SK_BN + 4];   // partial sums [wave][token][column]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x / tiles_n;
    const int n0 = (blockIdx.x % tiles_n) * SK_BN;
    const int l16 = lane & 15, kg = lane >> 4;          // fragment row, group of 8 consecutive k (of the step's 32)
    const int64_t m_base = (int64_t)blockIdx.y * (MT * 16);   // more tokens than one tile: grid.y walks tiles of 16 MT tokens

    // A fragment (16 rows x 32 k) is LOADED with four neighbouring lanes on the 64 contiguous bytes of one
    // row (lane = 4 row + piece: 16 requests of 64 bytes per instruction) and moved to the MFMA's order
    // (lane = 16 piece + row) by a cross-lane permute when it is used: loaded in the MFMA's order every
    // lane would be a 16-byte request of its own, which the load path serves several times slower.
    const int ld_row = lane >> 2, ld_piece = lane & 3;
    const int from_lane = (l16 * 4 + kg) * 4;           // byte index of the lane that loaded this lane's piece
    // fragment sources: weight row n0 + ld_row, token rows mt*16 + ld_row
    int n = n0 + ld_row;
    if (n > d.N - 1) n = d.N - 1;                       // rows past N repeat the last row; never stored
    const int64_t nr = d.b_div ? (int64_t)(n % d.b_div) * d.b_mul + n / d.b_div : n;
    const bf16_t* wp = (const bf16_t*)d.B + (int64_t)g * d.b_gs + nr * d.b_rs;
    const bf16_t* xp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int64_t m = m_base + mt * 16 + ld_row;
        if (m > d.M - 1) m = d.M - 1;
        xp[mt] = (const bf16_t*)d.A + (int64_t)g * d.a_gs + m * d.a_rs;
    }
    // this wavefront's k32 steps
    const int nk = (d.K + 31) >> 5;
    const int per = (nk + SK_WAVES - 1) / SK_WAVES;
    const int s_begin = wave * per;
    int s_end = s_begin + per;
    if (s_end > nk) s_end = nk;
    const int nsteps = s_end > s_begin ? s_end - s_begin : 0;

    // register ring, slots indexed statically; loads unconditional (clamped), zeroed on use past K
    uint4 rw[D], rx[D][MT];
    auto gload = [&](auto SLOT, int s) {
        constexpr int slot = decltype(SLOT)::value;
        int ks = s_begin + s;
        if (ks > nk - 1) ks = nk - 1;                   // steps past the end repeat the last one; never consumed
        int k = ks * 32 + ld_piece * 8;
        if (k > d.K - 8) k = d.K - 8;                   // k groups past K re-read valid data (K is a multiple of 8)
        rw[slot] = *(const uint4*)(wp + k);
        // segmented contraction index of A: a k32 step lies inside one segment (uniform division)
        const int64_t ka = d.a_seg ? (int64_t)((ks * 32) / d.a_seg) * (d.a_seg_stride - d.a_seg) + k : k;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) rx[slot][mt] = *(const uint4*)(xp[mt] + ka);
    };
    auto to_mfma_order = [&](uint4 v) -> uint4 {
        return make_uint4((unsigned)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.x), (unsigned)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.y),
                          (unsigned)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.z), (unsigned)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.w));
    };
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto step = [&](auto U, int s) {
        constexpr int u = decltype(U)::value;
        const bool ok = (s_begin + s) * 32 + kg * 8 < d.K;
        const uint4 w = keep_if(ok, to_mfma_order(rw[u]));
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const uint4 x = to_mfma_order(rx[u][mt]);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const bf16x8*)&w, *(const bf16x8*)&x, acc[mt], 0, 0, 0);
        }
        gload(U, s + D);
    };
    static_for<D>([&](auto U) { gload(U, decltype(U)::value); });
    int s0 = 0;
    for (; s0 + D <= nsteps; s0 += D) static_for<D>([&](auto U) { step(U, s0 + decltype(U)::value); });
    static_for<D - 1>([&](auto U) { if (s0 + decltype(U)::value < nsteps) step(U, s0 + decltype(U)::value); });

    // acc[mt][e]: token mt*16 + l16, column 4*kg + e
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
        *(float4*)&part[wave][mt * 16 + l16][4 * kg] = make_float4(acc[mt][0], acc[mt][1], acc[mt][2], acc[mt][3]);
    __syncthreads();

    // sum the K splits in wavefront order and store: one item = one token x 8 columns
    bf16_t* Cp = (bf16_t*)d.C;
    for (int id = tid; id < MT * 16 * (SK_BN / 8); id += 64 * SK_WAVES) {
        const int row = id / (SK_BN / 8), c8 = (id % (SK_BN / 8)) * 8;
        const int nn = n0 + c8;
        const int64_t mrow = m_base + row;
        if (mrow >= d.M || nn >= d.N) continue;
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = part[0][row][c8 + i];
#pragma unroll
        for (int w = 1; w < SK_WAVES; ++w)
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] += part[w][row][c8 + i];
        if (cvec) {                                     // 8 consecutive (8-aligned) columns are 16 contiguous bytes of C
            const int64_t col = (int64_t)g * d.c_gs + (int64_t)(nn / d.c_div) * d.c_hi + (int64_t)(nn % d.c_div) * d.c_lo;
            *(uint4*)(Cp + mrow * d.c_rs + col) =
                make_uint4(pack2_bf16(v[0], v[1]), pack2_bf16(v[2], v[3]), pack2_bf16(v[4], v[5]), pack2_bf16(v[6], v[7]));
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int ni = nn + i;
                if (ni < d.N) {
                    const int64_t col = (int64_t)g * d.c_gs + (int64_t)(ni / d.c_div) * d.c_hi + (int64_t)(ni % d.c_div) * d.c_lo;
                    Cp[mrow * d.c_rs + col] = float_to_bf16(v[i]);
                }
            }
        }
    }
}

template <int MT, int D>
hipError_t launch_skinny(const GemmDesc& d, int cvec, hipStream_t s) {
    const int tiles_n = (d.N + SK_BN - 1) / SK_BN;
    const unsigned tiles_m = (unsigned)((d.M + MT * 16 - 1) / (MT * 16));
    hipLaunchKernelGGL((gemm_skinny_kernel<MT, D>), dim3((unsigned)(tiles_n * d.G), tiles_m), dim3(64 * SK_WAVES), 0, s, d, tiles_n, cvec);
    return hipGetLastError();
}

}  // namespace

bool skinny_gemm_supported(const GemmDesc& d) {
    return d.M <= 32 && (int64_t)((d.N + SK_BN - 1) / SK_BN) * d.G < (1ll << 31);
}

hipError_t launch_gemm_skinny(const GemmDesc& d, bool cvec, hipStream_t s) {
    if (d.M <= 16) return launch_skinny<1, 8>(d, cvec, s);
    return launch_skinny<2, 8>(d, cvec, s);             // more than 32 tokens: one workgroup per 32-token tile and 16 weight rows
}

bool skinny_gemm_tiled_supported(const GemmDesc& d) {
    return d.M <= 65535ll * 32 && (int64_t)((d.N + SK_BN - 1) / SK_BN) * d.G < (1ll << 31);
}

}  // namespace blr
