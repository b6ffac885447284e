// Monarch (and, with one block, low-rank) layers of small width in ONE kernel: both batched products of
// Section 2.1 "Monarch" with the intermediate kept on chip, the stride permutation and the output order
// folded into the indexing (Section 4, optimisations 1-3).
//
// Why: for the narrow layers of the paper's layer-wise table (ViT-B, GPT2-S, DiT widths at a few hundred
// to a thousand tokens) two GEMM launches are each bound by their launch and pipeline-fill latency and
// lose to the single dense GEMM they replace; one launch that never writes the intermediate wins that
// back. The large layers keep the two GEMMs: there the weights are re-used over 256-token tiles.
//
// A workgroup (4 or 8 wavefronts) owns 32 tokens, one output block k and a range of that block's outputs:
//   phase 0  X[32][n_in] -> LDS (rows past T repeat the last row and are never stored)
//   phase 1  Z'_k[t][l r' + rho] = sum_a X[t][l p + a] R[l][rho b2 + k][a]        -> LDS, bf16
//            (all input blocks l, i.e. everything output block k needs; a workgroup of another output
//             range of the same k computes it again)
//   phase 2  Y[t][o(k, j)] = sum_m Z'_k[t][m] L[k][j][m] for the workgroup's j     -> LDS (over the dead X tile)
//   phase 3  rows of the staged tile -> Y: 16-byte stores when the outputs of the range are contiguous
//            (blocked order, or a single block), element-wise for the interleaved order.
// Both products run on v_mfma_f32_16x16x32_bf16 with the weight rows as FIRST operand, straight from
// global memory (a fragment is one 16-byte load per lane, four lanes per 64 contiguous bytes of a weight
// row, permuted across lanes into the MFMA's order; every fragment serves both 16-token halves), the
// token operand from LDS. Accumulator element e of a lane is output column 4 (lane / 16) + e of token
// lane % 16. Wavefronts split the 16-wide column tiles of each phase and fetch the weights three tiles
// ahead of the MFMAs that use them.
#include "blr_common.h"

namespace blr {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));   // (arrays of HIP's uint4 struct stay in scratch memory)

constexpr int MF_TT = 32;          // tokens per workgroup
constexpr int MF_MAX_WAVES = 8;    // wavefronts per workgroup: 8 when the launch has at most one workgroup per compute unit, else 4
constexpr int MF_KC = 8;           // k32 steps of a tile at most (one register buffer holds a tile's weight fragments)

struct MonarchFusedArgs {
    const bf16_t *X, *R, *L;
    bf16_t* Y;
    int64_t T;
    int n_in, n_out, b1, b2, rp, p, q, w1, w2;   // w1 = r' b2 rows per first-factor block, w2 = b1 r' middle width per output block
    int jsplit, qt;                              // output ranges per block and their length (a multiple of 16)
    int nblk;                                    // workgroups: token tiles * jsplit * b2
    int out_blocked;
    int xstr, zstr, ystr;                        // LDS row strides in bytes
};

// KS1 / KS2: k32 steps of a tile in phase 1 (= p / 32) / phase 2 (= b1 r' / 32). Compile-time, so that every
// fragment of a tile is one load or LDS read with an immediate offset from one address per tile: with run-time
// counts the index arithmetic per fragment, not the memory system, bounded the kernel (1 us per tile).
template <int KS1, int KS2>
__global__ __launch_bounds__(64 * MF_MAX_WAVES) void monarch_fused_kernel(MonarchFusedArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nw = (int)(blockDim.x >> 6);              // 4 or 8
    const int l16 = lane & 15, kg = lane >> 4;
    // Work items in the order (token tile, output range, block k) with k fastest, each XCD on a contiguous
    // range of them: the b2 workgroups that interleave their outputs into the same cache lines then
    // share an L2, where their partial-line writes merge (on different XCDs every partial line goes to
    // memory on its own: +2 us measured with a 2-D grid of token tiles x blocks at 25 token tiles, which
    // deals the blocks of one token tile to different XCDs).
    const int lg = xcd_contiguous(blockIdx.x, a.nblk);
    const int k = lg % a.b2;
    const int j0 = ((lg / a.b2) % a.jsplit) * a.qt;
    const int64_t t0 = (int64_t)(lg / (a.b2 * a.jsplit)) * MF_TT;
    const int nj = a.q - j0 < a.qt ? a.q - j0 : a.qt;   // outputs of this range that exist (> 0 by the launcher's choice of qt)
    const int xy = a.xstr > a.ystr ? a.xstr : a.ystr;
    unsigned char* Xs = smem;                           // [32][xstr]; later the staged output tile [32][ystr]
    unsigned char* Zs = smem + MF_TT * xy;              // [32][zstr]

    // ---- phase 0: a wavefront moves whole token rows, all eight of its rows at once (all loads, then all
    // LDS writes), so that the tile costs one memory latency. Rows past T repeat the last row. Offsets
    // from the tile's first row are 32-bit (the launcher checks 32 n_in elements).
    auto load_x_tile = [&]() {
        const int pieces = a.n_in >> 3;                 // 16-byte pieces per row
        const unsigned char* xt = (const unsigned char*)(a.X + t0 * a.n_in);
        const int last = a.T - t0 > MF_TT ? MF_TT - 1 : (int)(a.T - t0) - 1;
#pragma unroll 1
        for (int c0 = 0; c0 < pieces; c0 += 128) {
            u32x4 v[MF_TT / 4][2];                      // rows wave, wave + nw, ...: 8 of them with 4 wavefronts, 4 with 8
#pragma unroll
            for (int i = 0; i < MF_TT / 4; ++i) {
                if (nw * i >= MF_TT) break;             // uniform
                int row = wave + nw * i;
                if (row > last) row = last;
                const unsigned roff = (unsigned)(row * a.n_in) * 2u;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    int c = c0 + h * 64 + lane;
                    if (c > pieces - 1) c = pieces - 1;
                    v[i][h] = *(const u32x4*)(xt + (roff + (unsigned)c * 16u));
                }
            }
#pragma unroll
            for (int i = 0; i < MF_TT / 4; ++i)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int c = c0 + h * 64 + lane;
                    if (c < pieces && wave + nw * i < MF_TT) *(u32x4*)(Xs + (wave + nw * i) * a.xstr + c * 16) = v[i][h];
                }
        }
    };

    // ---- phases 1 and 2 as ONE stream of weight tiles per wavefront. A tile is 16 weight rows (16 middle
    // columns of Z'_k, then 16 outputs of the range) over its whole contraction index; a wavefront takes
    // a contiguous share of the tiles of either phase. The weights depend on nothing, so their loads run
    // three tiles ahead of the MFMAs, across the barrier that separates the phases (four register
    // buffers in rotation): the kernel is a stream of the factors through the CU.
    const int n1 = a.w2 >> 4, n2 = (nj + 15) >> 4;
    const int ch1 = (n1 + nw - 1) / nw, ch2 = (n2 + nw - 1) / nw;
    const int s1 = wave * ch1, s2 = wave * ch2;
    const int c1 = n1 - s1 < ch1 ? (n1 - s1 > 0 ? n1 - s1 : 0) : ch1;    // this wavefront's tiles of phase 1 / phase 2
    const int c2 = n2 - s2 < ch2 ? (n2 - s2 > 0 ? n2 - s2 : 0) : ch2;
    const int ntl = c1 + c2;
    // A weight fragment is LOADED with four neighbouring lanes on the 64 contiguous bytes of one row
    // (lane = 4 row + piece: 16 requests of 64 bytes per instruction) and then moved to the MFMA's order
    // (lane = 16 piece + row) by a cross-lane permute. Loading in the MFMA's order directly makes every
    // lane its own 16-byte request.
    const int ld_row = lane >> 2, ld_piece = lane & 3;
    const int from_lane = (l16 * 4 + kg) * 4;           // byte index of the lane that loaded this lane's piece
    // Middle column m = l r' + rho of output block k is row m b2 + k of the first factor seen as one
    // matrix of rows of p (row (l, rho b2 + k) of R[b1][r' b2][p]): no division by r' is needed.
    const unsigned char* Rk = (const unsigned char*)(a.R + (int64_t)k * a.p);
    const unsigned char* Lk = (const unsigned char*)(a.L + (int64_t)k * a.q * a.w2);
    auto fetch = [&](bf16x8 (&w)[MF_KC], int i) {
        if (i >= ntl) return;                           // uniform
        if (i < c1) {
            const unsigned off = ((unsigned)((s1 + i) * 16 + ld_row) * (unsigned)(a.b2 * a.p) + ld_piece * 8u) * 2u;
#pragma unroll
            for (int u = 0; u < KS1; ++u) w[u] = *(const bf16x8*)(Rk + off + u * 64);
        } else {
            int j = j0 + (s2 + i - c1) * 16 + ld_row;
            if (j > a.q - 1) j = a.q - 1;               // rows past the block repeat its last row and are never stored
            const unsigned off = ((unsigned)j * (unsigned)a.w2 + ld_piece * 8u) * 2u;
#pragma unroll
            for (int u = 0; u < KS2; ++u) w[u] = *(const bf16x8*)(Lk + off + u * 64);
        }
    };
    auto to_mfma_order = [&](bf16x8 v) -> bf16x8 {
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        i32x4 x = __builtin_bit_cast(i32x4, v), y;
#pragma unroll
        for (int d = 0; d < 4; ++d) y[d] = __builtin_amdgcn_ds_bpermute(from_lane, x[d]);
        return __builtin_bit_cast(bf16x8, y);
    };
    // one tile: all token fragments are read before the MFMAs (one LDS latency per tile); accumulator
    // element e is token l16 (+16 in the second accumulator), column 4 kg + e of the tile
    auto tile = [&](auto KS, const bf16x8 (&w)[MF_KC], const unsigned char* tok, int half, unsigned char* out, int ohalf) {
        constexpr int ks = decltype(KS)::value;
        bf16x8 x0[ks], x1[ks];
#pragma unroll
        for (int u = 0; u < ks; ++u) {
            x0[u] = *(const bf16x8*)(tok + u * 64);
            x1[u] = *(const bf16x8*)(tok + half + u * 64);
        }
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < ks; ++u) {
            const bf16x8 wf = to_mfma_order(w[u]);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, x0[u], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, x1[u], acc1, 0, 0, 0);
        }
        *(uint2*)out = make_uint2(pack2_bf16(acc0[0], acc0[1]), pack2_bf16(acc0[2], acc0[3]));
        *(uint2*)(out + ohalf) = make_uint2(pack2_bf16(acc1[0], acc1[1]), pack2_bf16(acc1[2], acc1[3]));
    };
    // input block and position inside it of the next phase-1 tile's first middle column (tiles are consumed in order)
    int cl = (s1 * 16) / a.rp, crho = (s1 * 16) % a.rp;
    auto consume = [&](const bf16x8 (&w)[MF_KC], int i) {
        if (i >= ntl) return;                           // uniform
        if (i == c1) __syncthreads();                   // Z'_k is complete (every wavefront passes here once, or below)
        if (i < c1) {
            const int m0 = (s1 + i) * 16;
            tile(std::integral_constant<int, KS1>{}, w, Xs + l16 * a.xstr + (cl * a.p + kg * 8) * 2, 16 * a.xstr,
                 Zs + l16 * a.zstr + (m0 + 4 * kg) * 2, 16 * a.zstr);
            crho += 16;
            if (crho == a.rp) { crho = 0; ++cl; }
        } else {
            tile(std::integral_constant<int, KS2>{}, w, Zs + l16 * a.zstr + kg * 16, 16 * a.zstr,
                 Xs + l16 * a.ystr + ((s2 + i - c1) * 16 + 4 * kg) * 2, 16 * a.ystr);
        }
    };
    {
        bf16x8 b0[MF_KC], b1[MF_KC], b2[MF_KC], b3[MF_KC];
        fetch(b0, 0); fetch(b1, 1); fetch(b2, 2);       // the weights depend on nothing: requested ahead of the X tile
        load_x_tile();
        __syncthreads();                                // the X tile is in LDS
#pragma unroll 1
        for (int i = 0; i < ntl; i += 4) {
            fetch(b3, i + 3); consume(b0, i);
            fetch(b0, i + 4); consume(b1, i + 1);
            fetch(b1, i + 5); consume(b2, i + 2);
            fetch(b2, i + 6); consume(b3, i + 3);
        }
        if (c2 == 0) __syncthreads();                   // a wavefront without tiles in phase 2 has not met the others yet
    }
    __syncthreads();

    // ---- phase 3: a wavefront writes whole token rows
    const bool contiguous = a.out_blocked || a.b2 == 1;
    const int64_t col0 = contiguous ? (int64_t)k * a.q + j0 : (int64_t)j0 * a.b2 + k;
    if (contiguous && (nj & 7) == 0 && (col0 & 7) == 0 && (a.n_out & 7) == 0) {
        const int pieces = nj >> 3;
        for (int row = wave; row < MF_TT; row += nw) {
            const int64_t t = t0 + row;
            if (t >= a.T) break;                        // uniform
            for (int c = lane; c < pieces; c += 64)
                *(u32x4*)(a.Y + t * a.n_out + col0 + c * 8) = *(const u32x4*)(Xs + row * a.ystr + c * 16);
        }
    } else {
        const int cstep = contiguous ? 1 : a.b2;
        for (int row = wave; row < MF_TT; row += nw) {
            const int64_t t = t0 + row;
            if (t >= a.T) break;                        // uniform
            for (int c = lane; c < nj; c += 64)
                a.Y[t * a.n_out + col0 + (int64_t)c * cstep] = *(const bf16_t*)(Xs + row * a.ystr + c * 2);
        }
    }
}

// output ranges per block: as many as still give at most one workgroup per compute unit (a few more
// workgroups than compute units cost a second round: 300 workgroups were measured 50 % slower than
// 200), each range a multiple of 16 outputs
inline void choose_ranges(int64_t T, int b2, int q, int& jsplit, int& qt) {
    const int64_t base = ((T + MF_TT - 1) / MF_TT) * b2;
    const int tiles = (q + 15) / 16;
    int s = base >= 256 ? 1 : (int)(256 / base);
    if (s > 8) s = 8;
    if (s > tiles) s = tiles;
    qt = ((tiles + s - 1) / s) * 16;
    jsplit = (q + qt - 1) / qt;
}

inline int lds_bytes(int n_in, int w2, int qt) {
    const int xstr = n_in * 2 + 16, zstr = w2 * 2 + 16, ystr = qt * 2 + 16;
    return MF_TT * (xstr > ystr ? xstr : ystr) + MF_TT * zstr;
}

template <int KS1, int KS2>
hipError_t launch_inst(const MonarchFusedArgs& a, dim3 grid, int lds, hipStream_t s) {
    static LdsLimitOnce lds_limit;
    if (hipError_t e = lds_limit.set({(const void*)monarch_fused_kernel<KS1, KS2>}, 160 * 1024); e != hipSuccess) return e;
    // one workgroup per compute unit at most: twice the wavefronts, i.e. twice the weight bytes in flight per compute unit
    const unsigned waves = (uint64_t)grid.x * grid.y <= 256 ? MF_MAX_WAVES : MF_MAX_WAVES / 2;
    hipLaunchKernelGGL((monarch_fused_kernel<KS1, KS2>), grid, dim3(64 * waves), lds, s, a);
    return hipGetLastError();
}

template <int KS1>
hipError_t launch_ks2(const MonarchFusedArgs& a, dim3 grid, int lds, hipStream_t s) {
    switch (a.w2 >> 5) {
        case 1: return launch_inst<KS1, 1>(a, grid, lds, s);
        case 2: return launch_inst<KS1, 2>(a, grid, lds, s);
        case 3: return launch_inst<KS1, 3>(a, grid, lds, s);
        case 4: return launch_inst<KS1, 4>(a, grid, lds, s);
        case 5: return launch_inst<KS1, 5>(a, grid, lds, s);
        case 6: return launch_inst<KS1, 6>(a, grid, lds, s);
        case 7: return launch_inst<KS1, 7>(a, grid, lds, s);
        case 8: return launch_inst<KS1, 8>(a, grid, lds, s);
    }
    return hipErrorInvalidValue;
}

inline hipError_t launch_ks1(const MonarchFusedArgs& a, dim3 grid, int lds, hipStream_t s) {
    switch (a.p >> 5) {
        case 1: return launch_ks2<1>(a, grid, lds, s);
        case 2: return launch_ks2<2>(a, grid, lds, s);
        case 3: return launch_ks2<3>(a, grid, lds, s);
        case 4: return launch_ks2<4>(a, grid, lds, s);
        case 5: return launch_ks2<5>(a, grid, lds, s);
        case 6: return launch_ks2<6>(a, grid, lds, s);
        case 7: return launch_ks2<7>(a, grid, lds, s);
        case 8: return launch_ks2<8>(a, grid, lds, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

bool monarch_fused_supported(int64_t T, int n_in, int n_out, int b1, int b2, int rp) {
    if (T <= 0 || b1 <= 0 || b2 <= 0 || rp <= 0 || n_in % b1 || n_out % b2) return false;
    const int p = n_in / b1, q = n_out / b2;
    const int64_t w2 = (int64_t)b1 * rp;
    if (rp % 16 || p % 32 || w2 % 32 || p > 32 * MF_KC || w2 > 32 * MF_KC || n_in > 8192 || n_out > (1 << 22)) return false;   // a tile's contraction index fits one register buffer
    if ((T + MF_TT - 1) / MF_TT * b2 * 8 >= (1ll << 31)) return false;     // workgroups (at most 8 output ranges per block)
    if (w2 * b2 * p >= (1ll << 30)) return false;                           // byte offsets into the first factor are 32-bit
    int jsplit, qt;
    choose_ranges(T, b2, q, jsplit, qt);
    return lds_bytes(n_in, (int)w2, qt) <= 160 * 1024;
}

int monarch_fused_lds_bytes(int64_t T, int n_in, int n_out, int b1, int b2, int rp) {
    int jsplit, qt;
    choose_ranges(T, b2, n_out / b2, jsplit, qt);
    return lds_bytes(n_in, b1 * rp, qt);
}

hipError_t launch_monarch_fused(const void* X, const void* R, const void* L, void* Y, int64_t T, int n_in, int n_out,
                                int b1, int b2, int rp, bool out_blocked, hipStream_t s) {
    MonarchFusedArgs a{};
    a.X = (const bf16_t*)X; a.R = (const bf16_t*)R; a.L = (const bf16_t*)L; a.Y = (bf16_t*)Y;
    a.T = T; a.n_in = n_in; a.n_out = n_out; a.b1 = b1; a.b2 = b2; a.rp = rp;
    a.p = n_in / b1; a.q = n_out / b2; a.w1 = rp * b2; a.w2 = b1 * rp;
    choose_ranges(T, b2, a.q, a.jsplit, a.qt);
    a.out_blocked = out_blocked ? 1 : 0;
    a.xstr = n_in * 2 + 16; a.zstr = a.w2 * 2 + 16; a.ystr = a.qt * 2 + 16;
    const int lds = lds_bytes(n_in, a.w2, a.qt);
    a.nblk = (int)((T + MF_TT - 1) / MF_TT) * b2 * a.jsplit;
    dim3 grid((unsigned)a.nblk);
    return launch_ks1(a, grid, lds, s);
}

}  // namespace blr
