// BLAST layers of small width and FEW, WIDE blocks (the b = 3, 6, 9 rows of the paper's layer-wise table) in ONE
// kernel: stage 1, the coupling and stage 3 of Section 2.1 "BLAST" with both intermediates kept on chip.
//
// Why: at a few hundred to a thousand tokens the three launches of the multi-kernel execution are each bound by
// launch and pipeline-fill latency and together lose to the single dense GEMM they replace. The whole-layer kernel
// for many narrow blocks (blast_fused.hip) wants p <= 64; here the blocks are wide and few, so the roles turn
// around: a workgroup owns 32 tokens, ONE output block i and a range of that block's outputs, and because it
// serves a single i the coupling needs no storage at all:
//     A_i[t][rho] = sum_j s_ij[rho] (X_j V_j)[t][rho]
// is accumulated in registers, one input block after the other, each block's fp32 product scaled per column by
// s_ij and added. (Z is therefore never rounded here; the multi-kernel executions round it to bf16 first.)
//   phase 0  X[32][n_in] -> LDS (rows past T repeat the last row and are never stored)
//   phase 1  A_i[t][rho] for all rho                                              -> LDS, bf16
//            (all of V streams through every workgroup; workgroups of other (i, range) compute their own A_i)
//   phase 2  Y[t][i p + a] = sum_rho A_i[t][rho] U[i][a][rho] for the workgroup's a -> LDS (over the dead X tile)
//   phase 3  rows of the staged tile -> Y
// Both products run on v_mfma_f32_16x16x32_bf16 with the weight rows as FIRST operand, straight from global
// memory (a fragment is one 16-byte load per lane, four lanes per 64 contiguous bytes of a weight row, permuted
// across lanes into the MFMA's order; every fragment serves both 16-token halves), the token operand from LDS.
// Accumulator element e of a lane is column 4 (lane / 16) + e of token lane % 16. Wavefronts split the 16-wide
// column tiles of each phase and fetch the weights three items ahead of the MFMAs that use them, across the
// barrier between the phases.
// Operands: Vt[b][r][q] (the transposed first factor of the packed buffer: contraction index contiguous),
// S[b][b][r] as S[i][j][rho], U[b][p][r].
#include "blr_common.h"

namespace blr {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int BN_TT = 32;          // tokens per workgroup
constexpr int BN_WAVES = 8;        // wavefronts per workgroup at most (4 when the launch has more workgroups than compute units)
constexpr int BN_KC = 8;           // k32 steps of an item at most (one register buffer holds an item's weight fragments)

struct BlastNarrowArgs {
    const bf16_t *X, *Vt, *S, *U;
    bf16_t* Y;
    int64_t T;
    int n_in, n_out, b, r, q, p;
    int jsplit, pt;                // output ranges per block and their length (a multiple of 16)
    int nblk;                      // workgroups: token tiles * jsplit * b
    int xstr, astr, ystr;          // LDS row strides in bytes
};

// KS1 / KS3: k32 steps of an item in phase 1 (= q / 32) / phase 2 (= r / 32). Compile-time, so that every fragment
// of an item is one load or LDS read with an immediate offset from one address per item.
template <int KS1, int KS3>
__global__ __launch_bounds__(64 * BN_WAVES) void blast_narrow_kernel(BlastNarrowArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nw = (int)(blockDim.x >> 6);              // 4 or 8
    const int l16 = lane & 15, kg = lane >> 4;
    // work items in the order (token tile, output range, block i) with i fastest, each XCD on a contiguous range:
    // the workgroups that share a token tile (and stream the same V) sit on one XCD's L2
    const int lg = xcd_contiguous(blockIdx.x, a.nblk);
    const int i = lg % a.b;
    const int a0 = ((lg / a.b) % a.jsplit) * a.pt;
    const int64_t t0 = (int64_t)(lg / (a.b * a.jsplit)) * BN_TT;
    const int na = a.p - a0 < a.pt ? a.p - a0 : a.pt;   // outputs of this range that exist (> 0 by the launcher's choice of pt)
    const int xy = a.xstr > a.ystr ? a.xstr : a.ystr;
    unsigned char* Xs = smem;                           // [32][xstr]; later the staged output tile [32][ystr]
    unsigned char* As = smem + BN_TT * xy;              // [32][astr]

    // ---- phase 0: a wavefront moves whole token rows, all of its rows at once (all loads, then all LDS writes)
    auto load_x_tile = [&]() {
        const int pieces = a.n_in >> 3;                 // 16-byte pieces per row
        const unsigned char* xt = (const unsigned char*)(a.X + t0 * a.n_in);
        const int last = a.T - t0 > BN_TT ? BN_TT - 1 : (int)(a.T - t0) - 1;
#pragma unroll 1
        for (int c0 = 0; c0 < pieces; c0 += 128) {
            u32x4 v[BN_TT / 4][2];                      // rows wave, wave + nw, ...: 8 of them with 4 wavefronts, 4 with 8
#pragma unroll
            for (int h8 = 0; h8 < BN_TT / 4; ++h8) {
                if (nw * h8 >= BN_TT) break;            // uniform
                int row = wave + nw * h8;
                if (row > last) row = last;
                const unsigned roff = (unsigned)(row * a.n_in) * 2u;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    int c = c0 + h * 64 + lane;
                    if (c > pieces - 1) c = pieces - 1;
                    v[h8][h] = *(const u32x4*)(xt + (roff + (unsigned)c * 16u));
                }
            }
#pragma unroll
            for (int h8 = 0; h8 < BN_TT / 4; ++h8)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int c = c0 + h * 64 + lane;
                    if (c < pieces && wave + nw * h8 < BN_TT) *(u32x4*)(Xs + (wave + nw * h8) * a.xstr + c * 16) = v[h8][h];
                }
        }
    };

    // ---- phases 1 and 2 as ONE stream of items per wavefront. Phase 1: a wavefront takes a contiguous share of
    // the 16-wide rank tiles; an item is (rank tile, input block j), j fastest: 16 rows of Vt[j] over all of q,
    // plus the four coupling values s_ij of this lane's columns. Phase 2: an item is 16 rows of U[i] over all of r.
    const int n1 = a.r >> 4, n2 = (na + 15) >> 4;
    const int ch1 = (n1 + nw - 1) / nw, ch2 = (n2 + nw - 1) / nw;
    const int s1 = wave * ch1, s2 = wave * ch2;
    const int c1t = n1 - s1 < ch1 ? (n1 - s1 > 0 ? n1 - s1 : 0) : ch1;   // this wavefront's rank tiles
    const int c1 = c1t * a.b;                                           // ... and items of phase 1
    const int c2 = n2 - s2 < ch2 ? (n2 - s2 > 0 ? n2 - s2 : 0) : ch2;
    const int nit = c1 + c2;
    const int ld_row = lane >> 2, ld_piece = lane & 3;  // a fragment is loaded with four lanes on one row's 64 contiguous bytes
    const int from_lane = (l16 * 4 + kg) * 4;           // byte index of the lane that loaded this lane's piece
    const unsigned char* Vb = (const unsigned char*)a.Vt;
    const unsigned char* Ui = (const unsigned char*)(a.U + (int64_t)i * a.p * a.r);
    const unsigned char* Si = (const unsigned char*)(a.S + (int64_t)i * a.b * a.r);
    // fetch cursor of phase 1 (items are fetched in order): rank tile and input block of the next item
    int ft = s1, fj = 0;
    auto fetch = [&](bf16x8 (&w)[BN_KC], uint2& sv, int it) {
        if (it >= nit) return;                          // uniform
        if (it < c1) {
            // row (fj, 16 ft + ld_row) of Vt; byte offsets are 32-bit (the launcher checks n_in r elements)
            const unsigned off = ((unsigned)(fj * a.r + ft * 16 + ld_row) * (unsigned)a.q + ld_piece * 8u) * 2u;
#pragma unroll
            for (int u = 0; u < KS1; ++u) w[u] = *(const bf16x8*)(Vb + off + u * 64);
            sv = *(const uint2*)(Si + ((unsigned)(fj * a.r + ft * 16 + 4 * kg)) * 2u);   // s_ij of columns 4 kg .. 4 kg + 3
            if (++fj == a.b) { fj = 0; ++ft; }
        } else {
            int row = a0 + (s2 + it - c1) * 16 + ld_row;
            if (row > a.p - 1) row = a.p - 1;           // rows past the block repeat its last row and are never stored
            const unsigned off = ((unsigned)row * (unsigned)a.r + ld_piece * 8u) * 2u;
#pragma unroll
            for (int u = 0; u < KS3; ++u) w[u] = *(const bf16x8*)(Ui + off + u * 64);
        }
    };
    auto to_mfma_order = [&](bf16x8 v) -> bf16x8 {
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        i32x4 x = __builtin_bit_cast(i32x4, v), y;
#pragma unroll
        for (int d = 0; d < 4; ++d) y[d] = __builtin_amdgcn_ds_bpermute(from_lane, x[d]);
        return __builtin_bit_cast(bf16x8, y);
    };
    // one item's product: all token fragments are read before the MFMAs (one LDS latency per item)
    auto product = [&](auto KS, const bf16x8 (&w)[BN_KC], const unsigned char* tok, int half, f32x4& acc0, f32x4& acc1) {
        constexpr int ks = decltype(KS)::value;
        bf16x8 x0[ks], x1[ks];
#pragma unroll
        for (int u = 0; u < ks; ++u) {
            x0[u] = *(const bf16x8*)(tok + u * 64);
            x1[u] = *(const bf16x8*)(tok + half + u * 64);
        }
#pragma unroll
        for (int u = 0; u < ks; ++u) {
            const bf16x8 wf = to_mfma_order(w[u]);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, x0[u], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, x1[u], acc1, 0, 0, 0);
        }
    };
    // consume cursor of phase 1 and the running A_i of the current rank tile (tokens l16 and 16 + l16)
    int ct = s1, cj = 0;
    f32x4 A0 = {0.f, 0.f, 0.f, 0.f}, A1 = {0.f, 0.f, 0.f, 0.f};
    auto consume = [&](const bf16x8 (&w)[BN_KC], const uint2& sv, int it) {
        if (it >= nit) return;                          // uniform
        if (it == c1) __syncthreads();                  // A_i is complete (every wavefront passes here once, or below)
        if (it < c1) {
            f32x4 z0 = {0.f, 0.f, 0.f, 0.f}, z1 = {0.f, 0.f, 0.f, 0.f};
            product(std::integral_constant<int, KS1>{}, w, Xs + l16 * a.xstr + (cj * a.q + kg * 8) * 2, 16 * a.xstr, z0, z1);
            const float s[4] = {__uint_as_float(sv.x << 16), __uint_as_float(sv.x & 0xFFFF0000u),
                                __uint_as_float(sv.y << 16), __uint_as_float(sv.y & 0xFFFF0000u)};
#pragma unroll
            for (int e = 0; e < 4; ++e) { A0[e] = fmaf(s[e], z0[e], A0[e]); A1[e] = fmaf(s[e], z1[e], A1[e]); }
            if (++cj == a.b) {                          // the rank tile is complete: to LDS as bf16
                unsigned char* out = As + l16 * a.astr + (ct * 16 + 4 * kg) * 2;
                *(uint2*)out = make_uint2(pack2_bf16(A0[0], A0[1]), pack2_bf16(A0[2], A0[3]));
                *(uint2*)(out + 16 * a.astr) = make_uint2(pack2_bf16(A1[0], A1[1]), pack2_bf16(A1[2], A1[3]));
                A0 = f32x4{0.f, 0.f, 0.f, 0.f}; A1 = f32x4{0.f, 0.f, 0.f, 0.f};
                cj = 0; ++ct;
            }
        } else {
            f32x4 y0 = {0.f, 0.f, 0.f, 0.f}, y1 = {0.f, 0.f, 0.f, 0.f};
            product(std::integral_constant<int, KS3>{}, w, As + l16 * a.astr + kg * 16, 16 * a.astr, y0, y1);
            unsigned char* out = Xs + l16 * a.ystr + ((s2 + it - c1) * 16 + 4 * kg) * 2;
            *(uint2*)out = make_uint2(pack2_bf16(y0[0], y0[1]), pack2_bf16(y0[2], y0[3]));
            *(uint2*)(out + 16 * a.ystr) = make_uint2(pack2_bf16(y1[0], y1[1]), pack2_bf16(y1[2], y1[3]));
        }
    };
    {
        bf16x8 b0[BN_KC], b1[BN_KC], b2[BN_KC], b3[BN_KC];
        uint2 v0 = {0u, 0u}, v1 = {0u, 0u}, v2 = {0u, 0u}, v3 = {0u, 0u};
        fetch(b0, v0, 0); fetch(b1, v1, 1); fetch(b2, v2, 2);   // the weights depend on nothing: requested ahead of the X tile
        load_x_tile();
        __syncthreads();                                // the X tile is in LDS
        // the staged output tile overwrites the X tile: phase 2 may only start once EVERY wavefront is done with X,
        // which the barrier at it == c1 guarantees (each wavefront reaches it after its last phase-1 item)
#pragma unroll 1
        for (int it = 0; it < nit; it += 4) {
            fetch(b3, v3, it + 3); consume(b0, v0, it);
            fetch(b0, v0, it + 4); consume(b1, v1, it + 1);
            fetch(b1, v1, it + 5); consume(b2, v2, it + 2);
            fetch(b2, v2, it + 6); consume(b3, v3, it + 3);
        }
        if (c2 == 0) __syncthreads();                   // a wavefront without items in phase 2 has not met the others yet
    }
    __syncthreads();

    // ---- phase 3: a wavefront writes whole token rows; the range's outputs are contiguous in Y
    const int64_t col0 = (int64_t)i * a.p + a0;
    if ((na & 7) == 0 && (col0 & 7) == 0 && (a.n_out & 7) == 0) {
        const int pieces = na >> 3;
        for (int row = wave; row < BN_TT; row += nw) {
            const int64_t t = t0 + row;
            if (t >= a.T) break;                        // uniform
            for (int c = lane; c < pieces; c += 64)
                *(u32x4*)(a.Y + t * a.n_out + col0 + c * 8) = *(const u32x4*)(Xs + row * a.ystr + c * 16);
        }
    } else {
        for (int row = wave; row < BN_TT; row += nw) {
            const int64_t t = t0 + row;
            if (t >= a.T) break;                        // uniform
            for (int c = lane; c < na; c += 64)
                a.Y[t * a.n_out + col0 + c] = *(const bf16_t*)(Xs + row * a.ystr + c * 2);
        }
    }
}

// output ranges per block: as many as still give at most one workgroup per compute unit, at most 8, each a
// multiple of 16 outputs (every further range streams all of V once more)
inline void choose_ranges(int64_t T, int b, int p, int& jsplit, int& pt) {
    const int64_t base = ((T + BN_TT - 1) / BN_TT) * b;
    const int tiles = (p + 15) / 16;
    int s = base >= 256 ? 1 : (int)(256 / base);
    if (s > 8) s = 8;
    if (s > tiles) s = tiles;
    pt = ((tiles + s - 1) / s) * 16;
    jsplit = (p + pt - 1) / pt;
}

inline int lds_bytes(int n_in, int r, int pt) {
    const int xstr = n_in * 2 + 16, astr = r * 2 + 16, ystr = pt * 2 + 16;
    return BN_TT * (xstr > ystr ? xstr : ystr) + BN_TT * astr;
}

template <int KS1, int KS3>
hipError_t launch_inst(const BlastNarrowArgs& a, int lds, hipStream_t s) {
    static LdsLimitOnce lds_limit;
    if (hipError_t e = lds_limit.set({(const void*)blast_narrow_kernel<KS1, KS3>}, 160 * 1024); e != hipSuccess) return e;
    // one workgroup per compute unit at most: twice the wavefronts, i.e. twice the weight bytes in flight per compute unit
    const unsigned waves = a.nblk <= 256 ? BN_WAVES : BN_WAVES / 2;
    hipLaunchKernelGGL((blast_narrow_kernel<KS1, KS3>), dim3((unsigned)a.nblk), dim3(64 * waves), lds, s, a);
    return hipGetLastError();
}

template <int KS1>
hipError_t launch_ks3(const BlastNarrowArgs& a, int lds, hipStream_t s) {
    switch (a.r >> 5) {
        case 1: return launch_inst<KS1, 1>(a, lds, s);
        case 2: return launch_inst<KS1, 2>(a, lds, s);
        case 3: return launch_inst<KS1, 3>(a, lds, s);
        case 4: return launch_inst<KS1, 4>(a, lds, s);
        case 5: return launch_inst<KS1, 5>(a, lds, s);
        case 6: return launch_inst<KS1, 6>(a, lds, s);
        case 7: return launch_inst<KS1, 7>(a, lds, s);
        case 8: return launch_inst<KS1, 8>(a, lds, s);
    }
    return hipErrorInvalidValue;
}

inline hipError_t launch_ks1(const BlastNarrowArgs& a, int lds, hipStream_t s) {
    switch (a.q >> 5) {
        case 1: return launch_ks3<1>(a, lds, s);
        case 2: return launch_ks3<2>(a, lds, s);
        case 3: return launch_ks3<3>(a, lds, s);
        case 4: return launch_ks3<4>(a, lds, s);
        case 5: return launch_ks3<5>(a, lds, s);
        case 6: return launch_ks3<6>(a, lds, s);
        case 7: return launch_ks3<7>(a, lds, s);
        case 8: return launch_ks3<8>(a, lds, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

bool blast_narrow_supported(int64_t T, int n_in, int n_out, int b, int r) {
    if (T <= 0 || b <= 0 || r <= 0 || n_in <= 0 || n_out <= 0 || n_in % b || n_out % b) return false;
    const int q = n_in / b, p = n_out / b;
    if (q % 32 || r % 32 || q > 32 * BN_KC || r > 32 * BN_KC || n_in > 8192 || n_out > (1 << 22) || b > 64) return false;   // an item's contraction index fits one register buffer
    if ((T + BN_TT - 1) / BN_TT * b * 8 >= (1ll << 31)) return false;      // workgroups (at most 8 output ranges per block)
    if ((int64_t)n_in * r >= (1ll << 30) || (int64_t)p * r >= (1ll << 30) || (int64_t)b * r >= (1ll << 30)) return false;   // 32-bit byte offsets into Vt, U[i], S[i]
    int jsplit, pt;
    choose_ranges(T, b, p, jsplit, pt);
    return lds_bytes(n_in, r, pt) <= 160 * 1024;
}

int64_t blast_narrow_workgroups(int64_t T, int n_out, int b) {
    int jsplit, pt;
    choose_ranges(T, b, n_out / b, jsplit, pt);
    return ((T + BN_TT - 1) / BN_TT) * b * jsplit;
}

int blast_narrow_lds_bytes(int64_t T, int n_in, int n_out, int b, int r) {
    int jsplit, pt;
    choose_ranges(T, b, n_out / b, jsplit, pt);
    return lds_bytes(n_in, r, pt);
}

hipError_t launch_blast_narrow(const void* X, const void* Vt, const void* S, const void* U, void* Y,
                               int64_t T, int n_in, int n_out, int b, int r, hipStream_t s) {
    BlastNarrowArgs a{};
    a.X = (const bf16_t*)X; a.Vt = (const bf16_t*)Vt; a.S = (const bf16_t*)S; a.U = (const bf16_t*)U; a.Y = (bf16_t*)Y;
    a.T = T; a.n_in = n_in; a.n_out = n_out; a.b = b; a.r = r; a.q = n_in / b; a.p = n_out / b;
    choose_ranges(T, b, a.p, a.jsplit, a.pt);
    a.xstr = n_in * 2 + 16; a.astr = r * 2 + 16; a.ystr = a.pt * 2 + 16;
    const int lds = lds_bytes(n_in, r, a.pt);
    a.nblk = (int)((T + BN_TT - 1) / BN_TT) * b * a.jsplit;
    return launch_ks1(a, lds, s);
}

}  // namespace blr
