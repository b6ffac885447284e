// BLAST stage 1 + coupling fused in one kernel (bf16 MFMA, gfx950).
//
// A workgroup owns a tile of 128 tokens x 64 rank indices. It loops over the input blocks j inside
// the workgroup (the reduction over j cannot be split across workgroups): for each j the tile
// Z_j = X_j V_j is a small GEMM on v_mfma_f32_32x32x16_bf16 whose operands stream from global memory
// straight into LDS (global_load_lds, no staging registers), and whose result is rounded to bf16 and
// kept in registers. When all j are done the tile goes through LDS as Zs[rho][t][j], 64 tokens at a
// time, and the coupling A[t][i][rho] = sum_j S[i][j][rho] Z[t][j][rho] is, for every rho, a
// (tokens x 16) . (16 x 16) product: one v_mfma_f32_16x16x16_bf16 per 16 tokens, with the per-rho
// 16x16 tile of S read from the packed tensor Sp[rho][i][j].
// Z never leaves the chip and the coupling runs on the matrix cores; only A goes to HBM.
#include "blr_common.h"

namespace blr {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));   // (arrays of HIP's uint4 struct stay in scratch memory)

constexpr int TN = 64, TR = 64;              // the coupling works on 64 tokens x 64 rank indices at a time
constexpr int ZSTR = TN * 32 + 8;            // bytes of one rho row of Zs: TN tokens x 16 j x 2 B, + 8 B pad
constexpr int ZS_BYTES = TR * ZSTR;
static_assert(ZS_BYTES % 16 == 0, "Zs is cleared with 16-byte stores");

// stage 1 of the fused kernel: TT tokens x 64 ranks per workgroup, 8 wavefronts; TT = 128: every wavefront
// computes a 32 x 32 part of the tile; TT = 64 (calls with too few 128-token tiles to fill the chip):
// wavefronts 0..3 compute, all 8 move the operands and take part in the coupling.
// BK contraction indices per step (one barrier per step): 128 where the input blocks are whole numbers of
// such chunks, 64 otherwise; 3 (128 tokens, 48 KB per stage) to 8 stages in LDS.
template <int TT, int BK>
struct StCfg {
    static constexpr int RB = BK * 2;             // bytes of an operand row in a stage
    static constexpr int PPR = RB / 16;           // 16-byte pieces per row
    static constexpr int RPL = 1024 / RB;         // rows one direct load (64 lanes x 16 bytes) fills
    static constexpr int SH = BK == 128 ? 0 : 1;  // swizzle: slot = piece ^ ((row >> SH) & (PPR - 1))
    static constexpr int KS = BK / 16;            // k16 steps per stage
    static constexpr int ROWS = TT + TR;          // operand rows of one stage: X rows, then Vt rows
    static constexpr int STAGE = ROWS * RB;
    // stages in LDS: as many as 144 KB hold, 8 at most (a workgroup is alone on its compute unit, and with
    // few tokens its steps are as long as a load takes to arrive divided by the steps in flight)
    static constexpr int NS = 147456 / STAGE > 8 ? 8 : 147456 / STAGE;
    static constexpr int PD = NS - 1;             // steps of loads in flight
    static constexpr int CT = TT == 128 ? 64 : TT;                // tokens the coupling takes per pass
    static constexpr int ZS = TR * (CT * 32 + 8);                 // bytes of Zs[rho][t][j] for one pass
    static constexpr int LDS = NS * STAGE > ZS ? NS * STAGE : ZS;
    static constexpr int LPW = ROWS / RPL / 8;    // direct-to-LDS loads per wavefront and stage
    static constexpr int CW = TT / 16 < 8 ? TT / 16 : 8;          // wavefronts that own a 32 x 32 part of the tile
    static_assert(TT == 128 || TT == 64, "token tiles of the fused kernel");
    static_assert(BK == 64 || BK == 128, "step depths of the fused kernel");
    static_assert(LDS <= 160 * 1024, "LDS budget");
    static_assert(ROWS % (RPL * 8) == 0 && TT % RPL == 0, "every wavefront issues the same number of loads per stage, none straddling X and Vt");
    static_assert(LPW * (PD - 1) < 64, "vmcnt range");
};

// asynchronous 16-byte LDS read the compiler does not see as a memory access (reads it can see make it
// wait for ALL outstanding direct-to-LDS loads); the caller waits on lgkmcnt itself and passes the
// value through tie_to_wait after that wait, before the first use
__device__ __forceinline__ bf16x8 lds_read_b128_async(unsigned addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
__device__ __forceinline__ bf16x8 tie_to_wait(bf16x8 v) {
    asm volatile("" : "+v"(v));
    return v;
}


// Coupling of one 64-token x 64-rank tile whose Z values sit in LDS as Zs[rho][t][j] (bf16):
// A[t][i][rho] = sum_j S[i][j][rho] Z[t][j][rho] on v_mfma_f32_16x16x16_bf16, one MFMA per rank index
// and 16 tokens, S tiles from the packed Sp[rho][i][j]. The 64 rank indices form 8 groups of 8; a
// group's result replaces the group's own Z rows IN PLACE as As[i][t][8 rho] (the group is read
// completely first and only one wavefront touches it), so that A leaves with full-line stores.
constexpr int GROUP = 8 * ZSTR;
static_assert(16 * TN * 16 <= GROUP, "in-place A must fit in the rows it replaces");

// the S tiles of group c as MFMA B operands (lane: output block i = lane % 16, input blocks 4 (lane / 16) ..)
__device__ __forceinline__ void load_s_group(const bf16_t* __restrict__ Sp, int rho0, int c, int r, s16x4 (&sfrag)[8]) {
    const int lane = threadIdx.x & 63, ci = lane & 15, cg = lane >> 4;
#pragma unroll
    for (int ri = 0; ri < 8; ++ri) {
        int rg = rho0 + c * 8 + ri;
        if (rg > r - 1) rg = r - 1;                     // groups past r are computed on repeated tiles and not stored
        sfrag[ri] = *(const s16x4*)(Sp + (int64_t)rg * 256 + ci * 16 + cg * 4);
    }
}

// Must be entered after a barrier that follows the last write to Zs. The four 8-byte units (4 blocks
// each) of a token's 32 bytes are stored XOR 2 for tokens 8..15 of every 16, so that the 32 lanes a
// fragment read serves per clock (16 tokens x 2 units) touch all 64 banks once.
template <int TNT = TN>                                  // tokens in the tile (rows of Zs hold TNT tokens)
__device__ __forceinline__ void couple_group(unsigned char* grp, const s16x4 (&sfrag)[8]) {
    constexpr int ZSTR = TNT * 32 + 8;
    const int lane = threadIdx.x & 63, ci = lane & 15, cg = lane >> 4;
    // Two batches of 16 fragment reads, each issued back to back before its MFMAs, so that the LDS
    // latency is paid once per batch instead of once per MFMA.
    f32x4 d[TNT / 16][8];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        s16x4 a[4][TNT / 16];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
#pragma unroll
            for (int tg = 0; tg < TNT / 16; ++tg)
                a[r4][tg] = *(const s16x4*)(grp + (half * 4 + r4) * ZSTR + (tg * 16 + ci) * 32 + (cg ^ (2 * (ci >> 3))) * 8);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
#pragma unroll
            for (int tg = 0; tg < TNT / 16; ++tg)
                d[tg][half * 4 + r4] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[r4][tg], sfrag[half * 4 + r4], f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    // d[tg][ri][e]: token tg*16 + 4*(lane/16) + e, output block i = lane%16
#pragma unroll
    for (int tg = 0; tg < TNT / 16; ++tg)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int tok = tg * 16 + 4 * cg + e;
            *(uint4*)(grp + (ci * TNT + (tok ^ ci)) * 16) =
                make_uint4(pack2_bf16(d[tg][0][e], d[tg][1][e]), pack2_bf16(d[tg][2][e], d[tg][3][e]),
                           pack2_bf16(d[tg][4][e], d[tg][5][e]), pack2_bf16(d[tg][6][e], d[tg][7][e]));
        }
}

// A[t][i][rho0 .. rho0+63] from the in-place groups: 8 lanes write the 128 contiguous bytes of one
// (token, block). tok(t) is the token (relative to t0) that row t of the tile stands for. A thread's
// items go in batches of four: the LDS reads of a batch are issued together, then its stores, so that
// the LDS latency is paid once per batch.
// Must be entered after a barrier that follows couple_group.
template <int NW, class TokMap, int TNT = TN>          // NW wavefronts in the workgroup, TNT tokens in the tile
__device__ __forceinline__ void store_a_tile(const unsigned char* Zs, bf16_t* __restrict__ A,
                                             int64_t T, int64_t t0, int rho0, int b, int r, TokMap tok) {
    const int tid = threadIdx.x, c8 = tid & 7;
    constexpr int PER = NW * 8;                         // (token, block) items per sweep of the workgroup
    constexpr int UB = 4;
    const int di = PER % b, dt = PER / b;
    int v = tid >> 3, i = v % b, t = v / b;
    if (rho0 + c8 * 8 >= r) return;
    const unsigned char* src = Zs + c8 * (8 * (TNT * 32 + 8));
    bf16_t* dst = A + t0 * b * r + rho0 + c8 * 8;
    const int tokens_left = T - t0 < TNT * 2 ? (int)(T - t0) : TNT * 2;   // tok() stays below 2 TNT
    for (; v < TNT * b; v += PER * UB) {
        u32x4 val[UB];
        int off[UB];                                    // elements from dst; (tile tokens) * b * r fits 32 bits (host-checked)
        bool ok[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int tk = tok(t);
            ok[u] = v + u * PER < TNT * b && tk < tokens_left;
            const int tt = ok[u] ? t : 0;               // keep the LDS address inside the tile
            val[u] = *(const u32x4*)(src + (i * TNT + (tt ^ (i & 15))) * 16);
            off[u] = (tk * b + i) * r;
            i += di; t += dt;
            if (i >= b) { i -= b; ++t; }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < UB; ++u)
            if (ok[u]) *(u32x4*)(dst + off[u]) = val[u];
    }
}

// Stand-alone coupling (the middle kernel of the three-kernel path): Z[T][b][r] -> A[T][b][r].
// The Z tile is read with full-line loads (8 lanes per 128-byte row segment) and transposed on its
// way into LDS; blocks j and j+1 travel together so that every LDS write is a bf16 pair.
// TNT tokens per workgroup: 64, or 32 or 16 when larger tiles would leave most of the chip idle.
// Z8: Z holds 8-bit floats (E4M3, written by the stage-1 product of the quantised-intermediate execution),
// one byte per element in the same [T][b][r] order; they are widened to bf16 (exactly) on their way into LDS.
template <int TNT, bool Z8>
__global__ __launch_bounds__(512)
void blast_coupling_kernel(const bf16_t* __restrict__ Z, const bf16_t* __restrict__ Sp, bf16_t* __restrict__ A,
                           int64_t T, int b, int r, int tiles_r, int nblk) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* Zs = smem;
    constexpr int ZSTR = TNT * 32 + 8, GROUP = 8 * ZSTR, ZS_BYTES = TR * ZSTR;   // (shadow the 64-token values)
    static_assert(16 * TNT * 16 <= GROUP && ZS_BYTES % 16 == 0, "in-place A must fit; Zs is cleared with 16-byte stores");
    constexpr int NTHR = 512;                            // 8 wavefronts: one group of 8 rank indices each
    const int tid = threadIdx.x;
    const int logical = xcd_contiguous(blockIdx.x, nblk);
    const int tile_t = logical / tiles_r, tile_r = logical % tiles_r;
    const int64_t t0 = (int64_t)tile_t * TNT;
    const int rho0 = tile_r * TR;
    s16x4 sfrag[8];
    load_s_group(Sp, rho0, tid >> 6, r, sfrag);          // in flight while Z is brought in
    const int c8 = tid & 7;                              // which 8 rank indices of the 64
    int rho = rho0 + c8 * 8;
    if (rho > r - 8) rho = r - 8;                        // past r: repeat valid data, never stored (r is a multiple of 8)
    const int npair = (b + 1) >> 1;
    if (b < 16)
        for (int i = tid * 16; i < ZS_BYTES; i += NTHR * 16) *(uint4*)(Zs + i) = make_uint4(0, 0, 0, 0);
    if (b < 16) __syncthreads();
    // work item = (token, block pair): 8 lanes cover its 128-byte segment; 4 items in flight per thread
    const int items = TNT * npair;
    constexpr int IPS = NTHR / 8;                        // items per sweep of the workgroup
    for (int base = 0; base < items; base += IPS * 4) {
        uint4 v0[4], v1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int it = base + u * IPS + (tid >> 3);
            if (it > items - 1) it = items - 1;
            const int t = it / npair, jp = it - t * npair;
            int64_t tok = t0 + t;
            if (tok > T - 1) tok = T - 1;
            const int j1 = 2 * jp + 1 < b ? 2 * jp + 1 : 2 * jp;
            if constexpr (Z8) {
                const unsigned char* Zb = (const unsigned char*)Z;
                const uint2 q0 = *(const uint2*)(Zb + (tok * b + 2 * jp) * r + rho);
                const uint2 q1 = *(const uint2*)(Zb + (tok * b + j1) * r + rho);
                auto widen = [](uint2 q) {              // 8 x E4M3 -> 8 x bf16 (every E4M3 value is a bf16 value)
                    const auto a = __builtin_amdgcn_cvt_pk_f32_fp8((int)q.x, false), bq = __builtin_amdgcn_cvt_pk_f32_fp8((int)q.x, true);
                    const auto c = __builtin_amdgcn_cvt_pk_f32_fp8((int)q.y, false), dq = __builtin_amdgcn_cvt_pk_f32_fp8((int)q.y, true);
                    return make_uint4(pack2_bf16(a[0], a[1]), pack2_bf16(bq[0], bq[1]), pack2_bf16(c[0], c[1]), pack2_bf16(dq[0], dq[1]));
                };
                v0[u] = widen(q0);
                v1[u] = widen(q1);
            } else {
                v0[u] = *(const uint4*)(Z + (tok * b + 2 * jp) * r + rho);
                v1[u] = *(const uint4*)(Z + (tok * b + j1) * r + rho);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int it = base + u * IPS + (tid >> 3);
            if (it < items) {
                const int t = it / npair, jp = it - t * npair;
                const bool has1 = 2 * jp + 1 < b;
                const uint32_t w0[4] = {v0[u].x, v0[u].y, v0[u].z, v0[u].w};
                const uint32_t w1[4] = {v1[u].x, v1[u].y, v1[u].z, v1[u].w};
                unsigned char* dst = Zs + (c8 * 8) * ZSTR + t * 32 + ((jp >> 1) ^ (2 * ((t >> 3) & 1))) * 8 + (jp & 1) * 4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t hi = has1 ? w1[e] : 0u;
                    *(uint32_t*)(dst + (2 * e) * ZSTR) = (w0[e] & 0xFFFFu) | (hi << 16);
                    *(uint32_t*)(dst + (2 * e + 1) * ZSTR) = (w0[e] >> 16) | (hi & 0xFFFF0000u);
                }
            }
        }
    }
    __syncthreads();
    couple_group<TNT>(Zs + (tid >> 6) * GROUP, sfrag);
    __syncthreads();
    auto same = [](int t) { return t; };
    store_a_tile<8, decltype(same), TNT>(Zs, A, T, t0, rho0, b, r, same);
}

// Stage 1 + coupling. Per step (one chunk of BK input columns of one input block j) a stage of LDS holds
// TT X rows and 64 Vt rows of 2 BK bytes; its 16-byte pieces are XOR-swizzled by the row so that the 16
// lanes a ds_read_b128 serves per clock (16 consecutive rows) hit 16 different 16-byte columns of the 64
// banks, without the row padding that a direct-to-LDS load cannot produce (lane l of such a load always
// lands at base + 16 l). Loads for step s + PD are issued right after the barrier of step s, while the
// matrix pipe is idle (a load issued while the SIMD's matrix pipe is busy takes three times as long to
// issue); vmcnt counts them, so one wait + one barrier per step is all the synchronisation.
// The fragment reads are inline assembly with their own lgkmcnt waits (reads that the compiler can see
// make it wait for ALL outstanding direct-to-LDS loads first) and go out in batches of two k16 steps,
// two batches ahead of the MFMAs that consume them.
// A step costs a fixed 250 ... 300 clocks of barrier, waits and cursor arithmetic whatever its depth
// (measured with the loads, the reads and the MFMAs removed in turn), which is why it is as deep as LDS
// allows, and why the fetch cursor only does arithmetic at block boundaries.
// The chunks are aligned to BK GLOBAL input columns (n_in is a multiple of BK), not to the start of the
// block: block j walks chunks floor(j q / BK) .. ceil((j+1) q / BK) - 1, so every X piece is whole
// 128-byte lines whatever q is. The columns of a boundary chunk that belong to a neighbouring block
// meet zeros in Va (the chunk-aligned copy of Vt, rows of qp elements), so nothing has to be masked.
template <int TT, int BK>
__global__ __launch_bounds__(512)
void blast_stage12_kernel(const bf16_t* __restrict__ X, const bf16_t* __restrict__ Va,
                          const bf16_t* __restrict__ Sp, bf16_t* __restrict__ A,
                          int64_t T, int n_in, int b, int r, int qp, int tiles_r, int nblk) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    using C = StCfg<TT, BK>;
    constexpr int ST_STAGE = C::STAGE, ST_LPW = C::LPW, ST_NS = C::NS, ST_PD = C::PD, KS = C::KS;
    constexpr int LOG_BK = BK == 128 ? 7 : 6;
    const bool computes = wave < C::CW;                  // uniform: this wavefront owns a 32 x 32 part of the tile
    const int wm = (wave >> 1) % (TT / 32), wn = wave & 1;   // token part, rank half of this wavefront's 32 x 32
    const int logical = xcd_contiguous(blockIdx.x, nblk);
    const int tile_t = logical / tiles_r, tile_r = logical % tiles_r;
    const int64_t t0 = (int64_t)tile_t * TT;
    const int rho0 = tile_r * TR;
    const int q = n_in / b;
    auto chunk_begin = [&](int j) { return (j * q) >> LOG_BK; };
    auto chunks_of = [&](int j) { return (((j + 1) * q + BK - 1) >> LOG_BK) - ((j * q) >> LOG_BK); };
    const int nsteps = [&] { int n = 0; for (int j = 0; j < b; ++j) n += chunks_of(j); return n; }();

    // Load h of this wavefront fills operand rows RPL (LPW wave + h) .. + RPL - 1 of a stage: lane l brings
    // the piece that belongs at row l / PPR of those, slot l % PPR.
    unsigned off[ST_LPW];
#pragma unroll
    for (int h = 0; h < ST_LPW; ++h) {
        const int row = C::RPL * (ST_LPW * wave + h) + lane / C::PPR;
        const int piece = (lane % C::PPR) ^ ((row >> C::SH) & (C::PPR - 1));
        if (row < TT) {
            int xr = row;
            if (t0 + xr > T - 1) xr = (int)(T - 1 - t0);    // rows past the end re-read the last row; never stored
            off[h] = (xr * n_in + piece * 8) * 2;           // bytes from the tile's first X row
        } else {
            int vr = rho0 + row - TT;
            if (vr > r - 1) vr = r - 1;
            off[h] = (vr * qp + piece * 8) * 2;             // bytes from Va[j]
        }
    }
    const unsigned char* xs = (const unsigned char*)(X + t0 * n_in);
    const unsigned char* vs = (const unsigned char*)Va;
    const int64_t v_block = (int64_t)r * qp * 2;        // bytes of one Va[j]

    // fetch cursor (uniform): pointers to the chunk of X and of Va[fj] it stands on; arithmetic other than
    // an increment only when it crosses into the next block
    int fj = 0, fk = 0, fetched = 0, fn = chunks_of(0);
    const unsigned char* xc = xs;
    const unsigned char* vc = vs;
    auto issue = [&](int stage_off) {
#pragma unroll
        for (int h = 0; h < ST_LPW; ++h) {
            const bool isx = C::RPL * (ST_LPW * wave + h) < TT;            // uniform
            asm volatile("" : "+v"(off[h]));                               // keeps the offset a register operand: scalar base + lane offset addressing, no address arithmetic
            __builtin_amdgcn_global_load_lds(BLR_GPTR((isx ? xc : vc) + off[h]),
                                             BLR_LPTR(smem + stage_off + (ST_LPW * wave + h) * 1024), 16, 0, 0);
        }
        if (fetched < nsteps - 1) {                     // the cursor stops at the last step; later issues repeat it
            ++fetched;
            if (++fk == fn) {
                fk = 0; ++fj; fn = chunks_of(fj);
                xc = xs + (size_t)chunk_begin(fj) * C::RB;
                vc = vs + fj * v_block;
            } else {
                xc += C::RB;
                vc += C::RB;
            }
        }
    };

    // fragment addresses inside a stage: row m of this wavefront's 32 tokens (resp. ranks), k group kg; the
    // piece of k16 step ks is (2 ks + kg) ^ swizzle(row) = (kg ^ swizzle(row)) ^ 2 ks
    const int m = lane & 31, kg = lane >> 5;
    const unsigned lds0 = (unsigned)(uintptr_t)BLR_LPTR(smem);
    const unsigned kgx16 = (unsigned)((kg ^ ((m >> C::SH) & (C::PPR - 1))) * 16);
    const unsigned rowa = lds0 + (wm * 32 + m) * C::RB, rowb = lds0 + (TT + wn * 32 + m) * C::RB;

    int cstage = 0, istage = ST_PD * ST_STAGE;          // byte offsets of the stage to compute on / to refill
    bf16x8 fr[2][2][2];                                 // [batch parity][k16 step in the batch][X, Vt]
    auto read_batch = [&](auto BQ, int stage_off) {     // the fragments of k16 steps 2 bq, 2 bq + 1
        constexpr int bq = decltype(BQ)::value;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const unsigned sw = kgx16 ^ (unsigned)((2 * bq + u) * 32);
            fr[bq & 1][u][0] = lds_read_b128_async(rowa + stage_off + sw);
            fr[bq & 1][u][1] = lds_read_b128_async(rowb + stage_off + sw);
        }
    };
    auto step = [&](f32x16& acc) {
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" :: "n"(ST_LPW * (ST_PD - 1)) : "memory");
        const int rstage = cstage;                      // the stage of this step
        const int wstage = istage;                      // the stage every wavefront finished reading one step ago
        cstage = cstage + ST_STAGE == ST_NS * ST_STAGE ? 0 : cstage + ST_STAGE;
        istage = istage + ST_STAGE == ST_NS * ST_STAGE ? 0 : istage + ST_STAGE;
        if (!computes) { issue(wstage); return; }       // moves operands only
        read_batch(std::integral_constant<int, 0>{}, rstage);
        read_batch(std::integral_constant<int, 1>{}, rstage);
        // the refill goes out here: the fragment reads are on their way, and the MFMAs that the wavefronts
        // of this SIMD issued before the barrier have drained by now
        issue(wstage);
        static_for<KS / 2>([&](auto BQ) {
            constexpr int bq = decltype(BQ)::value;
            if constexpr (bq + 1 < KS / 2) asm volatile("s_waitcnt lgkmcnt(4)" ::: "memory");   // in order: batch bq has arrived
            else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int u = 0; u < 2; ++u) { fr[bq & 1][u][0] = tie_to_wait(fr[bq & 1][u][0]); fr[bq & 1][u][1] = tie_to_wait(fr[bq & 1][u][1]); }
            __builtin_amdgcn_sched_barrier(0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[bq & 1][0][0], fr[bq & 1][0][1], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[bq & 1][1][0], fr[bq & 1][1][1], acc, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (bq + 2 < KS / 2) read_batch(std::integral_constant<int, bq + 2>{}, rstage);
        });
    };

    for (int s = 0; s < ST_PD; ++s) issue(s * ST_STAGE);

    // Z of the whole tile, bf16, in registers: zq[e][jp] = (Z_{2jp}, Z_{2jp+1}) of accumulator element e,
    // i.e. token 8 (e/4) + 4 (lane/32) + e%4 and rank lane%32 of this wavefront's 32 x 32
    uint32_t zq[16][8];
#pragma unroll
    for (int e = 0; e < 16; ++e)
#pragma unroll
        for (int jp = 0; jp < 8; ++jp) zq[e][jp] = 0u;  // blocks past b stay zero
    static_for<8>([&](auto JP) {
        constexpr int jp = decltype(JP)::value;
        if (2 * jp < b) {
            f32x16 acc;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0.f;
            const int n0 = chunks_of(2 * jp);
#pragma unroll 1
            for (int kc = 0; kc < n0; ++kc) step(acc);
#pragma unroll
            for (int e = 0; e < 16; ++e) { zq[e][jp] = pack2_bf16(acc[e], 0.f); acc[e] = 0.f; }
            if (2 * jp + 1 < b) {
                const int n1 = chunks_of(2 * jp + 1);
#pragma unroll 1
                for (int kc = 0; kc < n1; ++kc) step(acc);
#pragma unroll
                for (int e = 0; e < 16; ++e) zq[e][jp] |= pack2_bf16(0.f, acc[e]);
            }
        }
    });
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // the repeated loads of the last steps have landed too

    // coupling, 64 tokens at a time: pass hf takes tokens 16 hf .. 16 hf + 15 of every wavefront's 32 (so
    // that each wavefront hands over half of its registers per pass) and lays them out as Zs[rho][t][j];
    // wavefront w then couples the 8 rank indices of group w
    unsigned char* Zs = smem;
    s16x4 sfrag[8];
    load_s_group(Sp, rho0, wave, r, sfrag);             // in flight across the barrier and the Zs writes
    if constexpr (TT == 128) {
        static_for<2>([&](auto HF) {
            constexpr int hf = decltype(HF)::value;
            if (hf == 0 || T - t0 > 16) {               // uniform
                __syncthreads();                        // stages / the previous pass's A are no longer read
                unsigned char* zrow = Zs + (wn * 32 + m) * ZSTR + (wm * 16 + 4 * kg) * 32;
#pragma unroll
                for (int e2 = 0; e2 < 8; ++e2) {
                    unsigned char* dst = zrow + (8 * (e2 / 4) + (e2 % 4)) * 32;
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        *(uint2*)(dst + (v ^ (2 * ((e2 / 4) & 1))) * 8) = make_uint2(zq[8 * hf + e2][2 * v], zq[8 * hf + e2][2 * v + 1]);
                }
                __syncthreads();
                couple_group(Zs + wave * GROUP, sfrag);
                __syncthreads();
                store_a_tile<8>(Zs, A, T, t0, rho0, b, r, [](int t) { return (t >> 4) * 32 + hf * 16 + (t & 15); });
            }
        });
    } else {
        // 64 tokens: one pass; the four computing wavefronts hand over all 32 tokens of their parts
        constexpr int ZSTR_T = TT * 32 + 8, GROUP_T = 8 * ZSTR_T;
        __syncthreads();                                // the stages are no longer read
        if (computes) {
            unsigned char* zrow = Zs + (wn * 32 + m) * ZSTR_T + (wm * 32 + 4 * kg) * 32;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                unsigned char* dst = zrow + (8 * (e / 4) + (e % 4)) * 32;
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    *(uint2*)(dst + (v ^ (2 * ((e / 4) & 1))) * 8) = make_uint2(zq[e][2 * v], zq[e][2 * v + 1]);
            }
        }
        __syncthreads();
        couple_group<TT>(Zs + wave * GROUP_T, sfrag);
        __syncthreads();
        auto same = [](int t) { return t; };
        store_a_tile<8, decltype(same), TT>(Zs, A, T, t0, rho0, b, r, same);
    }
}

}  // namespace

bool blast_fused_supported(int64_t T, int n_in, int b, int r) {
    if (T <= 0 || b <= 0 || b > 16 || n_in % b) return false;
    const int q = n_in / b;
    const int64_t nblk = blast_fused_tiles(T, r);
    // 64 | n_in: the chunk grid is aligned to 64 input columns and must end with the row
    return q % 8 == 0 && r % 8 == 0 && n_in % 64 == 0 && nblk < (1ll << 30) &&
           ((int64_t)128 * n_in + 128) * 2 < (1ll << 31) && ((int64_t)r * blast_va_row(q, blast_chunk(n_in, b)) + 128) * 2 < (1ll << 31);
}

int64_t blast_fused_tiles(int64_t T, int r) { return ((T + 127) / 128) * ((r + TR - 1) / TR); }

namespace {
template <int TT, int BK>
hipError_t launch_stage12_inst(const void* X, const void* Va, const void* Sp, void* A,
                               int64_t T, int n_in, int b, int r, hipStream_t s) {
    static LdsLimitOnce lds_limit;
    constexpr int lds = StCfg<TT, BK>::LDS;
    if (hipError_t e = lds_limit.set({(const void*)blast_stage12_kernel<TT, BK>}, lds); e != hipSuccess) return e;
    const int tiles_t = (int)((T + TT - 1) / TT), tiles_r = (r + TR - 1) / TR;
    const int nblk = tiles_t * tiles_r;
    hipLaunchKernelGGL((blast_stage12_kernel<TT, BK>), dim3((unsigned)nblk), dim3(512), lds, s,
                       (const bf16_t*)X, (const bf16_t*)Va, (const bf16_t*)Sp, (bf16_t*)A, T, n_in, b, r,
                       blast_va_row(n_in / b, BK), tiles_r, nblk);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_blast_stage12(const void* X, const void* Va, const void* Sp, void* A,
                                int64_t T, int n_in, int b, int r, hipStream_t s) {
    // one workgroup per compute unit: 64-token tiles while they still fit in one round of the 256; steps of
    // 128 contraction indices where the input blocks are whole numbers of such chunks.
    // (32-token tiles for still fewer tokens were built and measured: 4096 x 4096, r = 640 at 512 tokens 37.9 ->
    // 33.6 us for the whole call against 29.8 us on three kernels, whose finer tiles keep every compute unit
    // busy; a lone workgroup walks 4096 contraction indices in 26 us however many stages it has in flight.)
    const bool small = blast_fused_tiles(T, r) <= 128;
    if (blast_chunk(n_in, b) == 128)
        return small ? launch_stage12_inst<64, 128>(X, Va, Sp, A, T, n_in, b, r, s) : launch_stage12_inst<128, 128>(X, Va, Sp, A, T, n_in, b, r, s);
    return small ? launch_stage12_inst<64, 64>(X, Va, Sp, A, T, n_in, b, r, s) : launch_stage12_inst<128, 64>(X, Va, Sp, A, T, n_in, b, r, s);
}

template <int TNT, bool Z8>
static hipError_t launch_coupling_inst(const void* Z, const void* Sp, void* A, int64_t T, int b, int r, hipStream_t s) {
    constexpr int lds = TR * (TNT * 32 + 8);
    static LdsLimitOnce lds_limit;
    if (hipError_t e = lds_limit.set({(const void*)blast_coupling_kernel<TNT, Z8>}, lds); e != hipSuccess) return e;
    const int tiles_t = (int)((T + TNT - 1) / TNT), tiles_r = (r + TR - 1) / TR;
    const int nblk = tiles_t * tiles_r;
    hipLaunchKernelGGL((blast_coupling_kernel<TNT, Z8>), dim3((unsigned)nblk), dim3(512), lds, s,
                       (const bf16_t*)Z, (const bf16_t*)Sp, (bf16_t*)A, T, b, r, tiles_r, nblk);
    return hipGetLastError();
}

hipError_t launch_blast_coupling(const void* Z, const void* Sp, void* A, int64_t T, int b, int r, hipStream_t s, bool z_fp8) {
    // 64-token tiles unless they would leave most compute units without a workgroup
    const int64_t tiles64 = ((T + 63) / 64) * ((r + TR - 1) / TR);
    if (z_fp8) return tiles64 < 200 ? launch_coupling_inst<32, true>(Z, Sp, A, T, b, r, s) : launch_coupling_inst<64, true>(Z, Sp, A, T, b, r, s);
    // ... and 16-token tiles for the fewest tokens (4096 x 4096, r = 640 at 192 ... 384 tokens: 0.5 ... 1 us of the 20 ... 26 us call)
    if (tiles64 <= 64) return launch_coupling_inst<16, false>(Z, Sp, A, T, b, r, s);
    if (tiles64 < 200) return launch_coupling_inst<32, false>(Z, Sp, A, T, b, r, s);
    return launch_coupling_inst<64, false>(Z, Sp, A, T, b, r, s);
}

namespace {

// ---------------------------------------------------------------------------------------------
// Whole BLAST layer in one kernel, for layers whose coupled intermediate fits on chip:
// a workgroup (8 wavefronts) owns FT = 32 tokens and ALL rank indices and all blocks.
//   phase 0  the X tile (32 rows, contiguous) goes to LDS with fully coalesced 16-byte loads;
//   phase 1  Z_j = X_j V_j for every j (wavefronts split j) on v_mfma_f32_32x32x16_bf16; the V
//            fragments come straight from global memory in fragment order (Vf: one load instruction
//            of a wavefront reads one contiguous KiB, i.e. 8 cache lines instead of ~24), each is
//            used by exactly one wavefront; result as bf16 into LDS, Zs[rho][t][j];
//   phase 2  per group of 8 rank indices: A[t][i] = sum_j Z[t][j] S[i][j] on v_mfma_f32_16x16x16_bf16,
//            written back IN PLACE over the group's own Z rows as As[i][t][8 rho] (the group is read
//            completely before it is overwritten, and only one wavefront touches it);
//   phase 3  Y_i = A_i U_i^T (wavefronts split i) on v_mfma_f32_16x16x32_bf16, A fragments from LDS,
//            U fragments from global memory in fragment order (Uf), result staged in LDS (over the
//            dead X tile) and written to Y with 16-byte coalesced stores.
// Neither Z nor A ever leaves the chip: HBM traffic is X, the factors and Y. The factor fragments
// of the next phase are fetched while the current one runs.
// ---------------------------------------------------------------------------------------------
constexpr int FT = 32;                          // tokens per workgroup
constexpr int FZSTR = FT * 32 + 8;              // bytes of one rho row of Zs
constexpr int FCHUNK = 8 * FZSTR;               // 8 rho rows; also holds As[16 i][32 t][8 rho] (8192 B)
constexpr int FWAVES = 8;
constexpr int FTHREADS = 64 * FWAVES;
static_assert(16 * FT * 16 <= FCHUNK, "in-place A must fit in the chunk it replaces");

// r <= 32*NT rank indices; KG k-steps of 16 fetched per round; NPT = (n_out/b)/16 output tiles per block.
// Every global load is unconditional (indices are clamped, work that does not exist is computed on
// repeated data and not written) so that each wait counts exactly the loads older than the data it needs.
// 16-byte global load the compiler can neither move nor count: the caller waits on vmcnt itself
// (the count being the number of vector-memory operations issued after this one) and ties the
// result to that wait before using it. The "memory" clobber keeps other loads from crossing it.
__device__ __forceinline__ u32x4 global_load_b128_pinned(const void* uniform_base, unsigned lane_offset) {
    u32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(v) : "v"(lane_offset), "s"(uniform_base) : "memory");
    return v;
}

template <int NT, int KG, int NPT>
__global__ __launch_bounds__(FTHREADS) __attribute__((amdgpu_waves_per_eu(1, 2)))
void blast_full_kernel(const bf16_t* __restrict__ X, const bf16_t* __restrict__ Sp, const bf16_t* __restrict__ Vf,
                       const bf16_t* __restrict__ Uf, bf16_t* __restrict__ Y,
                       int64_t T, int n_in, int n_out, int b, int r) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int nchunks = r >> 3;                                     // r is a multiple of 8
    unsigned char* Zs = smem;
    unsigned char* XY = smem + NT * 4 * FCHUNK;                      // X tile [FT][n_in], later Y tile [FT][n_out]
    const int xstr = n_in * 2 + 16, ystr = n_out * 2 + 16;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: block and fragment offsets stay on the scalar unit
    const unsigned lane16 = (unsigned)lane * 16u;
    const int64_t t0 = (int64_t)blockIdx.x * FT;
    const int q = n_in / b, p = n_out / b;
    const int nks = (q + 15) >> 4;
    const int ci = lane & 15, cg = lane >> 4;
    const int l32 = lane & 31, kg = lane >> 5;
    // this wavefront's input blocks (phase 1), rank groups (phase 2) and output blocks (phase 3)
    const int jw[2] = {wave < b ? wave : b - 1, wave + FWAVES < b ? wave + FWAVES : b - 1};
    const int cw[2] = {wave < nchunks ? wave : nchunks - 1, wave + FWAVES < nchunks ? wave + FWAVES : nchunks - 1};

    // ---- phase 0a: the X tile is requested first, so that it is the first thing the vector-memory
    // pipe (64 bytes per clock and CU) delivers; the factor fragments queue up behind it and arrive
    // while the tile is written to LDS and the first products run. A wavefront brings 4 token rows,
    // 64 16-byte pieces per load (rows past T repeat the last row; lanes past the row end load and
    // later store the row's last piece once more, so that no load or store sits under a per-lane
    // condition, which would let the compiler move the load down to its use).
    constexpr int XH = 2;                                            // pieces of 64 x 16 bytes per row and round
    const int cpr_in = n_in >> 3;                                    // 16-byte pieces per row
    u32x4 xv[FT / FWAVES][XH];
#pragma unroll
    for (int u = 0; u < FT / FWAVES; ++u) {
        int64_t tx = t0 + wave * (FT / FWAVES) + u;
        if (tx > T - 1) tx = T - 1;
        const unsigned char* src = (const unsigned char*)(X + tx * n_in);
#pragma unroll
        for (int h = 0; h < XH; ++h) {
            const int cc = h * 64 + lane < cpr_in ? h * 64 + lane : cpr_in - 1;
            xv[u][h] = global_load_b128_pinned(src, (unsigned)cc * 16u);   // (the compiler would sink plain loads to their use, behind the factor loads)
        }
    }

    // V fragments (first round of k-steps)
    uint4 braw[2][KG][NT];
    auto load_vf = [&](int ks0) {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int u = 0; u < KG; ++u) {
                int ks = ks0 + u;
                if (ks > nks - 1) ks = nks - 1;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    braw[jj][u][nt] = *(const uint4*)((const unsigned char*)Vf + (((size_t)(jw[jj] * NT + nt) * nks + ks) << 10) + lane16);
            }
    };
    load_vf(0);
    // the 2 KG NT fragment loads above are the only vector-memory operations younger than the tile's
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * KG * NT) : "memory");
#pragma unroll
    for (int u = 0; u < FT / FWAVES; ++u)
#pragma unroll
        for (int h = 0; h < XH; ++h) asm volatile("" : "+v"(xv[u][h]));

    // ---- phase 0b: X tile -> LDS. The 16 pad bytes of a row are zeroed because the last k-step of
    // the last block may read them against zero V fragments.
    {
        if (tid < FT) *(uint4*)(XY + tid * xstr + n_in * 2) = make_uint4(0, 0, 0, 0);
        if (b < 16)                                                 // unused j slots must read as zero
            for (int i = tid * 16; i < NT * 4 * FCHUNK; i += FTHREADS * 16) *(uint4*)(Zs + i) = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < FT / FWAVES; ++u)
#pragma unroll
            for (int h = 0; h < XH; ++h) {
                const int cc = h * 64 + lane < cpr_in ? h * 64 + lane : cpr_in - 1;
                *(u32x4*)(XY + (wave * (FT / FWAVES) + u) * xstr + cc * 16) = xv[u][h];
            }
        if (XH * 64 < cpr_in) {                                     // rows longer than 2 KiB (n_in <= 2048): a second round
            uint4 xw[FT / FWAVES][XH];
#pragma unroll
            for (int u = 0; u < FT / FWAVES; ++u) {
                int64_t tx = t0 + wave * (FT / FWAVES) + u;
                if (tx > T - 1) tx = T - 1;
                const unsigned char* src = (const unsigned char*)(X + tx * n_in);
#pragma unroll
                for (int h = 0; h < XH; ++h) {
                    const int cc = (XH + h) * 64 + lane < cpr_in ? (XH + h) * 64 + lane : cpr_in - 1;
                    xw[u][h] = *(const uint4*)(src + (unsigned)cc * 16u);
                }
            }
#pragma unroll
            for (int u = 0; u < FT / FWAVES; ++u)
#pragma unroll
                for (int h = 0; h < XH; ++h) {
                    const int cc = (XH + h) * 64 + lane < cpr_in ? (XH + h) * 64 + lane : cpr_in - 1;
                    *(uint4*)(XY + (wave * (FT / FWAVES) + u) * xstr + cc * 16) = xw[u][h];
                }
        }
    }
    __syncthreads();

    // S tiles of this wavefront's rank groups: in flight during phase 1
    // (Sp is in fragment order, two rank indices per 16 bytes: an 8-byte load costs the address path
    // of the memory pipe as much as a 16-byte one)
    s16x4 sfr[2][8];
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int rp = 0; rp < 4; ++rp) {
            const uint4 t = *(const uint4*)((const unsigned char*)Sp + ((size_t)(cw[cc] * 4 + rp) << 10) + lane16);
            const uint2 lo = make_uint2(t.x, t.y), hi = make_uint2(t.z, t.w);
            sfr[cc][2 * rp] = *(const s16x4*)&lo;
            sfr[cc][2 * rp + 1] = *(const s16x4*)&hi;
        }

    // ---- phase 1: both blocks of this wavefront, then one 4-byte LDS write per (token, rank index)
    // holding the pair (slots 2*wave, 2*wave+1 of the permuted block order j' = (j%8)*2 + j/8, which
    // the packed S tiles follow)
    uint4 ufr[2][NPT][NT];
    auto load_u = [&](auto II) {
        constexpr int ii = decltype(II)::value;
        const int i = wave + ii * FWAVES < b ? wave + ii * FWAVES : b - 1;
#pragma unroll
        for (int nt = 0; nt < NPT; ++nt)
#pragma unroll
            for (int ks = 0; ks < NT; ++ks)
                ufr[ii][nt][ks] = *(const uint4*)((const unsigned char*)Uf + ((size_t)((i * NPT + nt) * NT + ks) << 10) + lane16);
    };
    {
        f32x16 zacc[2][NT];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int e = 0; e < 16; ++e) zacc[jj][nt][e] = 0.f;
        auto mul = [&](int ks0) {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int u = 0; u < KG; ++u) {
                    if (ks0 + u < nks) {
                        const bf16x8 a = *(const bf16x8*)(XY + l32 * xstr + (jw[jj] * q + (ks0 + u) * 16 + kg * 8) * 2);
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            zacc[jj][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, *(const bf16x8*)&braw[jj][u][nt], zacc[jj][nt], 0, 0, 0);
                    }
                }
        };
        mul(0);
        for (int ks0 = KG; ks0 < nks; ks0 += KG) {                  // further rounds only if q > 16*KG
            load_vf(ks0);
            mul(ks0);
        }
        load_u(std::integral_constant<int, 0>{});                   // U of the first output block: in flight from here
        if (wave < b) {
            const bool has1 = wave + FWAVES < b;
            // zacc[jj][nt][e]: token 8*(e/4) + 4*kg + e%4, rank index nt*32 + l32
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int rho = nt * 32 + l32;
                if (rho < r) {
                    // The four 8-byte units of a token's 32 bytes (4 blocks each) are stored XOR 2 for tokens
                    // 8..15 of every 16: the 32 lanes that phase 2 serves per clock (16 tokens x 2 units)
                    // then touch all 64 banks once instead of half of them twice.
                    unsigned char* zrow = Zs + rho * FZSTR + (4 * kg) * 32 + (wave & 1) * 4;
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        *(uint32_t*)(zrow + (8 * (e / 4) + (e % 4)) * 32 + ((wave >> 1) ^ (2 * ((e / 4) & 1))) * 8) =
                            pack2_bf16(zacc[0][nt][e], has1 ? zacc[1][nt][e] : 0.f);
                }
            }
        }
    }
    __syncthreads();

    // ---- phase 2: one wavefront per group of 8 rank indices
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
        if (wave + cc * FWAVES >= nchunks) continue;                // uniform; no global loads inside
        unsigned char* chunk = Zs + cw[cc] * FCHUNK;
        f32x4 d[2][8];
        s16x4 a[8][2];                                             // all 16 fragment reads in flight before the first MFMA
#pragma unroll
        for (int ri = 0; ri < 8; ++ri)
#pragma unroll
            for (int tg = 0; tg < 2; ++tg) a[ri][tg] = *(const s16x4*)(chunk + ri * FZSTR + (tg * 16 + ci) * 32 + (cg ^ (2 * (ci >> 3))) * 8);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ri = 0; ri < 8; ++ri)
#pragma unroll
            for (int tg = 0; tg < 2; ++tg)
                d[tg][ri] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[ri][tg], sfr[cc][ri], f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        // every read of this chunk has been issued by this wavefront before the writes below, and
        // LDS operations of one wavefront complete in order; d[tg][ri][e]: token tg*16 + 4*cg + e, block ci
#pragma unroll
        for (int tg = 0; tg < 2; ++tg)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int tok = tg * 16 + 4 * cg + e;
                *(uint4*)(chunk + (ci * FT + (tok ^ ci)) * 16) =
                    make_uint4(pack2_bf16(d[tg][0][e], d[tg][1][e]), pack2_bf16(d[tg][2][e], d[tg][3][e]),
                               pack2_bf16(d[tg][4][e], d[tg][5][e]), pack2_bf16(d[tg][6][e], d[tg][7][e]));
            }
    }
    load_u(std::integral_constant<int, 1>{});                       // U of the second output block
    __syncthreads();

    // ---- phase 3: this wavefront's output blocks i = wave, wave + 8
    static_for<2>([&](auto II) {
        constexpr int ii = decltype(II)::value;
        const int i = wave + ii * FWAVES;
        if (i >= b) return;                                         // uniform; no global loads inside
        const int ic = i;
        // the A fragments depend on the k-step only: read them all first, then run every MFMA on them
        bf16x8 a0[NT], a1[NT];
#pragma unroll
        for (int ks = 0; ks < NT; ++ks) {
            int c = ks * 4 + cg;                                    // group of 8 rank indices this lane multiplies
            if (c > nchunks - 1) c = nchunks - 1;                   // past r the U fragment is zero; read a valid group
            const unsigned char* chunk = Zs + c * FCHUNK;
            a0[ks] = *(const bf16x8*)(chunk + (ic * FT + (ci ^ (ic & 15))) * 16);
            a1[ks] = *(const bf16x8*)(chunk + (ic * FT + ((16 + ci) ^ (ic & 15))) * 16);
        }
#pragma unroll
        for (int nt = 0; nt < NPT; ++nt) {
            f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < NT; ++ks) {
                acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const bf16x8*)&ufr[ii][nt][ks], a0[ks], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const bf16x8*)&ufr[ii][nt][ks], a1[ks], acc1, 0, 0, 0);
            }
            // U is the first operand, so acc[e] is output feature i*p + nt*16 + 4*cg + e of token
            // (mt*16) + ci: four consecutive features per lane, one 8-byte LDS write each
            unsigned char* ydst = XY + ci * ystr + (i * p + nt * 16 + 4 * cg) * 2;
            *(uint2*)ydst = make_uint2(pack2_bf16(acc0[0], acc0[1]), pack2_bf16(acc0[2], acc0[3]));
            *(uint2*)(ydst + 16 * ystr) = make_uint2(pack2_bf16(acc1[0], acc1[1]), pack2_bf16(acc1[2], acc1[3]));
        }
    });
    __syncthreads();

    // ---- coalesced copy of the staged output tile: a wavefront writes 4 token rows, 1 KiB per store;
    // all LDS reads first, then the stores
    {
        const int cpr = n_out >> 3;                                  // 16-byte pieces per row
        uint4 yv[FT / FWAVES][XH];                                  // n_out <= 1024: at most 2 x 64 pieces per row
#pragma unroll
        for (int u = 0; u < FT / FWAVES; ++u)
#pragma unroll
            for (int h = 0; h < XH; ++h) {
                const int cc = h * 64 + lane < cpr ? h * 64 + lane : cpr - 1;
                yv[u][h] = *(const uint4*)(XY + (wave * (FT / FWAVES) + u) * ystr + cc * 16);
            }
#pragma unroll
        for (int u = 0; u < FT / FWAVES; ++u) {
            const int row = wave * (FT / FWAVES) + u;
            unsigned char* dst = (unsigned char*)(Y + (t0 + row) * n_out);
            if (t0 + row < T)                                        // uniform
#pragma unroll
                for (int h = 0; h < XH; ++h) {
                    const int cc = h * 64 + lane < cpr ? h * 64 + lane : cpr - 1;
                    *(uint4*)(dst + cc * 16) = yv[u][h];
                }
        }
    }
}

inline int full_fusion_lds_bytes(int n_in, int n_out, int r) {
    const int nt = (r + 31) / 32;
    const int wide = n_in > n_out ? n_in : n_out;
    return nt * 4 * FCHUNK + FT * (wide * 2 + 16);
}

}  // namespace

bool blast_full_fusion_shape_ok(int n_in, int n_out, int b, int r) {
    if (b <= 0 || b > 16 || n_in <= 0 || n_out <= 0 || r <= 0 || n_in % b || n_out % b) return false;
    const int q = n_in / b, p = n_out / b;
    if (q % 8 || r % 8 || p % 16 || p > 64 || r > 128 || n_in > 2048) return false;   // (rows are moved in at most 4 x 64 pieces)
    return full_fusion_lds_bytes(n_in, n_out, r) <= 160 * 1024;
}

bool blast_full_fusion_supported(int64_t T, int n_in, int n_out, int b, int r) {
    return T > 0 && (T + FT - 1) / FT < (1ll << 30) && blast_full_fusion_shape_ok(n_in, n_out, b, r);
}

size_t blast_vf_bytes(int n_in, int b, int r) {
    return (size_t)b * ((r + 31) / 32) * ((n_in / b + 15) / 16) * 1024;
}

size_t blast_uf_bytes(int n_out, int b, int r) {
    return (size_t)b * (n_out / b / 16) * ((r + 31) / 32) * 1024;
}

template <int NT, int KG, int NPT>
static hipError_t launch_full_inst(const void* X, const void* Sp, const void* Vf, const void* Uf, void* Y,
                                   int64_t T, int n_in, int n_out, int b, int r, hipStream_t s) {
    static LdsLimitOnce lds_limit;
    const int lds = full_fusion_lds_bytes(n_in, n_out, r);
    auto kern = blast_full_kernel<NT, KG, NPT>;
    if (hipError_t e = lds_limit.set({(const void*)kern}, 160 * 1024); e != hipSuccess) return e;
    const unsigned nblk = (unsigned)((T + FT - 1) / FT);
    hipLaunchKernelGGL(kern, dim3(nblk), dim3(FTHREADS), lds, s, (const bf16_t*)X, (const bf16_t*)Sp,
                       (const bf16_t*)Vf, (const bf16_t*)Uf, (bf16_t*)Y, T, n_in, n_out, b, r);
    return hipGetLastError();
}

// KG (k-steps fetched per round) is fixed per NT so that the fragment arrays stay in registers
template <int NT>
static hipError_t launch_full_nt(const void* X, const void* Sp, const void* Vf, const void* Uf, void* Y,
                                 int64_t T, int n_in, int n_out, int b, int r, hipStream_t s) {
    constexpr int KG = NT <= 2 ? 4 : (NT == 3 ? 3 : 1);
    switch (n_out / b / 16) {
        case 1: return launch_full_inst<NT, KG, 1>(X, Sp, Vf, Uf, Y, T, n_in, n_out, b, r, s);
        case 2: return launch_full_inst<NT, KG, 2>(X, Sp, Vf, Uf, Y, T, n_in, n_out, b, r, s);
        case 3: return launch_full_inst<NT, KG, 3>(X, Sp, Vf, Uf, Y, T, n_in, n_out, b, r, s);
        case 4: return launch_full_inst<NT, KG, 4>(X, Sp, Vf, Uf, Y, T, n_in, n_out, b, r, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_blast_full(const void* X, const void* Sp, const void* Vf, const void* Uf, void* Y,
                             int64_t T, int n_in, int n_out, int b, int r, hipStream_t s) {
    switch ((r + 31) / 32) {
        case 1: return launch_full_nt<1>(X, Sp, Vf, Uf, Y, T, n_in, n_out, b, r, s);
        case 2: return launch_full_nt<2>(X, Sp, Vf, Uf, Y, T, n_in, n_out, b, r, s);
        case 3: return launch_full_nt<3>(X, Sp, Vf, Uf, Y, T, n_in, n_out, b, r, s);
        case 4: return launch_full_nt<4>(X, Sp, Vf, Uf, Y, T, n_in, n_out, b, r, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace blr
