// bf16 MFMA batched "NT" GEMM for gfx950 with index maps on the B rows and the C columns.
//
// A workgroup of WGM x WGN wavefronts owns a BM x BN output tile; each wavefront owns
// (BM/WGM) x (BN/WGN) as a grid of 32x32 v_mfma_f32_32x32x16_bf16 tiles with fp32 accumulators.
// Operand tiles (both with the contraction index contiguous) stream global -> LDS directly
// (global_load_lds), one barrier per step. Three kernels share the layout conventions and the epilogue:
// gemm_wide_kernel (256 x 256 tile, steps of 64 contraction indices = whole cache lines per operand row, two
// stages), gemm_line_kernel (the smaller tiles in steps of 64 or 128, two to four stages) and gemm_dma_kernel
// (steps of 32, four stages: short contractions, split contraction index, problems that do not fill the chip).
// The weight tile is the FIRST MFMA operand: an accumulator lane then holds four consecutive
// output columns of one token, which go to an LDS copy of the C tile as 8-byte writes and from
// there to global memory as 16-byte row-contiguous stores (or element-wise through the column map
// when the map scatters).
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin over the 8 XCDs) owns a
// contiguous range of tiles, walked in groups of 8 row-tiles per column-tile, so the operand
// panels an XCD touches at one time fit its own L2.
#include "blr_common.h"
#include <cstdlib>

namespace blr {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;

// Tile and batch index of this workgroup. The grid is one-dimensional over all tiles of all batches;
// workgroup ids are remapped so that each XCD owns a contiguous range of logical ids. Three orders:
// 0, batch index SLOWEST: an XCD works on one batch (or a few) at a time, so the operand panels that
//    meet in its L2 are those of that batch only (with 4 batches and a few hundred tokens every XCD
//    used to fetch the whole activation matrix); within a batch, groups of 8 row tiles per column tile.
//    For operands that stay in the caches.
// 2, groups of 8 row tiles with ALL batches of the group together: the batches of every BLR product
//    interleave inside the rows of the A operand (X[T][b][p], Z'[T][b][r], A[T][b][r]), so this order
//    streams whole rows of a large A from HBM, where order 0 picks one batch's slice out of every row
//    (stage 3 of BLAST with 16 blocks at 8192 tokens: 96 us against 139 us).
// 1, batch index FASTEST, for scattering column maps: the G workgroups that interleave their columns
//    into the same cache lines run side by side on one XCD and their partial-line writes merge in its L2.
__device__ inline void workgroup_tile(const GemmDesc& d, int tiles_m, int tiles_n, int order, int& g, int& tile_m, int& tile_n) {
    // row tiles per column tile in a group: 8; 2 in the batch-fastest order, where the G batches of a tile already
    // multiply the panels that meet in an L2 (4 batches: 2 rows x 4 columns x 4 batches = 24 panels per 32
    // workgroups instead of 36; stage 2 of the 4096 -> 11008 layer at 8192 tokens 246 -> 238 us)
    const int GM = order == 1 ? 2 : 8;
    const int per_batch = tiles_m * tiles_n;
    const int lg = xcd_contiguous(blockIdx.x, per_batch * d.G);
    const int group_size = GM * tiles_n;                // tiles of one batch in a group of GM row tiles
    int first_m, in_group;
    if (order == 1) {                                   // batch index fastest
        g = lg % d.G;
        const int logical = lg / d.G;
        first_m = (logical / group_size) * GM;
        in_group = logical % group_size;
    } else if (order == 2) {                            // groups of row tiles, all batches of a group together
        const int rg = lg / (group_size * d.G);         // (only the last group may have fewer than GM row tiles)
        first_m = rg * GM;
        const int gm_here = tiles_m - first_m < GM ? tiles_m - first_m : GM;
        const int rest = lg - rg * group_size * d.G;
        g = rest / (gm_here * tiles_n);
        in_group = rest - g * gm_here * tiles_n;
    } else {                                            // batch index slowest
        g = lg / per_batch;
        const int logical = lg - g * per_batch;
        first_m = (logical / group_size) * GM;
        in_group = logical % group_size;
    }
    const int gm = tiles_m - first_m < GM ? tiles_m - first_m : GM;
    tile_m = first_m + in_group % gm;
    tile_n = in_group / gm;
}

// Epilogue: accumulators -> bf16 C tile in LDS -> global memory. With the weight fragment as first
// MFMA operand, accumulator element e of tile (i, j) is output column j*32 + 8*(e/4) + 4*(lane/32) + e%4
// of token i*32 + lane%32: 8-byte LDS writes, then 16-byte row-contiguous stores (or element-wise
// through the column map when the map scatters). Must be entered after a barrier that follows the
// last read of the operand stages, which the C tile overwrites.
template <int BM, int BN, int WTM, int WTN, int MI, int NI, int CSTR, int THREADS>
__device__ __forceinline__ void store_c_tile(const GemmDesc& d, const f32x16 (&acc)[MI][NI], unsigned char* Cs,
                                             int64_t m0, int n0, int g, int wm, int wn, int cvec) {
    const int tid = threadIdx.x, lane = tid & 63;
    {
        const int mrow = wm * WTM + (lane & 31);
        const int ncol = wn * WTN + 4 * (lane >> 5);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *(uint2*)(Cs + (mrow + i * 32) * CSTR + (ncol + j * 32 + 8 * q4) * 2) =
                        make_uint2(pack2_bf16(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1]),
                                   pack2_bf16(acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]));
    }
    __syncthreads();
    // A thread's column (group of 8 columns) is the same in every sweep of the workgroup over the
    // rows, so the column map (two integer divisions) is evaluated once per thread, not per element.
    // The sweeps go in batches: all LDS reads of a batch are issued, then its stores, so that the LDS
    // latency is paid once per batch and not once per store.
    bf16_t* Cp = (bf16_t*)d.C;
    if (cvec) {
        // groups of 8 consecutive columns map to 8 consecutive, 16-byte aligned elements of C
        constexpr int CPRC = BN / 8;
        static_assert(THREADS % CPRC == 0, "a thread keeps its column group");
        constexpr int RPS = THREADS / CPRC, SWEEPS = BM / RPS, UB = SWEEPS < 8 ? SWEEPS : 8;
        static_assert(BM % RPS == 0 && SWEEPS % UB == 0, "whole sweeps, whole batches");
        const int cc = tid % CPRC, row0 = tid / CPRC;
        const int n = n0 + cc * 8;
        if (n < d.N) {
            const int64_t col = (int64_t)g * d.c_gs + (int64_t)(n / d.c_div) * d.c_hi + (int64_t)(n % d.c_div) * d.c_lo;
            const unsigned char* src = Cs + row0 * CSTR + cc * 16;
            bf16_t* dst = Cp + (m0 + row0) * d.c_rs + col;
            const int64_t rows_left = d.M - m0 - row0;   // rows of this thread's first sweep and below that exist
#pragma unroll
            for (int s0 = 0; s0 < SWEEPS; s0 += UB) {
                u32x4 v[UB];                            // (a native vector type: arrays of HIP's uint4 struct stay in scratch memory)
#pragma unroll
                for (int u = 0; u < UB; ++u) v[u] = *(const u32x4*)(src + (s0 + u) * (RPS * CSTR));
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < UB; ++u)
                    if ((int64_t)(s0 + u) * RPS < rows_left) *(u32x4*)(dst + (int64_t)(s0 + u) * RPS * d.c_rs) = v[u];
            }
        }
    } else {
        static_assert(THREADS % BN == 0, "a thread keeps its column");
        constexpr int RPS = THREADS / BN, SWEEPS = BM / RPS, UB = SWEEPS < 16 ? SWEEPS : 16;
        static_assert(BM % RPS == 0 && SWEEPS % UB == 0, "whole sweeps, whole batches");
        const int nn = tid % BN, row0 = tid / BN;
        const int n = n0 + nn;
        if (n < d.N) {
            const int64_t col = (int64_t)g * d.c_gs + (int64_t)(n / d.c_div) * d.c_hi + (int64_t)(n % d.c_div) * d.c_lo;
            const unsigned char* src = Cs + row0 * CSTR + nn * 2;
            bf16_t* dst = Cp + (m0 + row0) * d.c_rs + col;
            const int64_t rows_left = d.M - m0 - row0;
#pragma unroll
            for (int s0 = 0; s0 < SWEEPS; s0 += UB) {
                bf16_t v[UB];
#pragma unroll
                for (int u = 0; u < UB; ++u) v[u] = *(const bf16_t*)(src + (s0 + u) * (RPS * CSTR));
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < UB; ++u)
                    if ((int64_t)(s0 + u) * RPS < rows_left) dst[(int64_t)(s0 + u) * RPS * d.c_rs] = v[u];
            }
        }
    }
}

// The same epilogue with C stored as 8-bit floats (E4M3, the intermediate of a quantised-intermediate
// execution): a lane's four consecutive columns become one 32-bit word (two v_cvt_pk_fp8_f32 after a
// clamp to the format's largest finite value, 448), the tile goes through LDS with rows of BN + 16
// bytes, and leaves as 16-byte stores of 16 consecutive columns. Column map: contiguous (host-checked).
template <int BM, int BN, int WTM, int WTN, int MI, int NI, int THREADS>
__device__ __forceinline__ void store_c_tile_fp8(const GemmDesc& d, const f32x16 (&acc)[MI][NI], unsigned char* Cs,
                                                 int64_t m0, int n0, int g, int wm, int wn) {
    constexpr int CSTR8 = BN + 16;
    const int tid = threadIdx.x, lane = tid & 63;
    auto q8 = [](float x) { return __builtin_amdgcn_fmed3f(x, -448.f, 448.f); };
    {
        const int mrow = wm * WTM + (lane & 31);
        const int ncol = wn * WTN + 4 * (lane >> 5);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    int w = __builtin_amdgcn_cvt_pk_fp8_f32(q8(acc[i][j][4 * q4]), q8(acc[i][j][4 * q4 + 1]), 0, false);
                    w = __builtin_amdgcn_cvt_pk_fp8_f32(q8(acc[i][j][4 * q4 + 2]), q8(acc[i][j][4 * q4 + 3]), w, true);
                    *(int*)(Cs + (mrow + i * 32) * CSTR8 + (ncol + j * 32 + 8 * q4)) = w;
                }
    }
    __syncthreads();
    constexpr int CPRC = BN / 16;                       // groups of 16 columns per row
    static_assert(THREADS % CPRC == 0, "a thread keeps its column group");
    constexpr int RPS = THREADS / CPRC, SWEEPS = BM / RPS;
    static_assert(BM % RPS == 0, "whole sweeps");
    const int cc = tid % CPRC, row0 = tid / CPRC;
    const int n = n0 + cc * 16;
    if (n >= d.N) return;
    unsigned char* dst = (unsigned char*)d.C + (m0 + row0) * d.c_rs + (int64_t)g * d.c_gs + n;
    const unsigned char* src = Cs + row0 * CSTR8 + cc * 16;
    const int64_t rows_left = d.M - m0 - row0;
#pragma unroll
    for (int s0 = 0; s0 < SWEEPS; ++s0)
        if ((int64_t)s0 * RPS < rows_left) *(u32x4*)(dst + (int64_t)s0 * RPS * d.c_rs) = *(const u32x4*)(src + s0 * (RPS * CSTR8));
}

// ---------------------------------------------------------------------------------------------
// Operand tiles stream global -> LDS directly (global_load_lds): no staging registers and no LDS
// store instructions, so the prefetch depth is set by LDS capacity (NS stages of BK = 32) instead of
// by the register file. A stage holds BM A rows and BN B rows of 64 bytes = four
// 16-byte pieces; a direct load lands lane l at base + 16 l, so rows cannot be padded and the pieces
// are XOR-swizzled instead: piece c of row w sits in slot c ^ ((w >> 2) & 3), which puts the 16
// rows that a ds_read_b128 serves per clock into 16 different 16-byte columns of the 64 banks.
// Loads for step s + PD are issued when step s has been consumed and vmcnt counts them, so one wait
// and one barrier per step is all the synchronisation. The fragment reads are inline assembly with their own
// lgkmcnt waits: LDS reads that the compiler can see make it wait for ALL outstanding direct loads.
// 16 zero bytes in global memory: the source of operand pieces that lie past K
__device__ __attribute__((aligned(16))) const unsigned char zero_piece[16] = {0};

// asynchronous 16-byte LDS read the compiler does not see as a memory access; the caller waits on
// lgkmcnt itself and ties the result to that wait before using it
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}

template <int BM, int BN, int WGM, int WGN, int NSTAGES>
struct DmaCfg {
    static constexpr int BK = 32, NS = NSTAGES, PD = NS;   // stages in LDS = steps of loads in flight
    static constexpr int WAVES = WGM * WGN, THREADS = 64 * WAVES;
    static constexpr int ROWS = BM + BN;
    static constexpr int STAGE = ROWS * BK * 2;
    static constexpr int LPW = ROWS / 16 / WAVES;    // direct loads (16 rows each) per wavefront and stage
    static constexpr int CSTR = BN * 2 + 16;
    static constexpr int C_BYTES = BM * CSTR;
    static constexpr int LDS_BYTES = NS * STAGE > C_BYTES ? NS * STAGE : C_BYTES;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int MI = WTM / 32, NI = WTN / 32;
    static_assert(ROWS % (16 * WAVES) == 0 && BM % 16 == 0, "whole direct loads per wavefront, none straddling A and B");
    static_assert(PD >= 2 && MI >= 1 && NI >= 1 && LPW * (PD - 1) < 64, "tile / vmcnt range");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert((MI * 32 - 32) * 64 < 65536 && (NI * 32 - 32) * 64 < 65536, "fragment offsets are ds_read immediates");
};

// TAIL: K is not a multiple of 32, the last step is partial
template <int BM, int BN, int WGM, int WGN, int NS, bool TAIL>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_dma_kernel(GemmDesc d, int tiles_m, int tiles_n, int cvec, int order, int kspan) {
    using C = DmaCfg<BM, BN, WGM, WGN, NS>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    int g, tile_m, tile_n;
    workgroup_tile(d, tiles_m, tiles_n, order, g, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;
    // Split contraction: workgroup z of a tile covers k steps [z kspan, (z+1) kspan) and leaves its fp32
    // accumulators in the scratch buffer; a second kernel adds the parts in a fixed order.
    const int kb = blockIdx.z * kspan * C::BK;         // first contraction index of this workgroup
    const int Kloc = d.K - kb < kspan * C::BK ? d.K - kb : kspan * C::BK;
    const unsigned char* Abase = (const unsigned char*)((const bf16_t*)d.A + (int64_t)g * d.a_gs + m0 * d.a_rs);
    const unsigned char* Bbase = (const unsigned char*)((const bf16_t*)d.B + (int64_t)g * d.b_gs + kb);

    // Direct load h of this wavefront fills stage rows 16 (LPW wave + h) .. + 15 (A rows first, then B
    // rows): lane l brings the piece that belongs at row l / 4 of those, slot l % 4. Offsets are bytes
    // from Abase / Bbase (the launcher checks that they fit 32 bits).
    unsigned off[C::LPW];
    bool bad[C::LPW];
    const int nk = (Kloc + C::BK - 1) / C::BK;
#pragma unroll
    for (int h = 0; h < C::LPW; ++h) {
        const int row = 16 * (C::LPW * wave + h) + (lane >> 2);
        const int piece = (lane & 3) ^ ((row >> 2) & 3);
        if (row < BM) {
            int64_t m = row;
            if (m0 + m > d.M - 1) m = d.M - 1 - m0;     // rows past the end re-read the last row; never stored
            off[h] = (unsigned)((m * d.a_rs + piece * 8) * 2);
        } else {
            int n = n0 + row - BM;
            if (n > d.N - 1) n = d.N - 1;
            const int64_t nr = d.b_div ? (int64_t)(n % d.b_div) * d.b_mul + n / d.b_div : n;
            off[h] = (unsigned)((nr * d.b_rs + piece * 8) * 2);
        }
        bad[h] = TAIL && (nk - 1) * C::BK + piece * 8 >= Kloc;   // in the last step this piece lies past K
    }
    int kf = 0;                                         // fetch cursor (uniform); stops at the last step
    // byte offset of the cursor's k range inside an A row: k itself, or, with a segmented contraction
    // index, the segment's start plus the position inside the segment (a step never straddles segments)
    int a_pos = d.a_seg ? kb % d.a_seg : 0;
    int64_t a_koff = d.a_seg ? ((int64_t)(kb / d.a_seg) * d.a_seg_stride + a_pos) * 2 : (int64_t)kb * 2;
    // loads H0 .. H1-1 of the step under the cursor; advance = this completes the step's loads
    auto issue = [&](int stage_off, auto H0, auto H1, bool advance) {
        const bool lastk = TAIL && kf == nk - 1;
#pragma unroll
        for (int h = decltype(H0)::value; h < decltype(H1)::value; ++h) {
            const bool isa = 16 * (C::LPW * wave + h) < BM;                 // uniform
            asm volatile("" : "+v"(off[h]));                                // keeps the offset a register operand: scalar base + lane offset addressing, no address arithmetic
            const unsigned char* p = (isa ? Abase + a_koff : Bbase + (size_t)kf * (C::BK * 2)) + off[h];
            if (TAIL) p = (lastk && bad[h]) ? zero_piece : p;
            __builtin_amdgcn_global_load_lds(BLR_GPTR(p), BLR_LPTR(smem + stage_off + (C::LPW * wave + h) * 1024), 16, 0, 0);
        }
        if (advance && kf < nk - 1) {
            ++kf;
            a_koff += C::BK * 2;
            if (d.a_seg) {
                a_pos += C::BK;
                if (a_pos == d.a_seg) { a_pos = 0; a_koff += (d.a_seg_stride - d.a_seg) * 2; }
            }
        }
    };
    constexpr std::integral_constant<int, 0> L0{};
    constexpr std::integral_constant<int, (C::LPW + 1) / 2> LH{};
    constexpr std::integral_constant<int, C::LPW> LN{};

    // fragment addresses inside a stage: row m of a 32-row MFMA operand, k group kg, k16 step ks
    const int m = lane & 31, kg = lane >> 5;
    const unsigned lds0 = (unsigned)(uintptr_t)BLR_LPTR(smem);
    unsigned fa[2], fb[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const unsigned sw = (unsigned)(((2 * ks + kg) ^ ((m >> 2) & 3)) * 16);
        fa[ks] = lds0 + (wm * C::WTM + m) * (C::BK * 2) + sw;
        fb[ks] = lds0 + (BM + wn * C::WTN + m) * (C::BK * 2) + sw;
    }

    f32x16 acc[C::MI][C::NI];
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // Software pipeline inside every wavefront: the fragment reads of one half step (k16 step) are in
    // flight while the MFMAs of the previous half step run, so the LDS and the matrix cores overlap even
    // though the barrier keeps all wavefronts of the workgroup in phase.
    bf16x8 af[2][C::MI], bfr[2][C::NI];
    auto read_frags = [&](auto KS, int stage_off) {
        constexpr int ks = decltype(KS)::value;
        const unsigned aa = fa[ks] + stage_off, ab = fb[ks] + stage_off;
        static_for<C::MI>([&](auto I) { af[ks][decltype(I)::value] = lds_read_b128<decltype(I)::value * 32 * C::BK * 2>(aa); });
        static_for<C::NI>([&](auto J) { bfr[ks][decltype(J)::value] = lds_read_b128<decltype(J)::value * 32 * C::BK * 2>(ab); });
    };
    auto mfma_half = [&](auto KS) {
        constexpr int ks = decltype(KS)::value;
        // tie the fragments to the preceding wait, so that no MFMA is scheduled above it
#pragma unroll
        for (int i = 0; i < C::MI; ++i) asm volatile("" : "+v"(af[ks][i]));
#pragma unroll
        for (int j = 0; j < C::NI; ++j) asm volatile("" : "+v"(bfr[ks][j]));
#pragma unroll
        for (int i = 0; i < C::MI; ++i)
#pragma unroll
            for (int j = 0; j < C::NI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks][j], af[ks][i], acc[i][j], 0, 0, 0);
    };
    constexpr std::integral_constant<int, 0> K0{};
    constexpr std::integral_constant<int, 1> K1{};

    for (int s = 0; s < C::PD; ++s) issue(s * C::STAGE, L0, LN, true);
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" :: "n"(C::LPW * (C::PD - 1)) : "memory");
    int cstage = 0, fstage = 0;                         // stage being computed on / stage freed at the last barrier
    read_frags(K0, cstage);
#pragma unroll 1
    for (int kt = 0; kt < nk; ++kt) {
        read_frags(K1, cstage);
        asm volatile("s_waitcnt lgkmcnt(%0)" :: "n"(C::MI + C::NI) : "memory");    // in-order: half step 0 has arrived
        __builtin_amdgcn_sched_barrier(0);              // keep the schedule as written: MFMAs between the waits
        __builtin_amdgcn_s_setprio(1);
        mfma_half(K0);
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        // The loads of step kt + PD - 1 go out in two halves, each behind a burst of MFMAs, so that their
        // issue (which can stall on a full queue) never delays the matrix pipe: second half here.
        if (kt > 0) issue(fstage, LH, LN, true);
        // all reads of this stage are done and the next stage has landed (own loads: vmcnt; others': barrier)
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" :: "n"(C::LPW * (C::PD - 2)) : "memory");
        fstage = cstage;                                // step kt + PD refills the stage just consumed
        cstage = cstage + C::STAGE == C::NS * C::STAGE ? 0 : cstage + C::STAGE;
        // Never leave a read without a consumer: the compiler sees its destination registers as dead and
        // reuses them, and the late LDS return would overwrite their new contents.
        if (kt + 1 < nk) read_frags(K0, cstage);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(1);
        mfma_half(K1);
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        issue(fstage, L0, LH, false);                   // first half of the loads of step kt + PD
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // the repeated loads of the last steps have landed too
    if (gridDim.z > 1) {                                // split contraction: fp32 partial tile, accumulator order
        const int64_t tile = ((int64_t)g * tiles_m + tile_m) * tiles_n + tile_n;
        float* P = d.split_scratch + ((int64_t)blockIdx.z * tiles_m * tiles_n * d.G + tile) * (BM * BN);
#pragma unroll
        for (int i = 0; i < C::MI; ++i)
#pragma unroll
            for (int j = 0; j < C::NI; ++j)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *(float4*)(P + ((((i * C::NI + j) * 4 + q4) * C::THREADS + tid) << 2)) =
                        make_float4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]);
        return;
    }
    __syncthreads();
    if (d.c_fp8) store_c_tile_fp8<BM, BN, C::WTM, C::WTN, C::MI, C::NI, C::THREADS>(d, acc, smem, m0, n0, g, wm, wn);
    else store_c_tile<BM, BN, C::WTM, C::WTN, C::MI, C::NI, C::CSTR, C::THREADS>(d, acc, smem, m0, n0, g, wm, wn, cvec);
}

// ---------------------------------------------------------------------------------------------
// Tiles in DEEP steps: BK = 64 or 128 contraction indices per barrier, i.e. operand rows of 128 or 256 bytes
// (whole cache lines per request; 16-byte pieces XOR-swizzled by the row so that the 16 rows a ds_read_b128
// serves per clock cover all 64 banks). Two kernels use this layout: gemm_wide_kernel (the 256 x 256 tile on two
// stages) and gemm_line_kernel (the smaller tiles on three or four stages). For calls with FEW tiles (some
// hundreds of tokens) every workgroup walks its contraction index alone on its compute unit, and a step of 32
// costs the same chain of latencies (barrier, LDS read, dependent MFMAs) whatever the tile does in between:
// about 600 clocks for 128 to 256 clocks of matrix work; deep steps pay the chain once per 4 to 8 times the work.
template <int BM, int BN, int WGM, int WGN, int BKT, int NSTAGES>
struct DeepCfg {
    static constexpr int BK = BKT, NS = NSTAGES;
    static constexpr int RB = BK * 2;                 // bytes of an operand row in LDS
    static constexpr int PPR = RB / 16;               // 16-byte pieces per row
    static constexpr int RPL = 1024 / RB;             // rows one direct load (64 lanes x 16 bytes) fills
    static constexpr int SH = BK == 128 ? 0 : BK == 64 ? 1 : 2;   // swizzle: piece ^ ((row >> SH) & (PPR - 1))
    static constexpr int KS = BK / 16;                // k16 steps per stage
    static constexpr int WAVES = WGM * WGN, THREADS = 64 * WAVES;
    static constexpr int ROWS = BM + BN;
    static constexpr int STAGE = ROWS * RB;
    static constexpr int LPW = ROWS / RPL / WAVES;    // direct loads per wavefront and stage
    static constexpr int CSTR = BN * 2 + 16;
    static constexpr int C_BYTES = BM * CSTR;
    static constexpr int LDS_BYTES = NS * STAGE > C_BYTES ? NS * STAGE : C_BYTES;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int MI = WTM / 32, NI = WTN / 32;
    static_assert(BK == 64 || BK == 128, "deep steps");
    static_assert(ROWS % (RPL * WAVES) == 0 && BM % RPL == 0, "whole direct loads per wavefront, none straddling A and B");
    static_assert(NS >= 2 && MI >= 1 && NI >= 1 && LPW * (NS - 1) < 64, "tile / vmcnt range");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert((MI * 32 - 32) * RB < 65536 && (NI * 32 - 32) * RB < 65536, "fragment offsets are ds_read immediates");
};

// Direct load h of this wavefront fills stage rows RPL (LPW wave + h) .. + RPL - 1 (A rows first, then
// B rows): lane l brings the piece that belongs in slot l % PPR of row l / PPR of those. Offsets are
// bytes from Abase / Bbase; the launcher checks that they fit 32 bits, so the arithmetic is 32-bit.
template <class C, int BM, bool TAIL>
__device__ __forceinline__ void deep_load_offsets(const GemmDesc& d, int wave, int lane, int64_t m0, int n0, int nk,
                                                  unsigned (&off)[C::LPW], bool (&bad)[C::LPW]) {
    const int lrow = lane / C::PPR, slot = lane % C::PPR;
    const int rows_m = d.M - m0 < BM ? (int)(d.M - m0) : BM;      // rows of this tile that exist
    // B rows: n = n0 + row - BM walks upwards by RPL per load; its image under the row gather is kept as
    // (remainder, quotient) and advanced without divisions
    int bn = n0 + C::RPL * (C::LPW * wave) + lrow - BM;            // (negative while this wavefront is still on A rows)
    int brem = 0, bquo = 0;
    bool bstarted = false;
#pragma unroll
    for (int h = 0; h < C::LPW; ++h) {
        const int row = C::RPL * (C::LPW * wave + h) + lrow;
        const int piece = slot ^ ((row >> C::SH) & (C::PPR - 1));
        if (C::RPL * (C::LPW * wave + h) < BM) {                   // uniform
            const int mr = row < rows_m ? row : rows_m - 1;        // rows past the end re-read the last row; never stored
            off[h] = ((unsigned)mr * (unsigned)d.a_rs + (unsigned)piece * 8u) * 2u;
        } else {
            int n = bn + C::RPL * h;
            if (n > d.N - 1) n = d.N - 1;
            unsigned nr = (unsigned)n;
            if (d.b_div) {
                if (!bstarted || n == d.N - 1) { brem = n % d.b_div; bquo = n / d.b_div; bstarted = true; }
                nr = (unsigned)brem * (unsigned)d.b_mul + (unsigned)bquo;
                brem += C::RPL;
                while (brem >= d.b_div) { brem -= d.b_div; ++bquo; }
            }
            off[h] = (nr * (unsigned)d.b_rs + (unsigned)piece * 8u) * 2u;
        }
        bad[h] = TAIL && (nk - 1) * C::BK + piece * 8 >= d.K;       // in the last step this piece lies past K
    }
}

// ---------------------------------------------------------------------------------------------
// The 256 x 256 tile in steps of 64 contraction indices. The L2 serves one request per channel and clock whether
// it asks for 64 or for 128 bytes of a line (measured: 260 G requests/s over the chip either way), so the 32-deep
// steps of gemm_dma_kernel, whose operand rows are half lines, cap the operand stream at 16.7 TB/s, which is what
// the large tile needs at the matrix pipes' full rate. Whole lines need 64 KB per stage and LDS holds two:
// the refill of the stage that was computed on in step s - 1 goes out at the START of step s, one load behind each
// of the first MFMAs, and has the rest of the step to land; the wait for it and the step's one barrier sit in the
// MIDDLE of the last MFMA burst, followed by the first fragment reads of the next stage, so that neither the
// barrier nor the LDS latency after it meets an empty matrix pipe. The two wavefronts of a SIMD drift apart
// (one runs MFMAs while the other issues memory instructions), and a wavefront's VALU instructions barely issue
// while its sibling keeps the matrix pipe full (measured: an address add per load made the load phase three times
// longer): the loop body therefore has NO vector ALU work besides the MFMAs - loads address as scalar base +
// a fixed 32-bit lane offset, fragment reads use addresses computed once per stage and k16 step.
template <bool TAIL>
__global__ __launch_bounds__(512) void gemm_wide_kernel(GemmDesc d, int tiles_m, int tiles_n, int cvec, int order) {
    constexpr int BM = 256, BN = 256, WGN = 4;
    using C = DeepCfg<BM, BN, 2, WGN, 64, 2>;
    static_assert(C::LPW <= C::MI * C::NI && BM % (C::RPL * C::LPW) == 0, "one load behind each MFMA of the first burst; a wavefront loads A rows or B rows");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    int g, tile_m, tile_n;
    workgroup_tile(d, tiles_m, tiles_n, order, g, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;
    const unsigned char* Abase = (const unsigned char*)((const bf16_t*)d.A + (int64_t)g * d.a_gs + m0 * d.a_rs);
    const unsigned char* Bbase = (const unsigned char*)((const bf16_t*)d.B + (int64_t)g * d.b_gs);
    const int nk = (d.K + C::BK - 1) / C::BK;
    unsigned off[C::LPW];
    bool bad[C::LPW];
    deep_load_offsets<C, BM, TAIL>(d, wave, lane, m0, n0, nk, off, bad);
    const bool on_a = C::RPL * C::LPW * wave < BM;      // this wavefront's loads bring A rows (uniform)

    int kf = 0;                                         // step under the fetch cursor (uniform)
    int a_pos = 0;                                      // position inside the current segment of a segmented contraction index
    int64_t a_koff = 0;
    const unsigned char* src = on_a ? Abase : Bbase;    // this wavefront's operand at the cursor
    auto issue = [&](int stage_off, auto H) {
        constexpr int h = decltype(H)::value;
        asm volatile("" : "+v"(off[h]));                // the 32-bit offset stays a register operand: scalar base + lane offset addressing, no address arithmetic
        if (TAIL && kf == nk - 1) {
            // A branch, not a select: only the fetch of the last step pays for the per-lane choice. (The non-temporal
            // hint does no harm there and keeps the compiler from merging the two loads into one with a selected address.)
            unsigned o = off[h];
            asm volatile("" : "+v"(o));                 // (its own copy: a common address would be computed ahead of the branch, in vector registers)
            __builtin_amdgcn_global_load_lds(BLR_GPTR(bad[h] ? zero_piece : src + o), BLR_LPTR(smem + stage_off + (C::LPW * wave + h) * 1024), 16, 0, 2);
        } else {
            __builtin_amdgcn_global_load_lds(BLR_GPTR(src + off[h]), BLR_LPTR(smem + stage_off + (C::LPW * wave + h) * 1024), 16, 0, 0);
        }
    };
    auto advance = [&] {                                // (stops at the last step, which the last steps fetch again: never needed, always in bounds)
        if (kf == nk - 1) return;
        ++kf;
        a_koff += C::RB;
        if (d.a_seg) {
            a_pos += C::BK;
            if (a_pos == d.a_seg) { a_pos = 0; a_koff += (d.a_seg_stride - d.a_seg) * 2; }
        }
        src = on_a ? Abase + a_koff : Bbase + (size_t)kf * C::RB;
    };

    // fragment addresses, one per stage and k16 step (row m of a 32-row MFMA operand, k group kg), opaque to the
    // compiler so that it keeps them instead of recomputing them in the loop
    const int m = lane & 31, kg = lane >> 5;
    const unsigned lds0 = (unsigned)(uintptr_t)BLR_LPTR(smem);
    const unsigned swz = (unsigned)((m >> C::SH) & (C::PPR - 1));
    unsigned fa[2][C::KS], fb[2][C::KS];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const unsigned sw = (((unsigned)(2 * ks + kg)) ^ swz) * 16u + st * C::STAGE;
            fa[st][ks] = lds0 + (wm * C::WTM + m) * C::RB + sw;
            fb[st][ks] = lds0 + (BM + wn * C::WTN + m) * C::RB + sw;
            asm volatile("" : "+v"(fa[st][ks]), "+v"(fb[st][ks]));
        }

    f32x16 acc[C::MI][C::NI];
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    bf16x8 af[2][C::MI], bfr[2][C::NI];                 // fragments of two k16 steps in rotation
    auto read_frags = [&](auto ST, auto KSC) {
        constexpr int st = decltype(ST)::value, ks = decltype(KSC)::value;
        static_for<C::MI>([&](auto I) { af[ks & 1][decltype(I)::value] = lds_read_b128<decltype(I)::value * 32 * C::RB>(fa[st][ks]); });
        static_for<C::NI>([&](auto J) { bfr[ks & 1][decltype(J)::value] = lds_read_b128<decltype(J)::value * 32 * C::RB>(fb[st][ks]); });
    };
    // one step on stage ST
    auto step = [&](auto ST) {
        constexpr int st = decltype(ST)::value;
        static_for<C::KS>([&](auto KSC) {
            constexpr int ks = decltype(KSC)::value, b = ks & 1;
            if constexpr (ks + 1 < C::KS) {
                read_frags(ST, std::integral_constant<int, ks + 1>{});
                asm volatile("s_waitcnt lgkmcnt(%0)" :: "n"(C::MI + C::NI) : "memory");   // in order: k16 step ks has arrived
            } else {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < C::MI; ++i) asm volatile("" : "+v"(af[b][i]));         // tie the fragments to the preceding wait
#pragma unroll
            for (int j = 0; j < C::NI; ++j) asm volatile("" : "+v"(bfr[b][j]));
            static_for<C::MI * C::NI>([&](auto Q) {
                constexpr int q = decltype(Q)::value, i = q / C::NI, j = q % C::NI;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[b][j], af[b][i], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (ks == 0 && q < C::LPW) {
                    issue((1 - st) * C::STAGE, std::integral_constant<int, q>{});
                    if constexpr (q == C::LPW - 1) advance();
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (ks == C::KS - 1 && q == C::MI * C::NI / 2 - 1) {
                    // every wavefront is past its last read of this stage; the other stage has landed (own loads: vmcnt; the others': barrier)
                    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
                    read_frags(std::integral_constant<int, 1 - st>{}, std::integral_constant<int, 0>{});
                    __builtin_amdgcn_sched_barrier(0);
                }
            });
        });
    };

    static_for<C::LPW>([&](auto H) { issue(0, H); });
    advance();
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    read_frags(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
#pragma unroll 1
    for (int kt = 0; kt + 1 < nk; kt += 2) {            // (stages alternate: two steps per trip keep them compile-time constants)
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
    }
    if (nk & 1) step(std::integral_constant<int, 0>{});
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the fragments read ahead behind the last step are not used
#pragma unroll
    for (int i = 0; i < C::MI; ++i) asm volatile("" :: "v"(af[0][i]));     // (their registers stay theirs until they have arrived)
#pragma unroll
    for (int j = 0; j < C::NI; ++j) asm volatile("" :: "v"(bfr[0][j]));
    __syncthreads();
    if (d.c_fp8) store_c_tile_fp8<BM, BN, C::WTM, C::WTN, C::MI, C::NI, C::THREADS>(d, acc, smem, m0, n0, g, wm, wn);
    else store_c_tile<BM, BN, C::WTM, C::WTN, C::MI, C::NI, C::CSTR, C::THREADS>(d, acc, smem, m0, n0, g, wm, wn, cvec);
}

// ---------------------------------------------------------------------------------------------
// The schedule of gemm_wide_kernel for any tile of DeepCfg and 2 to 4 stages: the fragment reads of k16 step
// ks + 1 in flight while the MFMAs of step ks run, the direct loads of step s + NS - 1 behind the first MFMAs of
// step s, the barrier inside the last MFMA burst, no vector ALU work in the loop. The stages are interleaved in
// LDS in units of one direct load (1 KB: chunk c of stage st lies at (c NS + st) KB), so that the stage is part
// of the ds_read immediate and one set of fragment addresses (per k16 step) serves all stages; NS steps per loop
// trip keep the stage a compile-time constant. Against the same tiles with per-step address arithmetic and the
// barrier at the step's start: dense 4096 x 4096 at 128 / 512 / 2048 tokens 15.7 -> 13.9, 25.9 -> 24.2,
// 64.9 -> 61.2 us.
template <int BM, int BN, int WGM, int WGN, int BKT, int NS, bool TAIL>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_line_kernel(GemmDesc d, int tiles_m, int tiles_n, int cvec, int order) {
    using C = DeepCfg<BM, BN, WGM, WGN, BKT, NS>;
    constexpr int MFMAS = C::MI * C::NI, HALF = (MFMAS + 1) / 2;
    static_assert(C::LPW <= (C::KS - 1) * MFMAS + HALF, "the step's loads are out before its barrier");
    static_assert((C::MI * 32 - 32) * C::RB * NS + NS * 1024 < 65536 && (C::NI * 32 - 32) * C::RB * NS + NS * 1024 < 65536, "fragment offsets are ds_read immediates");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    int g, tile_m, tile_n;
    workgroup_tile(d, tiles_m, tiles_n, order, g, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;
    const unsigned char* Abase = (const unsigned char*)((const bf16_t*)d.A + (int64_t)g * d.a_gs + m0 * d.a_rs);
    const unsigned char* Bbase = (const unsigned char*)((const bf16_t*)d.B + (int64_t)g * d.b_gs);
    const int nk = (d.K + C::BK - 1) / C::BK;
    unsigned off[C::LPW];
    bool bad[C::LPW];
    deep_load_offsets<C, BM, TAIL>(d, wave, lane, m0, n0, nk, off, bad);

    int kf = 0;                                         // step under the fetch cursor (uniform)
    int a_pos = 0;                                      // position inside the current segment of a segmented contraction index
    int64_t a_koff = 0;
    const unsigned char* asrc = Abase;                  // the operands at the cursor
    const unsigned char* bsrc = Bbase;
    auto issue = [&](auto ST, auto H) __attribute__((always_inline)) {                 // load h of the step under the cursor, into stage st
        constexpr int st = decltype(ST)::value, h = decltype(H)::value;
        const bool isa = C::RPL * (C::LPW * wave + h) < BM;               // uniform
        asm volatile("" : "+v"(off[h]));                // the 32-bit offset stays a register operand: scalar base + lane offset addressing, no address arithmetic
        const unsigned char* base = isa ? asrc : bsrc;
        if (TAIL && kf == nk - 1) {                     // (a branch, a different cache hint and its own copy of the offset, as in gemm_wide_kernel)
            unsigned o = off[h];
            asm volatile("" : "+v"(o));
            __builtin_amdgcn_global_load_lds(BLR_GPTR(bad[h] ? zero_piece : base + o), BLR_LPTR(smem + ((C::LPW * wave + h) * NS + st) * 1024), 16, 0, 2);
        } else {
            __builtin_amdgcn_global_load_lds(BLR_GPTR(base + off[h]), BLR_LPTR(smem + ((C::LPW * wave + h) * NS + st) * 1024), 16, 0, 0);
        }
    };
    auto advance = [&]() __attribute__((always_inline)) {                                // (stops at the last step, which the last steps fetch again: never needed, always in bounds)
        if (kf == nk - 1) return;
        ++kf;
        a_koff += C::RB;
        if (d.a_seg) {
            a_pos += C::BK;
            if (a_pos == d.a_seg) { a_pos = 0; a_koff += (d.a_seg_stride - d.a_seg) * 2; }
        }
        asrc = Abase + a_koff;
        bsrc = Bbase + (size_t)kf * C::RB;
    };

    // fragment addresses in stage 0, one per k16 step (row of a 32-row MFMA operand, k group kg), opaque to the
    // compiler so that it keeps them instead of recomputing them in the loop
    const int m = lane & 31, kg = lane >> 5;
    const unsigned lds0 = (unsigned)(uintptr_t)BLR_LPTR(smem);
    const unsigned swz = (unsigned)((m >> C::SH) & (C::PPR - 1));
    unsigned fa[C::KS], fb[C::KS];
    {
        const int ra = wm * C::WTM + m, rb = BM + wn * C::WTN + m;       // stage rows
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const unsigned sw = (((unsigned)(2 * ks + kg)) ^ swz) * 16u;
            fa[ks] = lds0 + (ra / C::RPL) * (NS * 1024) + (ra % C::RPL) * C::RB + sw;
            fb[ks] = lds0 + (rb / C::RPL) * (NS * 1024) + (rb % C::RPL) * C::RB + sw;
            asm volatile("" : "+v"(fa[ks]), "+v"(fb[ks]));
        }
    }

    f32x16 acc[C::MI][C::NI];
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    bf16x8 af[2][C::MI], bfr[2][C::NI];                 // fragments of two k16 steps in rotation
    auto read_frags = [&](auto ST, auto KSC) __attribute__((always_inline)) {
        constexpr int st = decltype(ST)::value, ks = decltype(KSC)::value;
        static_for<C::MI>([&](auto I) { af[ks & 1][decltype(I)::value] = lds_read_b128<decltype(I)::value * 32 * C::RB * NS + st * 1024>(fa[ks]); });
        static_for<C::NI>([&](auto J) { bfr[ks & 1][decltype(J)::value] = lds_read_b128<decltype(J)::value * 32 * C::RB * NS + st * 1024>(fb[ks]); });
    };
    // one step on stage ST: fetches the step NS - 1 ahead into the stage that was computed on one step ago
    auto step = [&](auto ST) __attribute__((always_inline)) {
        constexpr int st = decltype(ST)::value;
        static_for<C::KS>([&](auto KSC) {
            constexpr int ks = decltype(KSC)::value, b = ks & 1;
            if constexpr (ks + 1 < C::KS) {
                read_frags(ST, std::integral_constant<int, ks + 1>{});
                asm volatile("s_waitcnt lgkmcnt(%0)" :: "n"(C::MI + C::NI) : "memory");   // in order: k16 step ks has arrived
            } else {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < C::MI; ++i) asm volatile("" : "+v"(af[b][i]));         // tie the fragments to the preceding wait
#pragma unroll
            for (int j = 0; j < C::NI; ++j) asm volatile("" : "+v"(bfr[b][j]));
            static_for<MFMAS>([&](auto Q) {
                constexpr int q = decltype(Q)::value, i = q / C::NI, j = q % C::NI, n = ks * MFMAS + q;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[b][j], af[b][i], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (n < C::LPW) {
                    issue(std::integral_constant<int, (st + NS - 1) % NS>{}, std::integral_constant<int, n>{});
                    if constexpr (n == C::LPW - 1) advance();
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (ks == C::KS - 1 && q == HALF - 1) {
                    // every wavefront is past its last read of this stage; the next stage has landed (own loads: vmcnt; the others': barrier)
                    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" :: "n"(C::LPW * (NS - 2)) : "memory");
                    read_frags(std::integral_constant<int, (st + 1) % NS>{}, std::integral_constant<int, 0>{});
                    __builtin_amdgcn_sched_barrier(0);
                }
            });
        });
    };

    static_for<NS - 1>([&](auto S) {
        static_for<C::LPW>([&](auto H) { issue(S, H); });
        advance();
    });
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" :: "n"(C::LPW * (NS - 2)) : "memory");
    read_frags(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    int kt = 0;
#pragma unroll 1
    for (; kt + NS <= nk; kt += NS) static_for<NS>([&](auto S) { step(S); });      // (NS steps per trip keep the stage a compile-time constant)
    const int rem = nk - kt;
    static_for<NS - 1>([&](auto S) { if (decltype(S)::value < rem) step(S); });
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // the repeated loads of the last steps and the fragments read ahead behind the last one
#pragma unroll
    for (int i = 0; i < C::MI; ++i) asm volatile("" :: "v"(af[0][i]));     // (their registers stay theirs until they have arrived)
#pragma unroll
    for (int j = 0; j < C::NI; ++j) asm volatile("" :: "v"(bfr[0][j]));
    __syncthreads();
    if (d.c_fp8) store_c_tile_fp8<BM, BN, C::WTM, C::WTN, C::MI, C::NI, C::THREADS>(d, acc, smem, m0, n0, g, wm, wn);
    else store_c_tile<BM, BN, C::WTM, C::WTN, C::MI, C::NI, C::CSTR, C::THREADS>(d, acc, smem, m0, n0, g, wm, wn, cvec);
}

// Second kernel of a split contraction: adds the nsplit partial tiles in index order (so the result
// does not depend on timing) and writes C through the column map. One thread per group of four
// consecutive columns (one float4 of the partial tile, which is in accumulator order: element e of
// float4 (q4, tid) of a 64 x 64 tile on 2 x 2 wavefronts is row wm*32 + lane%32, column
// wn*32 + 8*q4 + 4*(lane/32) + e); the loads of four parts are in flight together.
__global__ __launch_bounds__(256) void gemm_split_reduce_kernel(GemmDesc d, int tiles_m, int tiles_n, int cvec4, int nsplit) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q4 = blockIdx.x & 3;
    const int64_t tile = blockIdx.x >> 2;                                    // (g * tiles_m + tile_m) * tiles_n + tile_n
    const int tile_n = (int)(tile % tiles_n), tile_m = (int)((tile / tiles_n) % tiles_m), g = (int)(tile / ((int64_t)tiles_n * tiles_m));
    const int64_t part = (int64_t)tiles_m * tiles_n * d.G * 4096;             // floats per part
    const float* P = d.split_scratch + tile * 4096 + ((q4 * 256 + tid) << 2);
    float4 v = *(const float4*)P;
    for (int z = 1; z < nsplit; z += 4) {
        float4 w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) w[u] = *(const float4*)(P + (z + u < nsplit ? z + u : nsplit - 1) * part);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (z + u < nsplit) { v.x += w[u].x; v.y += w[u].y; v.z += w[u].z; v.w += w[u].w; }
    }
    const int64_t m = (int64_t)tile_m * 64 + (wave >> 1) * 32 + (lane & 31);
    const int n = tile_n * 64 + (wave & 1) * 32 + 8 * q4 + 4 * (lane >> 5);
    if (m >= d.M || n >= d.N) return;
    bf16_t* Cp = (bf16_t*)d.C + m * d.c_rs;
    if (cvec4) {                                                             // four consecutive columns are 8 contiguous bytes of C
        const int64_t col = (int64_t)g * d.c_gs + (int64_t)(n / d.c_div) * d.c_hi + (int64_t)(n % d.c_div) * d.c_lo;
        *(uint2*)(Cp + col) = make_uint2(pack2_bf16(v.x, v.y), pack2_bf16(v.z, v.w));
    } else {
        const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (n + i < d.N) {
                const int ni = n + i;
                Cp[(int64_t)g * d.c_gs + (int64_t)(ni / d.c_div) * d.c_hi + (int64_t)(ni % d.c_div) * d.c_lo] = float_to_bf16(e[i]);
            }
    }
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// How many workgroups share the contraction index of one tile, and how many k steps each takes.
// Splitting pays when a call has too few tiles to keep the chip's memory pipes full: every
// workgroup has a bounded number of bytes in flight, so the bandwidth a call can draw grows with
// the number of workgroups. Parts of at least 8 steps; about 384 workgroups; at most 16 parts.
// Only below 128 tiles: from there on one launch of the deep-step 64 x 64 kernel is faster than the parts
// plus their sum (low-rank 4096 x 4096, r = 1024 at 128 tokens: 21.8 -> 17.7 us; 11008 -> 4096, r = 1488 at
// 512 tokens: 66 -> 54 us); a threshold of 64 loses again (8192 -> 2048, r = 768 at 512 tokens: 30 -> 51 us).
struct SplitPlan { int nsplit, kspan; };
inline SplitPlan split_plan(int64_t ntiles, int K) {
    const int nk = (K + 31) / 32;
    SplitPlan sp{1, nk};
    if (ntiles >= 128 || nk < 16) return sp;
    int want = (int)((384 + ntiles - 1) / ntiles);
    if (want > 16) want = 16;
    if (want > nk / 8) want = nk / 8;
    if (want < 2) return sp;
    sp.kspan = (nk + want - 1) / want;
    sp.nsplit = (nk + sp.kspan - 1) / sp.kspan;
    return sp;
}

// order of the tiles over the XCDs (see workgroup_tile): the A operand of a batched product beyond what
// the memory-side cache holds is streamed by whole rows
inline int tile_order(const GemmDesc& d, bool gfast) {
    if (gfast) return 1;
    if (d.G > 1 && d.a_gs < d.a_rs && (int64_t)d.M * d.a_rs * 2 > (128ll << 20)) return 2;
    return 0;
}

// The order for a launch whose output stores are vectorised (vec) or element-wise.
// Column maps that scatter runs shorter than a 128-byte line: the batches whose runs share lines run
// side by side (batch index fastest). Element-wise stores always; vector stores only when the
// output is larger than the 256 MB memory-side cache, where the parts of a line would otherwise
// reach HBM one by one (stage 1 of Monarch with 16 to 48 ranks per block at 16 k and more tokens:
// 17-24 % faster; with a cache-resident output the batch-major order is up to 20 % faster).
inline int launch_tile_order(const GemmDesc& d, bool vec);

// can 8 consecutive (8-aligned) tile columns be stored as one 16-byte vector?
inline bool c_map_vectorizes(const GemmDesc& d) {
    if (!aligned16(d.C) || d.c_rs % 8 || d.N % 8 || d.c_gs % 8) return false;
    if (d.c_div == 1) return d.c_hi == 1;
    return d.c_div % 8 == 0 && d.c_lo == 1 && d.c_hi % 8 == 0;
}

inline int launch_tile_order(const GemmDesc& d, bool vec) {
    const bool runs_share_lines = vec && d.c_div > 1 && d.c_div < 64 && d.c_hi != d.c_div &&
                                  (int64_t)d.M * d.c_rs * 2 >= (256ll << 20);
    return tile_order(d, (!vec || runs_share_lines) && d.G > 1);
}

// per-lane source offsets are 32-bit; operands further apart than that take the portable kernel
inline bool dma_offsets_fit(const GemmDesc& d, int bm) {
    const int64_t max_brow = d.b_div ? (int64_t)(d.b_div - 1) * d.b_mul + (d.N - 1) / d.b_div : d.N - 1;
    return ((int64_t)bm * d.a_rs + 64) * 2 < (1ll << 32) && (max_brow * d.b_rs + 64) * 2 < (1ll << 32);
}

template <int BM, int BN, int WGM, int WGN, int NS = 4>
hipError_t launch_dma(const GemmDesc& d, hipStream_t s, bool allow_split = false) {
    using C = DmaCfg<BM, BN, WGM, WGN, NS>;
    static LdsLimitOnce lds_limit;
    if (hipError_t e = lds_limit.set({(const void*)gemm_dma_kernel<BM, BN, WGM, WGN, NS, false>,
                                      (const void*)gemm_dma_kernel<BM, BN, WGM, WGN, NS, true>}, C::LDS_BYTES); e != hipSuccess) return e;
    const int tiles_m = (int)((d.M + BM - 1) / BM);
    const int tiles_n = (d.N + BN - 1) / BN;
    const bool vec = c_map_vectorizes(d);
    const int64_t ntiles = (int64_t)tiles_m * tiles_n * d.G;
    SplitPlan sp = split_plan(ntiles, d.K);
    if (!allow_split || !d.split_scratch || (size_t)sp.nsplit * ntiles * BM * BN * sizeof(float) > d.split_scratch_bytes)
        sp = SplitPlan{1, (d.K + C::BK - 1) / C::BK};
    dim3 grid((unsigned)ntiles, 1u, (unsigned)sp.nsplit);
    const int order = launch_tile_order(d, vec);
    if (d.K % C::BK)
        hipLaunchKernelGGL((gemm_dma_kernel<BM, BN, WGM, WGN, NS, true>), grid, dim3(C::THREADS), C::LDS_BYTES, s, d, tiles_m, tiles_n, vec ? 1 : 0, order, sp.kspan);
    else
        hipLaunchKernelGGL((gemm_dma_kernel<BM, BN, WGM, WGN, NS, false>), grid, dim3(C::THREADS), C::LDS_BYTES, s, d, tiles_m, tiles_n, vec ? 1 : 0, order, sp.kspan);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || sp.nsplit == 1) return e;
    if constexpr (BM == 64 && BN == 64 && WGM == 2 && WGN == 2) {   // the only tile the split plan is used with
        // (a column map that keeps groups of 8 columns contiguous keeps groups of 4 contiguous too)
        hipLaunchKernelGGL(gemm_split_reduce_kernel, dim3((unsigned)(ntiles * 4)), dim3(256), 0, s, d, tiles_m, tiles_n, vec ? 1 : 0, sp.nsplit);
        e = hipGetLastError();
    }
    return e;
}

hipError_t launch_wide(const GemmDesc& d, hipStream_t s) {
    using C = DeepCfg<256, 256, 2, 4, 64, 2>;
    static LdsLimitOnce lds_limit;
    if (hipError_t e = lds_limit.set({(const void*)gemm_wide_kernel<false>, (const void*)gemm_wide_kernel<true>}, C::LDS_BYTES); e != hipSuccess) return e;
    const int tiles_m = (int)((d.M + 255) / 256);
    const int tiles_n = (d.N + 255) / 256;
    const bool vec = c_map_vectorizes(d);
    dim3 grid((unsigned)((int64_t)tiles_m * tiles_n * d.G), 1u, 1u);
    const int order = launch_tile_order(d, vec);
    if (d.K % 64)
        hipLaunchKernelGGL((gemm_wide_kernel<true>), grid, dim3(C::THREADS), C::LDS_BYTES, s, d, tiles_m, tiles_n, vec ? 1 : 0, order);
    else
        hipLaunchKernelGGL((gemm_wide_kernel<false>), grid, dim3(C::THREADS), C::LDS_BYTES, s, d, tiles_m, tiles_n, vec ? 1 : 0, order);
    return hipGetLastError();
}

template <int BM, int BN, int WGM, int WGN, int BK, int NS>
hipError_t launch_line(const GemmDesc& d, hipStream_t s) {
    using C = DeepCfg<BM, BN, WGM, WGN, BK, NS>;
    static LdsLimitOnce lds_limit;
    if (hipError_t e = lds_limit.set({(const void*)gemm_line_kernel<BM, BN, WGM, WGN, BK, NS, false>,
                                      (const void*)gemm_line_kernel<BM, BN, WGM, WGN, BK, NS, true>}, C::LDS_BYTES); e != hipSuccess) return e;
    const int tiles_m = (int)((d.M + BM - 1) / BM);
    const int tiles_n = (d.N + BN - 1) / BN;
    const bool vec = c_map_vectorizes(d);
    dim3 grid((unsigned)((int64_t)tiles_m * tiles_n * d.G), 1u, 1u);
    const int order = launch_tile_order(d, vec);
    if (d.K % BK)
        hipLaunchKernelGGL((gemm_line_kernel<BM, BN, WGM, WGN, BK, NS, true>), grid, dim3(C::THREADS), C::LDS_BYTES, s, d, tiles_m, tiles_n, vec ? 1 : 0, order);
    else
        hipLaunchKernelGGL((gemm_line_kernel<BM, BN, WGM, WGN, BK, NS, false>), grid, dim3(C::THREADS), C::LDS_BYTES, s, d, tiles_m, tiles_n, vec ? 1 : 0, order);
    return hipGetLastError();
}

// deep steps need the segments of a segmented contraction index to be whole steps
inline bool deep_ok(const GemmDesc& d, int bk) { return d.a_seg == 0 || d.a_seg % bk == 0; }

}  // namespace

bool mfma_gemm_supported(const GemmDesc& d) {
    return d.b_ks == 1 && d.K % 8 == 0 && d.a_rs % 8 == 0 && d.a_gs % 8 == 0 && d.b_rs % 8 == 0 &&
           d.b_gs % 8 == 0 && aligned16(d.A) && aligned16(d.B) && d.M > 0 && d.N > 0 && d.K > 0 &&
           (int64_t)((d.M + 63) / 64) * ((d.N + 63) / 64) * d.G < (1ll << 30) && dma_offsets_fit(d, 256) &&
           (d.a_seg == 0 || (d.a_seg % 32 == 0 && d.a_seg_stride % 8 == 0));
}

bool gemm_fp8_store_supported(const GemmDesc& d) {
    return mfma_gemm_supported(d) && aligned16(d.C) && d.N % 16 == 0 && d.c_rs % 16 == 0 && d.c_gs % 16 == 0 &&
           d.c_div == 1 && d.c_hi == 1;
}

size_t gemm_split_scratch_bytes(int64_t M, int N, int K, int G) {
    if (M <= 32) return 0;                              // the few-token kernel splits inside its workgroups
    const int64_t ntiles = (int64_t)((M + 63) / 64) * ((N + 63) / 64) * G;
    const SplitPlan sp = split_plan(ntiles, K);
    return sp.nsplit > 1 ? (size_t)sp.nsplit * ntiles * 64 * 64 * sizeof(float) : 0;
}

// compute units of the current device (256 on the part this is written for; asked once)
static int64_t compute_units() {
    static const int n = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
        return cus;
    }();
    return n;
}

hipError_t launch_gemm_mfma(const GemmDesc& d, hipStream_t s) {
    // the 256 x 256 tile: in whole-line steps of 64 unless a segmented contraction index has segments that are not whole steps
    auto big = [&](const GemmDesc& dd) { return deep_ok(dd, 64) ? launch_wide(dd, s) : launch_dma<256, 256, 2, 4>(dd, s); };
    if (d.c_fp8) {                                      // 8-bit C: the tile kernels only (no weight-streaming kernel, no split contraction)
        if (!gemm_fp8_store_supported(d)) return hipErrorInvalidValue;
        auto tiles8 = [&](int bm, int bn) { return (int64_t)((d.M + bm - 1) / bm) * ((d.N + bn - 1) / bn) * d.G; };
        if (d.M > 128 && d.N > 128 && d.K > 128 && tiles8(256, 256) >= 160) return big(d);
        const bool deep8 = d.K >= 128 && deep_ok(d, 64);     // (as for the 16-bit C below)
        if (d.M > 64 && d.N > 64 && tiles8(128, 128) >= 160) return deep8 ? launch_line<128, 128, 2, 2, 64, 2>(d, s) : launch_dma<128, 128, 2, 2>(d, s);
        if (d.M > 64 && tiles8(128, 64) >= 160) return deep8 ? launch_line<128, 64, 2, 2, 64, 2>(d, s) : launch_dma<128, 64, 2, 2>(d, s);
        return deep8 ? launch_line<64, 64, 2, 2, 64, 2>(d, s) : launch_dma<64, 64, 2, 2>(d, s);
    }
    if (skinny_gemm_supported(d)) return launch_gemm_skinny(d, c_map_vectorizes(d), s);
    constexpr int kSmallK = 128;     // very short contractions: 128 x 128 tiles, two workgroups per CU overlap prologue and epilogue
                                     // (measured at K = 256, M = 1024 ... 32768: 256 x 256 tiles are 16-23 % faster)
    auto tiles = [&](int bm, int bn) { return (int64_t)((d.M + bm - 1) / bm) * ((d.N + bn - 1) / bn) * d.G; };
    // large problems: 256 x 256 tiles on 8 wavefronts (half the LDS and L2 traffic per FLOP of 128 x 128)
    // (from 160 tiles on: the same scan as for kFill below, on Monarch, BLAST and low-rank layers at
    // 300 ... 6144 tokens, had 160 ahead of 256 by 5-17 % at the token counts where they differ, and ahead of 128 and 96 on balance)
    if (d.M > 128 && d.N > 128 && d.K > kSmallK && tiles(256, 256) >= 160) {
        // The 256 x 256 tiles run one per compute unit, in rounds; a last round that fills only part of the chip
        // costs a whole round. When that round would be at most 60 % full, the rows of tiles that fit the whole
        // rounds go out here and the remaining rows as a product of their own on 128 x 128 tiles, provided those
        // make a single round (two workgroups per compute unit; such a round takes 0.64 of a round of the large
        // tiles). 4096 -> 11008 at 1536 / 3072 / 6144 tokens: dense 200 -> 148, 318 -> 265, 547 -> 498 us, Monarch
        // stage 2 75 -> 58, 116 -> 106, 201 -> 193 us; remainders of two small rounds (2048, 8192 tokens) were 5 % slower.
        const int64_t per_row = (int64_t)((d.N + 255) / 256) * d.G, rows = (d.M + 255) / 256;
        const int64_t ncu = compute_units(), whole = rows * per_row / ncu, rest = rows * per_row % ncu;
        const int64_t rows1 = whole * ncu / per_row;
        const int64_t m2 = d.M - rows1 * 256;           // the remaining rows and their 128 x 128 tiles
        const int64_t small = ((m2 + 127) / 128) * ((d.N + 127) / 128) * d.G;
        if (whole >= 1 && rest > 0 && rest * 10 <= ncu * 6 && rows1 >= 1 && rows1 < rows && small <= 2 * ncu) {
            GemmDesc d1 = d, d2 = d;
            d1.M = rows1 * 256;
            d2.M = d.M - d1.M;
            d2.A = (const bf16_t*)d.A + d1.M * d.a_rs;
            d2.C = (bf16_t*)d.C + d1.M * d.c_rs;
            if (hipError_t e = big(d1); e != hipSuccess) return e;
            return deep_ok(d2, 64) ? launch_line<128, 128, 2, 2, 64, 2>(d2, s) : launch_dma<128, 128, 2, 2>(d2, s);
        }
        // The same along the columns, where the weight rows are not gathered and the column map is linear in whole
        // column tiles: the column tiles that fill whole rounds go out on the large tile, the remaining columns as a
        // product of their own (one round of smaller tiles by the rules below). Stage 2 of the 4096 -> 11008 Monarch
        // layer at 8192 tokens is 32 x 11 x 4 = 1408 tiles, 5.5 rounds paid as 6: 10 of the 11 column tiles are exactly
        // 5 rounds, the last 192 columns one round of 256 x 128 tiles (no gain there: that round costs 30 of the 34 us
        // it replaces); dense 4096 -> 11008 at 2048 / 5120 / 8192 tokens: 172 -> 148, 381 -> 365, 593 -> 576 us; no
        // shape of a scan over six layer shapes and ten token counts slower.
        const int64_t per_col = rows * d.G, cols = (d.N + 255) / 256;
        const int64_t cols1 = whole * ncu / per_col;
        const int64_t n1 = cols1 * 256;
        if (whole >= 1 && rest > 0 && rest * 10 <= ncu * 6 && cols1 >= 1 && cols1 < cols && d.b_div == 0 && !d.c_fp8 &&
            (d.c_div == 1 || n1 % d.c_div == 0)) {
            GemmDesc d1 = d, d2 = d;
            d1.N = (int)n1;
            d2.N = d.N - (int)n1;
            d2.B = (const bf16_t*)d.B + n1 * d.b_rs;
            d2.C = (bf16_t*)d.C + (d.c_div == 1 ? n1 * d.c_hi : (n1 / d.c_div) * d.c_hi);
            const int64_t t256 = rows * ((d2.N + 127) / 128) * d.G, t128 = ((d.M + 127) / 128) * ((d2.N + 127) / 128) * d.G;
            if (t256 <= ncu || t128 <= 2 * ncu) {
                if (hipError_t e = big(d1); e != hipSuccess) return e;
                return launch_gemm_mfma(d2, s);
            }
        }
        return big(d);
    }
    // Between the two, where the 256 x 256 tiles are too few: 256 x 128 on 8 wavefronts of 64 x 64, one workgroup per
    // compute unit; a quarter less operand traffic per FLOP than the 128 x 128 tile (4096 x 4096 at 2048 tokens:
    // 98.6 -> 85 us; 11008 -> 4096: 232 -> 197 us; Monarch 4096 x 4096 stages: 60 -> 53.5 us per call)
    // (with steps of 64 contraction indices, whole cache lines per operand row, and three stages where the shape allows:
    // another 2-7 %; the same change on the 256 x 256 tile leaves room for two stages only and loses up to 10 %)
    if (d.M > 128 && d.N > 64 && d.K > kSmallK && tiles(256, 128) >= 160)
        return deep_ok(d, 64) ? launch_line<256, 128, 4, 2, 64, 3>(d, s) : launch_dma<256, 128, 4, 2>(d, s);
    // otherwise the largest tile that still gives every compute unit a workgroup
    // 160 of the 256 compute units: a scan of token counts 33 ... 4096 on eight weight shapes had 160
    // ahead of 200 by 10-30 % wherever the two differ (e.g. 11008 -> 4096 at 640 tokens: 144 -> 98 us,
    // 160 tiles of 128 x 128 in one round instead of 320 of 128 x 64 in two) and 128 behind both
    constexpr int64_t kFill = 160;
    // Calls that are a single round of workgroups (at most one per compute unit) take deep steps of 128
    // (64 for the 128 x 128 tile) contraction indices per barrier: every workgroup is alone on its compute
    // unit, so nothing else hides the fixed cost of a step. Measured on the 4096- and 11008-wide layers at
    // 256 ... 2048 tokens: 5-25 % faster for one round; with more workgroups than compute units the
    // 32-deep steps, whose smaller LDS footprint lets two or three workgroups share a compute unit, stay.
    auto one_round = [&](int bm, int bn) { return d.K >= 256 && deep_ok(d, 128) && tiles(bm, bn) <= 256; };
    // With more workgroups than that: steps of 64 on two stages, whose 32 ... 64 KB of LDS let two or three workgroups
    // share a compute unit as the 32-deep kernel's do, in whole cache lines and on the schedule of gemm_line_kernel
    // (768 x 768 at 6304 tokens: 19.1 -> 14.4 us; 3072 -> 768: 58.6 -> 40.8 us; 1152 x 1152 at 1024 tokens: 10.9 -> 8.0 us)
    const bool rounds_deep = d.K >= 128 && deep_ok(d, 64);   // (from two steps on: 128 -> 2304 at 32768 tokens 53.7 -> 46.0 us; 192 -> 768 at 6304 tokens 8.4 -> 7.4 us)
    if (d.M > 64 && d.N > 64 && tiles(128, 128) >= kFill)
        return one_round(128, 128) ? launch_line<128, 128, 2, 2, 64, 4>(d, s) : rounds_deep ? launch_line<128, 128, 2, 2, 64, 2>(d, s) : launch_dma<128, 128, 2, 2>(d, s);
    if (d.M > 64 && tiles(128, 64) >= kFill)
        return one_round(128, 64) ? launch_line<128, 64, 2, 2, 128, 3>(d, s) : rounds_deep ? launch_line<128, 64, 2, 2, 64, 2>(d, s) : launch_dma<128, 64, 2, 2>(d, s);
    if (d.N > 64 && tiles(64, 128) >= kFill)
        return one_round(64, 128) ? launch_line<64, 128, 2, 2, 128, 3>(d, s) : rounds_deep ? launch_line<64, 128, 2, 2, 64, 2>(d, s) : launch_dma<64, 128, 2, 2>(d, s);
    // few tiles and a long contraction: 64 x 64 tiles, contraction index split over several workgroups
    // Few tiles and a long contraction index that would be split (two launches: the parts, then their
    // sum), small weights: the weight-streaming kernel over tiles of 32 tokens instead, one launch.
    // A workgroup streams 96 K bytes (16 weight rows, 32 token rows) at about 55 GB/s; worth it while
    // all rounds of workgroups together stay under about 6.5 us (first low-rank product of the 768-
    // and 1152-wide layers: 2 us less per call in graph replay; with K = 4096 the split parts, which
    // put more workgroups on the stream, are as fast or faster).
    if (d.split_scratch && split_plan(tiles(64, 64), d.K).nsplit > 1 && skinny_gemm_tiled_supported(d)) {
        const int64_t wgs = ((d.M + 31) / 32) * ((d.N + 15) / 16) * d.G;
        const double est_us = (double)((wgs + 255) / 256) * (d.K * 96 / 55e3 + 1.0);
        // ... or under about 9 us when one round of workgroups covers at least half of the chip (4096 x 1024
        // weights at 64 ... 128 tokens: 10 us against 12-13 us; with 32 workgroups the split parts win)
        if (est_us <= 6.5 || (wgs >= 128 && wgs <= 256 && est_us <= 9.0)) return launch_gemm_skinny(d, c_map_vectorizes(d), s);
    }
    if (d.split_scratch && split_plan(tiles(64, 64), d.K).nsplit > 1) return launch_dma<64, 64, 2, 2>(d, s, true);
    // the smallest tile already from 128 workgroups on: at 128 tokens it beats the weight-streaming kernel over
    // 32-token tiles (dense 4096 x 4096: 17.0 against 23.6 us; 11008 -> 4096: 36 against 55 us)
    if (tiles(64, 64) >= 128 || (d.M <= 64 && d.N <= 64))
        return one_round(64, 64) ? launch_line<64, 64, 2, 2, 128, 4>(d, s) : rounds_deep ? launch_line<64, 64, 2, 2, 64, 2>(d, s) : launch_dma<64, 64, 2, 2>(d, s);
    // Nothing fills the chip (a product of some tens of tokens with weights that are not split, e.g.
    // the dense reference at 33 ... 96 tokens): the weight-streaming kernel over tiles of 32 tokens puts
    // every compute unit on the stream, where the few tiles below would walk the whole contraction
    // index at about 0.17 us per step of 32 (dense 4096 x 4096 at 48 tokens: 29.6 -> 17.3 us;
    // 8192 -> 2048: 55.5 -> 17.4 us). Taken when its estimate (rounds of workgroups x the time to
    // stream 96 K bytes at 55 GB/s) is below that walk by a margin (level estimates went to the tiles).
    if (skinny_gemm_tiled_supported(d)) {
        const int64_t wgs = ((d.M + 31) / 32) * ((d.N + 15) / 16) * d.G;
        const double est_us = (double)((wgs + 255) / 256) * (d.K * 96 / 55e3 + 1.0);
        if (est_us < 0.85 * ((d.K + 31) / 32 * 0.17 + 3.0)) return launch_gemm_skinny(d, c_map_vectorizes(d), s);
    }
    // too small to fill the chip with any tile: fewest, largest tiles that fit the shape
    if (d.M > 64 && d.N > 64) return tiles(64, 64) >= 64 ? launch_dma<64, 64, 2, 2>(d, s) : launch_dma<128, 128, 2, 2>(d, s);
    if (d.M > 64) return launch_dma<128, 64, 2, 2>(d, s);
    return launch_dma<64, 64, 2, 2>(d, s);              // one row of tiles: the narrower tile doubles the workgroups on the stream
}

}  // namespace blr
