// BLAST stage 1 + coupling fused in one kernel (bf16 MFMA, gfx950).
//
// A workgroup owns a tile of TN tokens x TR rank indices. It loops over the input blocks j inside
// the workgroup (the reduction over j cannot be split across workgroups): for each j the tile
// Z_j = X_j V_j is a small GEMM on v_mfma_f32_32x32x16_bf16, whose result is rounded to bf16 and
// parked in LDS as Zs[rho][t][j]. When all j are done, the coupling A[t][i][rho] = sum_j S[i][j][rho]
// Z[t][j][rho] is, for every rho, a (tokens x 16) . (16 x 16) product: one v_mfma_f32_16x16x16_bf16
// per 16 tokens, with the per-rho 16x16 tile of S read from the packed tensor Sp[rho][i][j].
// Z never leaves the chip and the coupling runs on the matrix cores; only A goes to HBM.
#include "blr_common.h"

namespace blr {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int TN = 64, TR = 64, BK = 32;
constexpr int D = 8;                         // steps of global loads kept in flight (even)
constexpr int ZSTR = TN * 32 + 8;            // bytes of one rho row of Zs: TN tokens x 16 j x 2 B, + 8 B pad
constexpr int ZS_BYTES = TR * ZSTR;
constexpr int STR = BK * 2 + 16;             // staged operand row stride (bytes)
constexpr int STAGE = (TN + TR) * STR;
constexpr int LDS_BYTES = ZS_BYTES + 2 * STAGE;
static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
static_assert(D % 2 == 0, "ring slot parity must equal LDS stage parity");
static_assert(ZS_BYTES % 16 == 0, "Zs is cleared with 16-byte stores");

__device__ inline uint32_t pack2(float lo, float hi) { return pack2_bf16(lo, hi); }

// workgroup id -> logical tile id such that each XCD (workgroups are dealt round-robin over 8 XCDs)
// works on a contiguous range of logical ids, i.e. shares its X tiles in its own L2
__device__ inline int xcd_contiguous(int bid, int nblk) {
    const int q8 = nblk >> 3, rem = nblk & 7;
    const int xcd = bid & 7, slot = bid >> 3;
    return xcd * q8 + (xcd < rem ? xcd : rem) + slot;
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void blast_stage12_kernel(const bf16_t* __restrict__ X, const bf16_t* __restrict__ Vt,
                                                            const bf16_t* __restrict__ Sp, bf16_t* __restrict__ A,
                                                            int64_t T, int n_in, int b, int r, int tiles_r, int nblk) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* Zs = smem;
    unsigned char* stg = smem + ZS_BYTES;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int logical = xcd_contiguous(blockIdx.x, nblk);
    const int tile_t = logical / tiles_r, tile_r = logical % tiles_r;
    const int64_t t0 = (int64_t)tile_t * TN;
    const int rho0 = tile_r * TR;
    const int q = n_in / b;

    const int lrow = tid >> 2, lchunk = tid & 3;
    int64_t tx = t0 + lrow;
    if (tx > T - 1) tx = T - 1;                         // rows past the end re-read the last row; never stored
    int rr = rho0 + lrow;
    if (rr > r - 1) rr = r - 1;
    const bf16_t* xp = X + tx * n_in;
    const bf16_t* vp = Vt + (int64_t)rr * q;
    const int64_t v_jstride = (int64_t)r * q;

    if (b < 16)                                         // unused j slots must read as zero in the coupling
        for (int i = tid * 16; i < ZS_BYTES; i += 256 * 16) *(uint4*)(Zs + i) = make_uint4(0, 0, 0, 0);

    const int nkc = (q + BK - 1) / BK;
    const int nsteps = b * nkc;
    // Register ring of D steps of global loads in flight (as in the GEMM kernel); a step is (j, kc).
    // Loads are unconditional: the fetch cursor stops at the last step, chunks past q are zeroed on
    // their way to LDS.
    uint4 ra[D], rb[D];
    int pj = 0, pk = 0;                                 // cursor of the next step to fetch
    auto gload = [&](auto SLOT) {
        constexpr int slot = decltype(SLOT)::value;
        int k = pk * BK + lchunk * 8;
        if (k > q - 8) k = q - 8;                       // q is a multiple of 8
        ra[slot] = *(const uint4*)(xp + pj * q + k);
        rb[slot] = *(const uint4*)(vp + pj * v_jstride + k);
        if (pj * nkc + pk < nsteps - 1) { if (++pk == nkc) { pk = 0; ++pj; } }
    };
    auto sstore = [&](auto SLOT, int kc_of_slot) {
        constexpr int slot = decltype(SLOT)::value;
        constexpr int stage = slot & 1;              // D is even: slot parity == step parity
        unsigned char* base = stg + stage * STAGE;
        const bool ok = (kc_of_slot * BK + lchunk * 8) < q;
        *(uint4*)(base + lrow * STR + lchunk * 16) = keep_if(ok, ra[slot]);
        *(uint4*)(base + TN * STR + lrow * STR + lchunk * 16) = keep_if(ok, rb[slot]);
    };

    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;

    const int frag_off = (lane & 31) * STR + (lane >> 5) * 16;
    int j = 0, kc = 0;                                  // cursor of the step being computed
    auto step = [&](auto U) {                           // u = step % D, a compile-time constant
        constexpr int u = decltype(U)::value;
        const unsigned char* As = stg + (u & 1) * STAGE + (wm * 32) * STR + frag_off;
        const unsigned char* Bs = stg + (u & 1) * STAGE + TN * STR + (wn * 32) * STR + frag_off;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const bf16x8 af = *(const bf16x8*)(As + ks * 32);
            const bf16x8 bfr = *(const bf16x8*)(Bs + ks * 32);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc, 0, 0, 0);
        }
        const bool last_kc = (kc == nkc - 1);
        if (last_kc) {
            // Z_j tile done: element e is token 8*(e/4) + 4*(lane/32) + e%4, rank index lane%32 of this wave's quadrant
            unsigned char* zrow = Zs + (wn * 32 + (lane & 31)) * ZSTR + (wm * 32 + 4 * (lane >> 5)) * 32 + j * 2;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                *(bf16_t*)(zrow + (8 * (e / 4) + (e % 4)) * 32) = float_to_bf16(acc[e]);
                acc[e] = 0.f;
            }
        }
        const int kc_next = last_kc ? 0 : kc + 1;
        sstore(std::integral_constant<int, (u + 1) % D>{}, kc_next);   // past the last step this writes the unused stage
        gload(std::integral_constant<int, (u + 1) % D>{});
        __syncthreads();
        kc = kc_next;
        if (last_kc) ++j;
    };

    static_for<D>([&](auto U) { gload(U); });
    sstore(std::integral_constant<int, 0>{}, 0);
    gload(std::integral_constant<int, 0>{});
    __syncthreads();
    int s0 = 0;
    for (; s0 + D <= nsteps; s0 += D) static_for<D>([&](auto U) { step(U); });
    static_for<D - 1>([&](auto U) { if (s0 + decltype(U)::value < nsteps) step(U); });

    // coupling: this wave takes 16 consecutive rank indices of the tile
    const int rl0 = wave * 16;
    const int ci = lane & 15, cg = lane >> 4;
    s16x4 sfrag[16];
#pragma unroll
    for (int ri = 0; ri < 16; ++ri) {
        const int rg = rho0 + rl0 + ri;
        if (rg < r) sfrag[ri] = *(const s16x4*)(Sp + (int64_t)rg * 256 + ci * 16 + cg * 4);
        else sfrag[ri] = s16x4{0, 0, 0, 0};
    }
    const bool lo_ok = rho0 + rl0 < r, hi_ok = rho0 + rl0 + 8 < r;   // r is a multiple of 8
#pragma unroll 1
    for (int tg = 0; tg < TN / 16; ++tg) {
        f32x4 d[16];
#pragma unroll
        for (int ri = 0; ri < 16; ++ri) {
            const s16x4 a = *(const s16x4*)(Zs + (rl0 + ri) * ZSTR + (tg * 16 + ci) * 32 + cg * 8);
            d[ri] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, sfrag[ri], f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        }
        // d[ri][e]: token tg*16 + 4*(lane/16) + e, output block i = lane%16
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t tok = t0 + tg * 16 + 4 * cg + e;
            if (tok < T && ci < b) {
                bf16_t* dst = A + (tok * b + ci) * r + rho0 + rl0;
                if (lo_ok) *(uint4*)dst = make_uint4(pack2(d[0][e], d[1][e]), pack2(d[2][e], d[3][e]),
                                                     pack2(d[4][e], d[5][e]), pack2(d[6][e], d[7][e]));
                if (hi_ok) *(uint4*)(dst + 8) = make_uint4(pack2(d[8][e], d[9][e]), pack2(d[10][e], d[11][e]),
                                                           pack2(d[12][e], d[13][e]), pack2(d[14][e], d[15][e]));
            }
        }
    }
}

}  // namespace

bool blast_fused_supported(int64_t T, int n_in, int b, int r) {
    if (T <= 0 || b <= 0 || b > 16 || n_in % b) return false;
    const int q = n_in / b;
    const int64_t nblk = ((T + TN - 1) / TN) * ((r + TR - 1) / TR);
    return q % 8 == 0 && r % 8 == 0 && nblk < (1ll << 30);
}

hipError_t launch_blast_stage12(const void* X, const void* Vt, const void* Sp, void* A,
                                int64_t T, int n_in, int b, int r, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)blast_stage12_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_t = (int)((T + TN - 1) / TN), tiles_r = (r + TR - 1) / TR;
    const int nblk = tiles_t * tiles_r;
    hipLaunchKernelGGL(blast_stage12_kernel, dim3((unsigned)nblk), dim3(256), LDS_BYTES, s,
                       (const bf16_t*)X, (const bf16_t*)Vt, (const bf16_t*)Sp, (bf16_t*)A, T, n_in, b, r, tiles_r, nblk);
    return hipGetLastError();
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
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t t0 = (int64_t)blockIdx.x * FT;
    const int q = n_in / b, p = n_out / b;
    const int nks = (q + 15) >> 4;
    const int ci = lane & 15, cg = lane >> 4;
    const int l32 = lane & 31, kg = lane >> 5;
    // this wavefront's input blocks (phase 1), rank groups (phase 2) and output blocks (phase 3)
    const int jw[2] = {wave < b ? wave : b - 1, wave + FWAVES < b ? wave + FWAVES : b - 1};
    const int cw[2] = {wave < nchunks ? wave : nchunks - 1, wave + FWAVES < nchunks ? wave + FWAVES : nchunks - 1};

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
                    braw[jj][u][nt] = *(const uint4*)(Vf + (((int64_t)(jw[jj] * NT + nt) * nks + ks) * 64 + lane) * 8);
            }
    };
    load_vf(0);

    // ---- phase 0: X tile -> LDS with coalesced 16-byte loads (rows past T repeat the last row; the
    // 16 pad bytes of a row are zeroed because the last k-step of the last block may read them
    // against zero V fragments)
    {
        const int cpr = n_in >> 3;                                   // 16-byte chunks per row
        const int total = FT * cpr;
        for (int base = 0; base < total; base += FTHREADS * 4) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                int id = base + u * FTHREADS + tid;
                if (id > total - 1) id = total - 1;
                const int row = id / cpr, cc = id - row * cpr;
                int64_t tx = t0 + row;
                if (tx > T - 1) tx = T - 1;
                v[u] = *(const uint4*)(X + tx * n_in + cc * 8);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                int id = base + u * FTHREADS + tid;
                if (id > total - 1) id = total - 1;
                const int row = id / cpr, cc = id - row * cpr;
                *(uint4*)(XY + row * xstr + cc * 16) = v[u];
            }
        }
        if (tid < FT) *(uint4*)(XY + tid * xstr + n_in * 2) = make_uint4(0, 0, 0, 0);
        if (b < 16)                                                 // unused j slots must read as zero
            for (int i = tid * 16; i < NT * 4 * FCHUNK; i += FTHREADS * 16) *(uint4*)(Zs + i) = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();

    // S tiles of this wavefront's rank groups: in flight during phase 1
    s16x4 sfr[2][8];
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int ri = 0; ri < 8; ++ri)
            sfr[cc][ri] = *(const s16x4*)(Sp + (int64_t)(cw[cc] * 8 + ri) * 256 + ci * 16 + cg * 4);

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
                ufr[ii][nt][ks] = *(const uint4*)(Uf + (((int64_t)(i * NPT + nt) * NT + ks) * 64 + lane) * 8);
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
                    unsigned char* zrow = Zs + rho * FZSTR + (4 * kg) * 32 + wave * 4;
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        *(uint32_t*)(zrow + (8 * (e / 4) + (e % 4)) * 32) = pack2_bf16(zacc[0][nt][e], has1 ? zacc[1][nt][e] : 0.f);
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
#pragma unroll
        for (int ri = 0; ri < 8; ++ri)
#pragma unroll
            for (int tg = 0; tg < 2; ++tg) {
                const s16x4 a = *(const s16x4*)(chunk + ri * FZSTR + (tg * 16 + ci) * 32 + cg * 8);
                d[tg][ri] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, sfr[cc][ri], f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
            }
        // every read of this chunk has been issued by this wavefront before the writes below, and
        // LDS operations of one wavefront complete in order; d[tg][ri][e]: token tg*16 + 4*cg + e, block ci
#pragma unroll
        for (int tg = 0; tg < 2; ++tg)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int tok = tg * 16 + 4 * cg + e;
                *(uint4*)(chunk + (ci * FT + (tok ^ (ci & 7))) * 16) =
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
#pragma unroll
        for (int nt = 0; nt < NPT; ++nt) {
            f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < NT; ++ks) {
                int c = ks * 4 + cg;                                // group of 8 rank indices this lane multiplies
                if (c > nchunks - 1) c = nchunks - 1;               // past r the U fragment is zero; read a valid group
                const unsigned char* chunk = Zs + c * FCHUNK;
                const bf16x8 a0 = *(const bf16x8*)(chunk + (ic * FT + (ci ^ (ic & 7))) * 16);
                const bf16x8 a1 = *(const bf16x8*)(chunk + (ic * FT + ((16 + ci) ^ (ic & 7))) * 16);
                acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const bf16x8*)&ufr[ii][nt][ks], a0, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const bf16x8*)&ufr[ii][nt][ks], a1, acc1, 0, 0, 0);
            }
            // U is the first operand, so acc[e] is output feature i*p + nt*16 + 4*cg + e of token
            // (mt*16) + ci: four consecutive features per lane, one 8-byte LDS write each
            unsigned char* ydst = XY + ci * ystr + (i * p + nt * 16 + 4 * cg) * 2;
            *(uint2*)ydst = make_uint2(pack2_bf16(acc0[0], acc0[1]), pack2_bf16(acc0[2], acc0[3]));
            *(uint2*)(ydst + 16 * ystr) = make_uint2(pack2_bf16(acc1[0], acc1[1]), pack2_bf16(acc1[2], acc1[3]));
        }
    });
    __syncthreads();

    // ---- coalesced copy of the staged output tile
    {
        const int cpr = n_out >> 3;                                  // 16-byte chunks per row
        for (int id = tid; id < FT * cpr; id += FTHREADS) {
            const int row = id / cpr, cc = id - row * cpr;
            if (t0 + row < T) *(uint4*)(Y + (t0 + row) * n_out + cc * 8) = *(const uint4*)(XY + row * ystr + cc * 16);
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
    if (q % 8 || r % 8 || p % 16 || p > 64 || r > 128) return false;
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
    static bool attr_set = false;
    const int lds = full_fusion_lds_bytes(n_in, n_out, r);
    auto kern = blast_full_kernel<NT, KG, NPT>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
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
