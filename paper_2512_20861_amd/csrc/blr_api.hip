// C-ABI front end: argument validation, workspace planning, kernel selection. Host code only.
#include "../../include/blr.h"
#include "../../include/blr_measure.h"
#include "blr_common.h"
#include <algorithm>
#include <mutex>

using namespace blr;

namespace {

inline size_t elem_size(blr_dtype dt) { return dt == BLR_BF16 ? 2 : 4; }
inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
inline bool dtype_ok(blr_dtype dt) { return dt == BLR_F32 || dt == BLR_BF16; }
inline blr_status from_hip(hipError_t e) { return e == hipSuccess ? BLR_OK : BLR_ERR_LAUNCH; }

blr_status run_gemm(const GemmDesc& d, blr_dtype dt, bool allow_mfma, hipStream_t s) {
    if (allow_mfma && dt == BLR_BF16 && mfma_gemm_supported(d)) return from_hip(launch_gemm_mfma(d, s));
    return from_hip(launch_gemm_valu(d, dt == BLR_BF16 ? DType::BF16 : DType::F32, s));
}

bool monarch_shape_ok(int64_t T, int n_in, int n_out, int nblocks, int r) {
    return T >= 0 && n_in > 0 && n_out > 0 && nblocks > 0 && r > 0 && n_in % nblocks == 0 &&
           n_out % nblocks == 0 && r % nblocks == 0;
}

bool blast_shape_ok(int64_t T, int n_in, int n_out, int b, int r) {
    return T >= 0 && n_in > 0 && n_out > 0 && b > 0 && r > 0 && n_in % b == 0 && n_out % b == 0;
}

// Shapes the MFMA BLAST kernels take (the others run on the portable kernels): at most 16 blocks,
// 16-byte rows of V and of the rank index, and a rank whose tile offsets (tokens of a tile * b * r) fit 32 bits.
bool blast_mfma_shape_ok(int n_in, int b, int r) {
    return b <= 16 && (n_in / b) % 8 == 0 && r % 8 == 0 && r < (1 << 20);
}

// The quantised-intermediate execution (Z as 8-bit floats between the stage-1 product and the coupling) exists
// for bf16 layers on the matrix-core kernels of the three-kernel path, with packed factors whose buffer holds
// the stage-1 operand, and 16 | r (16 consecutive rank indices are one 16-byte store).
bool blast_z_fp8_ok(int n_in, int n_out, int b, int r, blr_dtype dt, unsigned flags);

// Where the re-laid-out BLAST factors live inside the packed buffer.
struct PackLayout {
    bool full;                       // served by the single-kernel path: fragment-ordered V and U
    size_t off_Sp, off_Sc, off_Vt, off_Va, off_Vf, off_Uf, total;   // Sc: canonical S; Va: chunk-aligned Vt (= Vt if 64 | q)
};

PackLayout pack_layout(int n_in, int n_out, int b, int r) {
    PackLayout pk{};
    size_t off = 0;
    pk.off_Sp = off; off += align_up((size_t)r * 256 * 2);
    pk.full = blast_full_fusion_shape_ok(n_in, n_out, b, r);
    if (pk.full) {
        pk.off_Vf = off; off += align_up(blast_vf_bytes(n_in, b, r));
        pk.off_Uf = off; off += align_up(blast_uf_bytes(n_out, b, r));
    } else {
        pk.off_Vt = off; off += align_up((size_t)n_in * r * 2);
        const int q = n_in / b;
        const int chunk = blast_chunk(n_in, b);
        if (q % chunk) { pk.off_Va = off; off += align_up((size_t)b * r * blast_va_row(q, chunk) * 2); }
        else pk.off_Va = pk.off_Vt;
        pk.off_Sc = off; off += align_up((size_t)b * b * r * 2);
    }
    pk.total = off;
    return pk;
}

// How a BLAST call is executed and where its temporaries live in the workspace.
struct BlastPlan {
    enum Path { GENERIC, MFMA_THREE, MFMA_STAGE12, MFMA_FULL, MFMA_NARROW } path;
    int64_t chunk;                   // tokens per pass of the three-kernel path (its Z and A chunks stay cache-resident)
    size_t off_A, off_Z, off_pack, total;
};

// The three-kernel path (stage-1 GEMM, MFMA coupling, stage-3 GEMM) walks the tokens in chunks whose
// two intermediates (Z and A, b*r bf16 per token each) together stay well inside the 256 MB
// memory-side cache, so that they are produced and consumed without a round trip to HBM.
constexpr size_t kChunkBytes = 48u << 20;
// The fused stage 1 + coupling kernel runs one workgroup per compute unit; below a number of 128-token
// tiles it leaves too much of the chip idle and the three-kernel path (finer tiles) is faster. What the
// fused kernel saves, the round trip of Z, grows with b r per token; what it pays, a stage 1 on tiles
// of half the arithmetic intensity of the GEMM's, grows with n_in r: the longer the input block
// q = n_in / b, the more tiles it takes to come out ahead (measured at q = 64 ... 688, r = 256 ... 1024).
inline int64_t fused_min_tiles(int n_in, int b) {
    const int q = n_in / b;
    return q <= 128 ? 80 : q <= 256 ? 120 : 224;
}
// Up to this many tokens the coupling runs as one thread per 8 outputs; from there on the MFMA coupling kernel on its
// 16-token tiles is ahead (BLAST 4096 x 4096, r = 640: 13.6 against 14.4 us at 33 tokens, 16.5 against 15.9 at 64,
// 17.4 against 15.5 at 100, 19.0 against 16.3 at 128).
constexpr int64_t kSmallCouplingTokens = 48;

// The single kernel for few, wide blocks: forced by its flag, else where it was measured ahead of the three kernels.
bool blast_narrow_possible(int64_t T, int n_in, int n_out, int b, int r, unsigned flags) {
    return !(flags & (BLR_BLAST_FUSED_STAGE12 | BLR_BLAST_THREE_KERNELS | BLR_BLAST_Z_FP8 | BLR_ONLY_FIRST_STAGE | BLR_ONLY_LAST_STAGE)) &&
           blast_narrow_supported(T, n_in, n_out, b, r) && !pack_layout(n_in, n_out, b, r).full;
}
bool blast_takes_narrow(int64_t T, int n_in, int n_out, int b, int r, unsigned flags) {
    if (!blast_narrow_possible(T, n_in, n_out, b, r, flags)) return false;
    if (flags & BLR_BLAST_ONE_KERNEL) return true;
    // Every workgroup streams all of V, so V has to be small (ViT-B / GPT2-S widths: 196 and 295 KB; with the
    // 590 KB of the DiT layers the three kernels are 30 % ahead), and the launch a single round of workgroups:
    // one per compute unit, or, with the smallest V, two where two fit LDS. Measured on the 768-wide layers of the
    // paper's layer-wise table at 128 ... 8192 tokens: b = 3, r = 128: 9.5 / 11.6 / 14.3 us against 11.9 / 15.7 /
    // 18.2 us on three kernels at 197 / 1024 / 2048 tokens, level at 3072 ... 4096; b = 6, r = 192: 15.5 against
    // 17.5 us at 1024 tokens, level below, behind from 1536 tokens on (23.6 against 19.0 us).
    if ((int64_t)n_in * r > 160 * 1024) return false;
    const int64_t wgs = blast_narrow_workgroups(T, n_out, b);
    return wgs <= 256 || (wgs <= 512 && (int64_t)n_in * r <= 100 * 1024 && blast_narrow_lds_bytes(T, n_in, n_out, b, r) <= 80 * 1024);
}

BlastPlan blast_plan(int64_t T, int n_in, int n_out, int b, int r, blr_dtype dt, unsigned flags) {
    BlastPlan pl{};
    const int q = n_in / b;
    const bool packed = flags & BLR_BLAST_PACKED;
    const bool mfma = dt == BLR_BF16 && !(flags & BLR_FORCE_GENERIC) && blast_mfma_shape_ok(n_in, b, r);
    const size_t per_token = (size_t)b * r * elem_size(dt);
    size_t off = 0;
    pl.chunk = T;
    if (!mfma) {
        pl.path = BlastPlan::GENERIC;
        pl.off_A = off; off += align_up((size_t)T * per_token);
        pl.off_Z = off; off += align_up((size_t)T * per_token);
    } else {
        if (flags & BLR_BLAST_Z_FP8) pl.path = BlastPlan::MFMA_THREE;      // (the caller has checked blast_z_fp8_ok)
        else if (blast_full_fusion_supported(T, n_in, n_out, b, r)) pl.path = BlastPlan::MFMA_FULL;
        else if (blast_takes_narrow(T, n_in, n_out, b, r, flags)) pl.path = BlastPlan::MFMA_NARROW;
        else if (!(flags & BLR_BLAST_THREE_KERNELS) && blast_fused_supported(T, n_in, b, r) &&
                 ((flags & BLR_BLAST_FUSED_STAGE12) || blast_fused_tiles(T, r) >= fused_min_tiles(n_in, b))) pl.path = BlastPlan::MFMA_STAGE12;
        else pl.path = BlastPlan::MFMA_THREE;
        if (pl.path == BlastPlan::MFMA_STAGE12) { pl.off_A = off; off += align_up((size_t)T * per_token); }
        if (pl.path == BlastPlan::MFMA_THREE) {
            int64_t c = (int64_t)(kChunkBytes / per_token) / 256 * 256;
            if (c < 256) c = 256;
            if (c < T) pl.chunk = c;
            pl.off_A = off; off += align_up((size_t)pl.chunk * per_token);
            pl.off_Z = off; off += align_up((size_t)pl.chunk * per_token / ((flags & BLR_BLAST_Z_FP8) ? 2 : 1));   // one byte per element of an 8-bit Z
        }
        if (!packed) { pl.off_pack = off; off += pack_layout(n_in, n_out, b, r).total; }
    }
    pl.total = off;
    return pl;
}

bool blast_z_fp8_ok(int n_in, int n_out, int b, int r, blr_dtype dt, unsigned flags) {
    return dt == BLR_BF16 && !(flags & (BLR_FORCE_GENERIC | BLR_BLAST_FUSED_STAGE12)) && blast_mfma_shape_ok(n_in, b, r) && r % 16 == 0 &&
           !pack_layout(n_in, n_out, b, r).full;
}

blr_status run_pack(const void* U, const void* S, const void* V, void* packed, int n_in, int n_out, int b, int r, hipStream_t s) {
    const PackLayout pk = pack_layout(n_in, n_out, b, r);
    unsigned char* base = (unsigned char*)packed;
    return from_hip(launch_blast_pack(U, S, V, base + pk.off_Sp, pk.full ? nullptr : base + pk.off_Sc, pk.full ? nullptr : base + pk.off_Vt,
                                      (pk.full || pk.off_Va == pk.off_Vt) ? nullptr : base + pk.off_Va,
                                      pk.full ? base + pk.off_Vf : nullptr, pk.full ? base + pk.off_Uf : nullptr,
                                      n_in, n_out, b, r, s));
}

// Is this call (Monarch with b1 x b2 blocks of rank rp; low-rank is 1 x 1) served by the single kernel
// that keeps the intermediate on chip? It can be when the shape fits and the call asks for neither
// the portable kernels, nor a single stage, nor a blocked input. It is by default where it was
// measured faster than the two GEMMs (narrow layers of the ViT-B / GPT2-S kind, 1.1-1.4x; within
// +-10 % for the lowest ranks at token counts that leave a partial round of workgroups): two
// workgroups fit a compute unit (half of LDS each) and not more tokens than one to two rounds of
// 32-token tiles.
constexpr int64_t kFusedMonarchMaxTokens = 4096;
constexpr int kFusedMonarchMaxLds = 80 * 1024;
bool monarch_fused_possible(int64_t T, int n_in, int n_out, int b1, int b2, int rp, blr_dtype dt, unsigned flags) {
    if (dt != BLR_BF16 || (flags & (BLR_FORCE_GENERIC | BLR_ONLY_FIRST_STAGE | BLR_ONLY_LAST_STAGE | BLR_MONARCH_IN_BLOCKED | BLR_MONARCH_TWO_KERNELS))) return false;
    return monarch_fused_supported(T, n_in, n_out, b1, b2, rp);
}
bool monarch_takes_fused(int64_t T, int n_in, int n_out, int b1, int b2, int rp, blr_dtype dt, unsigned flags) {
    if (!monarch_fused_possible(T, n_in, n_out, b1, b2, rp, dt, flags)) return false;
    if (flags & BLR_MONARCH_FUSED) return true;
    if (T <= 32) return false;
    if (T <= kFusedMonarchMaxTokens && monarch_fused_lds_bytes(T, n_in, n_out, b1, b2, rp) <= kFusedMonarchMaxLds) return true;
    // Wider layers, whose token tile takes more than half of LDS (one workgroup per compute unit): the
    // single kernel still wins while the call is one round of workgroups, with 16 or more output
    // blocks (2048 x 2048, b = 16, r' = 16: 8.8 / 10.0 / 12.5 us against 12.7 / 11.2 / 14.6 us at
    // 64 / 256 / 512 tokens; 1024 x 1024: 6.3-8.4 us against 9.6-14.1 us) and, for any number of
    // blocks, up to 64 tokens (8.0-8.9 us against 10.4-11.3 us); at 8 blocks and 197-512 tokens the
    // two GEMMs are level or up to 8 % faster and stay.
    const int64_t base = ((T + 31) / 32) * b2;
    return base <= 256 && (b2 >= 16 || T <= 64);
}

// The interleaved output order through 2-byte stores at stride b2 costs stage 2 up to twice its time
// on large outputs (2048 -> 8192, b = 16, T = 8192: 222 us against 83 us in the blocked order). From
// 4 M output elements on (2 M for wide rows in 16 and more blocks; graph-replay timings), stage 2 therefore writes the blocked order into the workspace, in chunks
// of tokens that stay in the memory-side cache, and a permutation pass (both sides 16-byte
// coalesced, about the time of a copy of the chunk) produces the interleaved order. With 8 blocks the
// two ways are level, with 4 and 2 the scattered stores are faster (8- and 4-byte gaps between a
// lane's elements instead of 32-byte ones: 4096 -> 11008, b = 4, T = 8192: 249 us against 285 us).
constexpr int kInterleavePassMinBlocks = 8;
constexpr int64_t kInterleavePassMinElems = 4ll << 20;
constexpr size_t kInterleaveChunkBytes = 64u << 20;
bool monarch_interleave_pass_shape(int64_t T, int n_out, int b2, blr_dtype dt) {
    // with 16 and more blocks and rows of 2048 and more elements the pass already pays from 2 M outputs on
    const int64_t min_elems = b2 >= 16 && n_out >= 2048 ? kInterleavePassMinElems / 2 : kInterleavePassMinElems;
    return dt == BLR_BF16 && b2 >= kInterleavePassMinBlocks && T * n_out >= min_elems && monarch_interleave_supported(T, n_out, b2);
}
int64_t monarch_interleave_chunk(int64_t T, int n_out) {
    int64_t c = (int64_t)(kInterleaveChunkBytes / ((size_t)n_out * 2)) / 256 * 256;
    if (c < 1024) c = 1024;
    return c < T ? c : T;
}
size_t monarch_workspace(int64_t T, int n_out, int b1, int b2, int rp, blr_dtype dt) {
    size_t bytes = align_up((size_t)T * b1 * b2 * rp * elem_size(dt));
    if (monarch_interleave_pass_shape(T, n_out, b2, dt)) bytes += align_up((size_t)monarch_interleave_chunk(T, n_out) * n_out * 2);
    return bytes;
}

// Both Monarch entry points: b1 input blocks, b2 output blocks, per-block rank rp.
blr_status monarch_run(const void* X, const void* R, const void* L, void* Y, int64_t T, int n_in, int n_out,
                       int b1, int b2, int rp, blr_dtype dt, unsigned flags, void* workspace, hipStream_t s) {
    const int p = n_in / b1, q = n_out / b2;
    const int w1 = rp * b2, w2 = b1 * rp;               // widths of one middle block before / after the permutation
    const bool allow_mfma = !(flags & BLR_FORCE_GENERIC);
    if (monarch_takes_fused(T, n_in, n_out, b1, b2, rp, dt, flags))
        return from_hip(launch_monarch_fused(X, R, L, Y, T, n_in, n_out, b1, b2, rp, flags & BLR_MONARCH_OUT_BLOCKED, s));

    // stage 1: block-diagonal R; tile column n' = k*r' + rho reads row rho*b2 + k of R[l] (the
    // re-layout of the first factor done in the load index) and lands at Z'[t][k][l*r' + rho]
    GemmDesc s1{};
    s1.A = X; s1.a_gs = p; s1.a_rs = n_in;
    s1.B = R; s1.b_gs = (int64_t)w1 * p; s1.b_rs = p; s1.b_ks = 1; s1.b_div = rp; s1.b_mul = b2;
    s1.C = workspace; s1.c_rs = (int64_t)b2 * w2; s1.c_gs = rp; s1.c_div = rp; s1.c_hi = w2; s1.c_lo = 1;
    s1.M = T; s1.N = w1; s1.K = p; s1.G = b1;
    if (flags & BLR_MONARCH_IN_BLOCKED) {             // input block l = b runs of p/b elements, run k at k*(n_in/b) + l*(p/b)
        s1.a_gs = p / b1; s1.a_seg = p / b1; s1.a_seg_stride = n_in / b1;
    }
    if (!(flags & BLR_ONLY_LAST_STAGE)) {
        blr_status st = run_gemm(s1, dt, allow_mfma, s);
        if (st != BLR_OK || (flags & BLR_ONLY_FIRST_STAGE)) return st;
    }

    // stage 2: block-diagonal L; the output order is a column map of the store
    GemmDesc s2{};
    s2.A = workspace; s2.a_gs = w2; s2.a_rs = (int64_t)b2 * w2;
    s2.B = L; s2.b_gs = (int64_t)q * w2; s2.b_rs = w2; s2.b_ks = 1; s2.b_div = 0; s2.b_mul = 0;
    s2.C = Y; s2.c_rs = n_out; s2.c_div = 1; s2.c_lo = 0;
    if (flags & BLR_MONARCH_OUT_BLOCKED) { s2.c_gs = q; s2.c_hi = 1; }
    else { s2.c_gs = 1; s2.c_hi = b2; }
    s2.M = T; s2.N = q; s2.K = w2; s2.G = b2;
    if ((flags & BLR_MONARCH_OUT_BLOCKED) || !allow_mfma || !monarch_interleave_pass_shape(T, n_out, b2, dt))
        return run_gemm(s2, dt, allow_mfma, s);
    // interleaved order of a large output: blocked order into the workspace, then the permutation pass
    unsigned char* Yb = (unsigned char*)workspace + align_up((size_t)T * b2 * w2 * 2);
    s2.C = Yb; s2.c_gs = q; s2.c_hi = 1;
    const int64_t chunk = monarch_interleave_chunk(T, n_out);
    for (int64_t c0 = 0; c0 < T; c0 += chunk) {
        const int64_t tc = T - c0 < chunk ? T - c0 : chunk;
        s2.A = (const unsigned char*)workspace + (size_t)c0 * b2 * w2 * 2;
        s2.M = tc;
        blr_status st = run_gemm(s2, dt, true, s);
        if (st != BLR_OK) return st;
        st = from_hip(launch_monarch_interleave(Yb, (unsigned char*)Y + (size_t)c0 * n_out * 2, tc, n_out, b2, s));
        if (st != BLR_OK) return st;
    }
    return BLR_OK;
}

bool monarch_rect_shape_ok(int64_t T, int n_in, int n_out, int b1, int b2, int rp) {
    return T >= 0 && n_in > 0 && n_out > 0 && b1 > 0 && b2 > 0 && rp > 0 && n_in % b1 == 0 && n_out % b2 == 0 &&
           (int64_t)b1 * b2 * rp < (1ll << 30);
}

}  // namespace

// A group runs on the bf16 MFMA kernels of stages 1 and 2 with the concatenated rank, or not at all.
static bool blast_group_ok(int64_t T, int n_in, int n_out, int b, int r, int members, blr_dtype dt, unsigned flags) {
    if (members <= 0 || r <= 0 || r % 8 || (int64_t)r * members > (1 << 24) || dt != BLR_BF16 || b > 16) return false;   // 8 | r: every member's range of A starts on a 16-byte boundary
    if (!blast_shape_ok(T, n_in, n_out, b, r * members) || !blast_mfma_shape_ok(n_in, b, r * members)) return false;
    if (pack_layout(n_in, n_out, b, r * members).full) return false;     // such a pack holds no stage-1 operand
    const BlastPlan::Path path = blast_plan(T > 0 ? T : 1, n_in, n_out, b, r * members, dt, flags | BLR_BLAST_PACKED).path;
    return path == BlastPlan::MFMA_STAGE12 || path == BlastPlan::MFMA_THREE;
}

// The multi-kernel executions of `members` BLAST layers of one shape that share X (members = 1: the
// plain layer; rm: rank of one member). Stages 1 and 2 act on every rank index by itself, so the
// members' rank indices simply concatenate there; stage 3 contracts each member's own range.
static blr_status blast_run(const void* X, const void* U, const void* S, const void* V, void* Y,
                            int64_t T, int n_in, int n_out, int b, int rm, int members,
                            blr_dtype dt, unsigned flags,
                            void* workspace, size_t workspace_bytes, hipStream_t s) {
    const int r = rm * members;                     // stages 1 and 2 see one layer of rank r
    const BlastPlan pl = blast_plan(T, n_in, n_out, b, r, dt, flags);
    if ((flags & BLR_BLAST_PACKED) && pl.path == BlastPlan::GENERIC) return BLR_ERR_UNSUPPORTED;
    if (pl.total > 0 && (!workspace || workspace_bytes < pl.total)) return BLR_ERR_WORKSPACE;
    const int q = n_in / b, p = n_out / b;
    unsigned char* ws = (unsigned char*)workspace;
    void* Aws = ws + pl.off_A;
    void* Zws = ws + pl.off_Z;

    // stage 3 (all multi-kernel paths), member m: Y[t][m*n_out + i*p + a] = sum_rho A[t][i][m*rm + rho] U_m[i][a][rho]
    const size_t es = elem_size(dt);
    const int64_t ldy = (int64_t)members * n_out;
    GemmDesc s3{};
    s3.a_gs = r; s3.a_rs = (int64_t)b * r;
    s3.b_gs = (int64_t)p * rm; s3.b_rs = rm; s3.b_ks = 1; s3.b_div = 0;
    s3.c_rs = ldy; s3.c_gs = p; s3.c_div = 1; s3.c_hi = 1; s3.c_lo = 0;
    s3.M = T; s3.N = p; s3.K = rm; s3.G = b;
    auto run_stage3 = [&](int64_t c0, int64_t tc, bool mfma) {   // tokens c0 .. c0 + tc - 1; A holds them from its start
        for (int m = 0; m < members; ++m) {
            s3.A = (const unsigned char*)Aws + (size_t)m * rm * es;
            s3.B = (const unsigned char*)U + (size_t)m * n_out * rm * es;
            s3.C = (unsigned char*)Y + ((size_t)c0 * ldy + (size_t)m * n_out) * es;
            s3.M = tc;
            blr_status st = run_gemm(s3, dt, mfma, s);
            if (st != BLR_OK) return st;
        }
        return BLR_OK;
    };

    // stage 1 as a stand-alone product: Z[t][j][rho]
    GemmDesc s1{};
    s1.A = X; s1.a_gs = q; s1.a_rs = n_in;
    s1.C = Zws; s1.c_rs = (int64_t)b * r; s1.c_gs = r; s1.c_div = 1; s1.c_hi = 1; s1.c_lo = 0;
    s1.M = T; s1.N = r; s1.K = q; s1.G = b;

    const bool first = !(flags & BLR_ONLY_LAST_STAGE), last = !(flags & BLR_ONLY_FIRST_STAGE);
    if (pl.path == BlastPlan::GENERIC) {
        if (members != 1) return BLR_ERR_UNSUPPORTED;
        if (first) {
            s1.B = V; s1.b_gs = (int64_t)q * r; s1.b_rs = 1; s1.b_ks = r; s1.b_div = 0;   // V[j][c][rho]: rho contiguous
            blr_status st = run_gemm(s1, dt, false, s);
            if (st != BLR_OK) return st;
            st = from_hip(launch_coupling_valu(Zws, S, Aws, T, b, r, dt == BLR_BF16 ? DType::BF16 : DType::F32, s));
            if (st != BLR_OK) return st;
        }
        return last ? run_stage3(0, T, false) : BLR_OK;
    }

    // one kernel: there are no stages to select, and a group is never packed for it (checked before anything is enqueued)
    if (pl.path == BlastPlan::MFMA_FULL && (!first || !last || members != 1)) return BLR_ERR_UNSUPPORTED;
    const unsigned char* pack = (const unsigned char*)V;
    if (!(flags & BLR_BLAST_PACKED)) {
        pack = ws + pl.off_pack;
        if (first) {
            blr_status st = run_pack(U, S, V, ws + pl.off_pack, n_in, n_out, b, r, s);
            if (st != BLR_OK) return st;
        }
    }
    const PackLayout pk = pack_layout(n_in, n_out, b, r);
    const void* Sp = pack + pk.off_Sp;
    const void* Vt = pack + pk.off_Vt;
    if (pl.path == BlastPlan::MFMA_FULL)
        return from_hip(launch_blast_full(X, Sp, pack + pk.off_Vf, pack + pk.off_Uf, Y, T, n_in, n_out, b, r, s));
    if (pl.path == BlastPlan::MFMA_NARROW) {
        if (members != 1) return BLR_ERR_UNSUPPORTED;
        return from_hip(launch_blast_narrow(X, Vt, pack + pk.off_Sc, U, Y, T, n_in, n_out, b, r, s));
    }
    if (pl.path == BlastPlan::MFMA_STAGE12) {
        if (first) {
            blr_status st = from_hip(launch_blast_stage12(X, pack + pk.off_Va, Sp, Aws, T, n_in, b, r, s));
            if (st != BLR_OK) return st;
        }
        return last ? run_stage3(0, T, true) : BLR_OK;
    }
    // three kernels per chunk of tokens: stage-1 GEMM -> Z, MFMA coupling Z -> A, stage-3 GEMM
    s1.B = Vt; s1.b_gs = (int64_t)q * r; s1.b_rs = q; s1.b_ks = 1; s1.b_div = 0;
    const bool z8 = flags & BLR_BLAST_Z_FP8;
    s1.c_fp8 = z8 ? 1 : 0;                              // Z[t][j][rho] as bytes: the same strides, counted in bytes
    for (int64_t c0 = 0; c0 < T; c0 += pl.chunk) {
        const int64_t tc = T - c0 < pl.chunk ? T - c0 : pl.chunk;
        if (first) {
            s1.A = (const unsigned char*)X + (size_t)c0 * n_in * 2;
            s1.M = tc;
            blr_status st = run_gemm(s1, dt, true, s);
            if (st != BLR_OK) return st;
            // few tokens: one thread per 8 outputs
            st = from_hip(z8 ? launch_blast_coupling(Zws, Sp, Aws, tc, b, r, s, true)
                          : tc <= kSmallCouplingTokens ? launch_coupling_small(Zws, pack + pk.off_Sc, Aws, tc, b, r, s)
                                                       : launch_blast_coupling(Zws, Sp, Aws, tc, b, r, s));
            if (st != BLR_OK) return st;
        }
        if (last) {
            blr_status st = run_stage3(c0, tc, true);
            if (st != BLR_OK) return st;
        }
    }
    return BLR_OK;
}


extern "C" {

const char* blr_status_string(blr_status s) {
    switch (s) {
        case BLR_OK: return "ok";
        case BLR_ERR_INVALID_ARG: return "invalid argument";
        case BLR_ERR_UNSUPPORTED: return "unsupported configuration";
        case BLR_ERR_WORKSPACE: return "workspace missing or too small";
        case BLR_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

size_t blr_monarch_workspace_bytes(int64_t T, int n_in, int n_out, int nblocks, int r, blr_dtype dt) {
    if (!monarch_shape_ok(T, n_in, n_out, nblocks, r) || !dtype_ok(dt)) return 0;
    return monarch_workspace(T, n_out, nblocks, nblocks, r / nblocks, dt);
}

blr_status blr_monarch_forward(const void* X, const void* R, const void* L, void* Y,
                               int64_t T, int n_in, int n_out, int nblocks, int r,
                               blr_dtype dt, unsigned flags,
                               void* workspace, size_t workspace_bytes, blr_stream stream) {
    if (!monarch_shape_ok(T, n_in, n_out, nblocks, r) || !dtype_ok(dt)) return BLR_ERR_INVALID_ARG;
    if (flags & ~(BLR_MONARCH_OUT_BLOCKED | BLR_MONARCH_IN_BLOCKED | BLR_FORCE_GENERIC | BLR_ONLY_FIRST_STAGE | BLR_ONLY_LAST_STAGE | BLR_MONARCH_FUSED | BLR_MONARCH_TWO_KERNELS)) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_MONARCH_FUSED) && (flags & (BLR_MONARCH_TWO_KERNELS | BLR_MONARCH_IN_BLOCKED | BLR_FORCE_GENERIC | BLR_ONLY_FIRST_STAGE | BLR_ONLY_LAST_STAGE))) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_ONLY_FIRST_STAGE) && (flags & BLR_ONLY_LAST_STAGE)) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_MONARCH_IN_BLOCKED) && (n_in / nblocks) % nblocks) return BLR_ERR_INVALID_ARG;
    if (!R || !L) return BLR_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(R) || !aligned16(L) || !aligned16(Y) || !aligned16(workspace)) return BLR_ERR_INVALID_ARG;
    if (T == 0) return BLR_OK;                      // X and Y of an empty batch may be null
    if (!X || !Y) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_MONARCH_FUSED) && !monarch_fused_possible(T, n_in, n_out, nblocks, nblocks, r / nblocks, dt, flags)) return BLR_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < blr_monarch_workspace_bytes(T, n_in, n_out, nblocks, r, dt)) return BLR_ERR_WORKSPACE;
    return monarch_run(X, R, L, Y, T, n_in, n_out, nblocks, nblocks, r / nblocks, dt, flags, workspace, (hipStream_t)stream);
}

// ---- Monarch forward for callers that cannot allocate: Z' lives in a static device array --------
// One array per GPU (each device that loads the library holds its own copy until the process ends).
// In host code the array's name is only a handle: the device address comes from hipGetSymbolAddress,
// looked up once per device with that device current, and only that address is handed to kernels.
}  // extern "C"

static __device__ __align__(256) unsigned char scratch[BLR_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
struct DeviceScratch { std::once_flag once; void* ptr = nullptr; hipError_t err = hipSuccess; };
DeviceScratch g_scratch[kMaxDevices];

// device address of this GPU's copy of `scratch` (nullptr and the HIP error on failure)
hipError_t static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    DeviceScratch& ds = g_scratch[dev];
    std::call_once(ds.once, [&] { ds.err = hipGetSymbolAddress(&ds.ptr, HIP_SYMBOL(scratch)); });
    *out = ds.ptr;
    return ds.err;
}
}  // namespace

extern "C" {

size_t blr_static_scratch_bytes(void) { return BLR_STATIC_SCRATCH_BYTES; }

blr_status blr_monarch_forward_static(const void* X, const void* R, const void* L, void* Y,
                                      int64_t T, int n_in, int n_out, int nblocks, int r,
                                      blr_dtype dt, unsigned flags, blr_stream stream) {
    if (!monarch_shape_ok(T, n_in, n_out, nblocks, r) || !dtype_ok(dt)) return BLR_ERR_INVALID_ARG;
    // sizes beyond the array are refused before anything else is looked at
    if (blr_monarch_workspace_bytes(T, n_in, n_out, nblocks, r, dt) > BLR_STATIC_SCRATCH_BYTES) return BLR_ERR_WORKSPACE;
    void* ws = nullptr;
    if (static_scratch(&ws) != hipSuccess || !ws) return BLR_ERR_LAUNCH;
    return blr_monarch_forward(X, R, L, Y, T, n_in, n_out, nblocks, r, dt, flags, ws, BLR_STATIC_SCRATCH_BYTES, stream);
}

size_t blr_monarch_rect_workspace_bytes(int64_t T, int n_in, int n_out, int b_in, int b_out, int r_block, blr_dtype dt) {
    if (!monarch_rect_shape_ok(T, n_in, n_out, b_in, b_out, r_block) || !dtype_ok(dt)) return 0;
    return monarch_workspace(T, n_out, b_in, b_out, r_block, dt);
}

blr_status blr_monarch_rect_forward(const void* X, const void* R, const void* L, void* Y,
                                    int64_t T, int n_in, int n_out, int b_in, int b_out, int r_block,
                                    blr_dtype dt, unsigned flags,
                                    void* workspace, size_t workspace_bytes, blr_stream stream) {
    if (!monarch_rect_shape_ok(T, n_in, n_out, b_in, b_out, r_block) || !dtype_ok(dt)) return BLR_ERR_INVALID_ARG;
    if (flags & ~(BLR_MONARCH_OUT_BLOCKED | BLR_FORCE_GENERIC | BLR_ONLY_FIRST_STAGE | BLR_ONLY_LAST_STAGE | BLR_MONARCH_FUSED | BLR_MONARCH_TWO_KERNELS)) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_MONARCH_FUSED) && (flags & (BLR_MONARCH_TWO_KERNELS | BLR_FORCE_GENERIC | BLR_ONLY_FIRST_STAGE | BLR_ONLY_LAST_STAGE))) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_ONLY_FIRST_STAGE) && (flags & BLR_ONLY_LAST_STAGE)) return BLR_ERR_INVALID_ARG;
    if (!R || !L) return BLR_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(R) || !aligned16(L) || !aligned16(Y) || !aligned16(workspace)) return BLR_ERR_INVALID_ARG;
    if (T == 0) return BLR_OK;
    if (!X || !Y) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_MONARCH_FUSED) && !monarch_fused_possible(T, n_in, n_out, b_in, b_out, r_block, dt, flags)) return BLR_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < blr_monarch_rect_workspace_bytes(T, n_in, n_out, b_in, b_out, r_block, dt)) return BLR_ERR_WORKSPACE;
    return monarch_run(X, R, L, Y, T, n_in, n_out, b_in, b_out, r_block, dt, flags, workspace, (hipStream_t)stream);
}

size_t blr_lowrank_workspace_bytes(int64_t T, int n_in, int n_out, int r, blr_dtype dt) {
    if (T < 0 || T >= (1ll << 31) || n_in <= 0 || n_out <= 0 || r <= 0 || !dtype_ok(dt)) return 0;
    size_t split = 0;                                   // fp32 partial tiles of a split contraction (either stage)
    if (dt == BLR_BF16) split = std::max(gemm_split_scratch_bytes(T, r, n_in, 1), gemm_split_scratch_bytes(T, n_out, r, 1));
    return align_up((size_t)T * r * elem_size(dt)) + align_up(split);
}

blr_status blr_lowrank_forward(const void* X, const void* V, const void* U, void* Y,
                               int64_t T, int n_in, int n_out, int r, blr_dtype dt, unsigned flags,
                               void* workspace, size_t workspace_bytes, blr_stream stream) {
    if (T < 0 || T >= (1ll << 31) || n_in <= 0 || n_out <= 0 || r <= 0 || !dtype_ok(dt)) return BLR_ERR_INVALID_ARG;
    if (flags & ~(BLR_FORCE_GENERIC | BLR_ONLY_FIRST_STAGE | BLR_ONLY_LAST_STAGE | BLR_MONARCH_FUSED | BLR_MONARCH_TWO_KERNELS)) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_MONARCH_FUSED) && (flags & (BLR_MONARCH_TWO_KERNELS | BLR_FORCE_GENERIC | BLR_ONLY_FIRST_STAGE | BLR_ONLY_LAST_STAGE))) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_ONLY_FIRST_STAGE) && (flags & BLR_ONLY_LAST_STAGE)) return BLR_ERR_INVALID_ARG;
    if (!V || !U) return BLR_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(V) || !aligned16(U) || !aligned16(Y) || !aligned16(workspace)) return BLR_ERR_INVALID_ARG;
    if (T == 0) return BLR_OK;
    if (!X || !Y) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_MONARCH_FUSED) && !monarch_fused_possible(T, n_in, n_out, 1, 1, r, dt, flags)) return BLR_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < blr_lowrank_workspace_bytes(T, n_in, n_out, r, dt)) return BLR_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    // a single block of a Monarch layer: V and U are its two factors in the same storage orders
    if (monarch_takes_fused(T, n_in, n_out, 1, 1, r, dt, flags))
        return from_hip(launch_monarch_fused(X, V, U, Y, T, n_in, n_out, 1, 1, r, true, s));
    const bool allow_mfma = !(flags & BLR_FORCE_GENERIC);
    // Z[T][r] = X V^T, then Y = Z U^T: two plain NT products, the narrow intermediate in the workspace.
    // With few tokens and a narrow rank the first product has few tiles and a long contraction index:
    // the rest of the workspace lets the GEMM split that index over several workgroups per tile.
    const size_t z_bytes = align_up((size_t)T * r * elem_size(dt));
    float* scratch = workspace_bytes > z_bytes ? (float*)((char*)workspace + z_bytes) : nullptr;
    GemmDesc s1{};
    s1.split_scratch = scratch; s1.split_scratch_bytes = workspace_bytes - z_bytes;
    s1.A = X; s1.a_rs = n_in;
    s1.B = V; s1.b_rs = n_in; s1.b_ks = 1;
    s1.C = workspace; s1.c_rs = r; s1.c_div = 1; s1.c_hi = 1;
    s1.M = T; s1.N = r; s1.K = n_in; s1.G = 1;
    if (!(flags & BLR_ONLY_LAST_STAGE)) {
        blr_status st = run_gemm(s1, dt, allow_mfma, s);
        if (st != BLR_OK || (flags & BLR_ONLY_FIRST_STAGE)) return st;
    }
    GemmDesc s2{};
    s2.split_scratch = scratch; s2.split_scratch_bytes = workspace_bytes - z_bytes;
    s2.A = workspace; s2.a_rs = r;
    s2.B = U; s2.b_rs = r; s2.b_ks = 1;
    s2.C = Y; s2.c_rs = n_out; s2.c_div = 1; s2.c_hi = 1;
    s2.M = T; s2.N = n_out; s2.K = r; s2.G = 1;
    return run_gemm(s2, dt, allow_mfma, s);
}

blr_status blr_monarch_group_first_factor(const void* R_stack, void* R_group, int n_in, int nblocks, int r, int members,
                                          blr_dtype dt, blr_stream stream) {
    if (!R_stack || !R_group || R_stack == R_group || !dtype_ok(dt)) return BLR_ERR_INVALID_ARG;
    if (n_in <= 0 || nblocks <= 0 || r <= 0 || members <= 0 || n_in % nblocks || r % nblocks) return BLR_ERR_INVALID_ARG;
    return from_hip(launch_monarch_group_first_factor(R_stack, R_group, n_in, nblocks, r, members,
                                                      dt == BLR_BF16 ? DType::BF16 : DType::F32, (hipStream_t)stream));
}

blr_status blr_monarch_permute_first_factor(const void* R, void* Rp, int n_in, int nblocks, int r,
                                            blr_dtype dt, blr_stream stream) {
    if (!R || !Rp || R == Rp || !dtype_ok(dt)) return BLR_ERR_INVALID_ARG;
    if (n_in <= 0 || nblocks <= 0 || r <= 0 || n_in % nblocks || (n_in / nblocks) % nblocks) return BLR_ERR_INVALID_ARG;
    return from_hip(launch_monarch_permute_first_factor(R, Rp, n_in, nblocks, r, dt == BLR_BF16 ? DType::BF16 : DType::F32, (hipStream_t)stream));
}

size_t blr_blast_workspace_bytes(int64_t T, int n_in, int n_out, int b, int r, blr_dtype dt, unsigned flags) {
    if (!blast_shape_ok(T, n_in, n_out, b, r) || !dtype_ok(dt)) return 0;
    if ((flags & BLR_BLAST_Z_FP8) && !blast_z_fp8_ok(n_in, n_out, b, r, dt, flags)) return 0;
    return blast_plan(T, n_in, n_out, b, r, dt, flags).total;
}

size_t blr_blast_packed_bytes(int n_in, int n_out, int b, int r, blr_dtype dt) {
    if (dt != BLR_BF16 || !blast_shape_ok(0, n_in, n_out, b, r) || !blast_mfma_shape_ok(n_in, b, r)) return 0;
    return pack_layout(n_in, n_out, b, r).total;
}

blr_status blr_blast_pack(const void* U, const void* S, const void* V, void* packed,
                          int n_in, int n_out, int b, int r, blr_dtype dt, blr_stream stream) {
    if (!U || !S || !V || !packed) return BLR_ERR_INVALID_ARG;
    if (!blast_shape_ok(0, n_in, n_out, b, r) || dt != BLR_BF16 || b > 16) return BLR_ERR_INVALID_ARG;
    if (!blast_mfma_shape_ok(n_in, b, r)) return BLR_ERR_UNSUPPORTED;   // such layers run on the portable kernels, unpacked
    if (!aligned16(U) || !aligned16(S) || !aligned16(V) || !aligned16(packed)) return BLR_ERR_INVALID_ARG;
    return run_pack(U, S, V, packed, n_in, n_out, b, r, (hipStream_t)stream);
}

blr_status blr_blast_forward(const void* X, const void* U, const void* S, const void* V, void* Y,
                             int64_t T, int n_in, int n_out, int b, int r,
                             blr_dtype dt, unsigned flags,
                             void* workspace, size_t workspace_bytes, blr_stream stream) {
    if (!U || !V || (!S && !(flags & BLR_BLAST_PACKED))) return BLR_ERR_INVALID_ARG;
    if (!blast_shape_ok(T, n_in, n_out, b, r) || !dtype_ok(dt)) return BLR_ERR_INVALID_ARG;
    if (flags & ~(BLR_BLAST_PACKED | BLR_BLAST_ONE_KERNEL | BLR_FORCE_GENERIC | BLR_ONLY_FIRST_STAGE | BLR_ONLY_LAST_STAGE | BLR_BLAST_FUSED_STAGE12 | BLR_BLAST_THREE_KERNELS | BLR_BLAST_Z_FP8)) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_BLAST_Z_FP8) && (flags & (BLR_BLAST_FUSED_STAGE12 | BLR_FORCE_GENERIC))) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_ONLY_FIRST_STAGE) && (flags & BLR_ONLY_LAST_STAGE)) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_BLAST_FUSED_STAGE12) && (flags & BLR_BLAST_THREE_KERNELS)) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_BLAST_ONE_KERNEL) && (flags & (BLR_BLAST_FUSED_STAGE12 | BLR_BLAST_THREE_KERNELS | BLR_BLAST_Z_FP8 | BLR_FORCE_GENERIC | BLR_ONLY_FIRST_STAGE | BLR_ONLY_LAST_STAGE))) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_BLAST_PACKED) && (dt != BLR_BF16 || b > 16 || (flags & BLR_FORCE_GENERIC))) return BLR_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(U) || !aligned16(S) || !aligned16(V) || !aligned16(Y) || !aligned16(workspace)) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_BLAST_Z_FP8) && !blast_z_fp8_ok(n_in, n_out, b, r, dt, flags)) return BLR_ERR_UNSUPPORTED;
    if ((flags & BLR_BLAST_ONE_KERNEL) && (dt != BLR_BF16 || !blast_mfma_shape_ok(n_in, b, r) || !blast_narrow_possible(T > 0 ? T : 1, n_in, n_out, b, r, flags))) return BLR_ERR_UNSUPPORTED;
    if (T == 0) return BLR_OK;                      // X and Y of an empty batch may be null
    if (!X || !Y) return BLR_ERR_INVALID_ARG;
    return blast_run(X, U, S, V, Y, T, n_in, n_out, b, r, 1, dt, flags, workspace, workspace_bytes, (hipStream_t)stream);
}

size_t blr_blast_group_workspace_bytes(int64_t T, int n_in, int n_out, int b, int r, int members, blr_dtype dt, unsigned flags) {
    if (!blast_group_ok(T, n_in, n_out, b, r, members, dt, flags)) return 0;
    return blast_plan(T, n_in, n_out, b, r * members, dt, flags | BLR_BLAST_PACKED).total;
}

blr_status blr_blast_group_forward(const void* X, const void* U, const void* packed, void* Y,
                                   int64_t T, int n_in, int n_out, int b, int r, int members,
                                   blr_dtype dt, unsigned flags,
                                   void* workspace, size_t workspace_bytes, blr_stream stream) {
    if (!U || !packed || members <= 0 || !dtype_ok(dt)) return BLR_ERR_INVALID_ARG;
    if (r <= 0 || (int64_t)r * members > (1 << 24)) return BLR_ERR_INVALID_ARG;
    if (!blast_shape_ok(T, n_in, n_out, b, r * members)) return BLR_ERR_INVALID_ARG;
    if (flags & ~(BLR_BLAST_FUSED_STAGE12 | BLR_BLAST_THREE_KERNELS)) return BLR_ERR_INVALID_ARG;
    if ((flags & BLR_BLAST_FUSED_STAGE12) && (flags & BLR_BLAST_THREE_KERNELS)) return BLR_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(U) || !aligned16(packed) || !aligned16(Y) || !aligned16(workspace)) return BLR_ERR_INVALID_ARG;
    if (!blast_group_ok(T, n_in, n_out, b, r, members, dt, flags)) return BLR_ERR_UNSUPPORTED;
    if (T == 0) return BLR_OK;
    if (!X || !Y) return BLR_ERR_INVALID_ARG;
    return blast_run(X, U, nullptr, packed, Y, T, n_in, n_out, b, r, members, dt, flags | BLR_BLAST_PACKED,
                     workspace, workspace_bytes, (hipStream_t)stream);
}

blr_status blr_dense_reference_forward(const void* X, const void* W, void* Y,
                                       int64_t T, int n_in, int n_out, blr_dtype dt,
                                       unsigned flags, blr_stream stream) {
    if (!W) return BLR_ERR_INVALID_ARG;
    if (T < 0 || n_in <= 0 || n_out <= 0 || !dtype_ok(dt)) return BLR_ERR_INVALID_ARG;
    if (flags & ~BLR_FORCE_GENERIC) return BLR_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(W) || !aligned16(Y)) return BLR_ERR_INVALID_ARG;
    if (T == 0) return BLR_OK;
    if (!X || !Y) return BLR_ERR_INVALID_ARG;
    GemmDesc d{};
    d.A = X; d.a_gs = 0; d.a_rs = n_in;
    d.B = W; d.b_gs = 0; d.b_rs = n_in; d.b_ks = 1; d.b_div = 0;
    d.C = Y; d.c_rs = n_out; d.c_gs = 0; d.c_div = 1; d.c_hi = 1; d.c_lo = 0;
    d.M = T; d.N = n_out; d.K = n_in; d.G = 1;
    return run_gemm(d, dt, !(flags & BLR_FORCE_GENERIC), (hipStream_t)stream);
}

}  // extern "C"
