/*
 * blr.h - C ABI of the block low-rank (BLR) linear forward library for AMD MI355X (gfx950).
 *
 * The library evaluates Y = X W^T for a weight W[n_out][n_in] that is never formed, but given
 * by Monarch, BLAST or plain low-rank factors (paper Section 2.1, "Weight Structures"), plus a plain
 * dense product that serves as the speed-up denominator, and the row-wise / elementwise steps that
 * sit between the linears of a decoder-layer chain.
 *
 * Conventions shared by every entry point
 *   - All pointers are DEVICE pointers (HIP global memory), 16-byte aligned, to dense row-major
 *     tensors without padding. Storage type `dt`: BLR_BF16 (bfloat16 bit patterns, arithmetic in
 *     bf16 x bf16 -> fp32 MFMA, intermediates that leave the chip rounded to bf16, Y rounded to
 *     bf16) or BLR_F32 (everything fp32).
 *   - Ownership: the caller owns every buffer, including the workspace. The library allocates
 *     nothing, frees nothing and never synchronises; it only enqueues kernels on `stream`
 *     (a hipStream_t passed as void*; NULL is the default stream). Buffers must stay alive and
 *     unmodified until the stream has passed the call. Inputs are read-only; Y and the workspace
 *     are overwritten; Y and the workspace must not alias any input or each other.
 *   - Errors: the return code only. No exceptions, no abort, no output to stderr. All argument
 *     checks happen on the host before anything is enqueued, so an error return means nothing
 *     was launched (except BLR_ERR_LAUNCH, which reports hipGetLastError() after a launch).
 *     T == 0 returns BLR_OK without launching (X and Y may then be null; the factors may not).
 *   - Calls on different streams may overlap as long as their Y/workspace buffers are distinct.
 */
#ifndef BLR_H
#define BLR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BLR_OK = 0,
    BLR_ERR_INVALID_ARG = 1,   /* null pointer, negative T, non-positive or non-divisible sizes, bad dtype/flags */
    BLR_ERR_UNSUPPORTED = 2,   /* valid by the mathematics but no kernel covers it */
    BLR_ERR_WORKSPACE = 3,     /* workspace missing or smaller than blr_*_workspace_bytes() */
    BLR_ERR_LAUNCH = 4         /* the HIP runtime reported an error when launching */
} blr_status;

typedef enum { BLR_F32 = 0, BLR_BF16 = 1 } blr_dtype;

typedef void* blr_stream;      /* a hipStream_t */

/* flags of blr_monarch_forward: order of the output features (paper Section 4, optimisation 3).
 * INTERLEAVED is the (n, q, b2) order of the full operator P L P^T R: Y[t][j*nblocks + k].
 * BLOCKED is the cheaper (n, b2, q) order, Y[t][k*q + j], usable when the consumer's weight rows
 * are permuted offline. */
#define BLR_MONARCH_OUT_INTERLEAVED 0u
#define BLR_MONARCH_OUT_BLOCKED     1u
/* flag of blr_monarch_forward: X is in the BLOCKED order of an upstream layer with the same nblocks
 * (feature j*nblocks + k stored at k*(n_in/nblocks) + j), and R is the re-ordered first factor
 * written by blr_monarch_permute_first_factor (paper Section 4, optimisation 3: the upstream
 * layer's final permutation is folded into this layer's static weight; any elementwise step in
 * between commutes with the permutation). Needs nblocks^2 | n_in. */
#define BLR_MONARCH_IN_BLOCKED      4u
/* flag of blr_blast_forward: the `V` argument is the buffer written by blr_blast_pack (the one-time
 * offline weight re-layout of paper Section 4, optimisations 1 and 5) and `S` is ignored. */
#define BLR_BLAST_PACKED            2u
/* Flag bits 0x100, 0x200 and 0x400 of every forward are test and measurement aids (portable kernels only;
 * only the first / only the last stage of a multi-kernel call). They are declared in blr_measure.h and
 * are not needed by an application. */
/* flags of blr_blast_forward for layers too large for the single-kernel path. Two executions exist:
 * (a) stage 1 and the coupling fused in one kernel (Z stays on chip; the paper's optimisation 4 with
 * the coupling on the matrix cores) followed by the stage-3 GEMM, and (b) three kernels over
 * cache-resident token chunks (the paper's optimisation 5). By default the library picks (a) when
 * the call has enough 128-token x 64-rank tiles to fill the chip and (b) otherwise; these flags
 * force one of them (mutually exclusive) so that tests and the benchmark can run both. */
#define BLR_BLAST_FUSED_STAGE12     0x800u
#define BLR_BLAST_THREE_KERNELS     0x1000u
/* flag of blr_blast_forward: force the single-kernel execution for layers of FEW, WIDE blocks (the b = 3, 6, 9
 * layers of the paper's layer-wise table): one workgroup per (32 tokens, output block, range of its outputs) runs
 * stage 1 for every input block, accumulates the coupling in registers (Z is never rounded nor stored) and runs
 * stage 3 on its range. bf16; needs 32 | n_in/b, n_in/b <= 256, 32 | r, r <= 256 and a 32-token tile of X within
 * LDS, else BLR_ERR_UNSUPPORTED. By default the library takes this execution where it was measured faster than
 * the three kernels (few hundred to a few thousand tokens). Not combinable with the other execution flags of
 * blr_blast_forward nor with the stage flags of blr_measure.h. */
#define BLR_BLAST_ONE_KERNEL        0x10000u
/* flag of blr_blast_forward: quantised intermediate (the paper's "Limitation and Future Work": quantising the
 * intermediate activations). Runs execution (b) with Z = X_j V_j stored as 8-bit floats (OCP E4M3: 4 exponent
 * and 3 mantissa bits, round to nearest even from the fp32 accumulator, clamped to the largest finite value
 * 448) between the stage-1 product and the coupling, which widens them again; A and Y are as without the flag.
 * Halves the bytes of the Z round trip at the price of one more rounding of 2^-4 relative size per element of
 * Z. bf16 only, 16 | r, not for layers the single-kernel path serves (BLR_ERR_UNSUPPORTED, workspace query 0);
 * cannot be combined with BLR_BLAST_FUSED_STAGE12. The workspace query takes the flag. */
#define BLR_BLAST_Z_FP8             0x8000u
/* flags of the Monarch and low-rank forwards (bf16). Two executions exist: (a) two GEMM kernels with
 * the intermediate in the workspace, and (b) ONE kernel that keeps the intermediate on chip (the
 * full fusion of the paper's appendix on low-rank layers, applied to every Monarch form), for narrow
 * layers: it needs 16 | r/nblocks (resp. r_block, r), 32 | n_in/b_in, 32 | b_in r_block and a
 * 32-token tile of X plus its intermediate within LDS. By default the library picks (b) for narrow
 * layers at small and medium token counts, where two launches cost more than their work; these flags
 * force one of them (mutually exclusive; FUSED returns BLR_ERR_UNSUPPORTED where (b) does not apply,
 * and cannot be combined with the stage flags or BLR_MONARCH_IN_BLOCKED). */
#define BLR_MONARCH_FUSED           0x2000u
#define BLR_MONARCH_TWO_KERNELS     0x4000u

/*
 * Monarch forward (paper Section 2.1 "Monarch"; Section 4 "Monarch", optimisations 1-3).
 * With b = nblocks, p = n_in/b, q = n_out/b, r' = r/b:
 *   Z'[t][k][l*r'+rho] = sum_a X[t][l*p+a] * R[l][rho*b+k][a]     (block-diagonal R, permutation folded into the store)
 *   Y[t][o(k,j)]       = sum_m Z'[t][k][m] * L[k][j][m]           (block-diagonal L), o = j*b+k or k*q+j by flags
 * X[T][n_in]; R[b][r][p] (the paper's first stored factor, middle dimension ordered b2-fastest);
 * L[b][q][r] (second stored factor, innermost dimension ordered r'-fastest then b1); Y[T][n_out].
 * r is the width of one middle block (r = r'*b); nblocks must divide n_in, n_out and r.
 * workspace: at least blr_monarch_workspace_bytes(...) bytes (holds Z'; for large interleaved bf16
 * outputs with 8 or more blocks also a blocked-order copy of up to 64 MiB of Y).
 */
size_t     blr_monarch_workspace_bytes(int64_t T, int n_in, int n_out, int nblocks, int r, blr_dtype dt);
blr_status blr_monarch_forward(const void* X, const void* R, const void* L, void* Y,
                               int64_t T, int n_in, int n_out, int nblocks, int r,
                               blr_dtype dt, unsigned flags,
                               void* workspace, size_t workspace_bytes, blr_stream stream);

/*
 * blr_monarch_forward for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments,
 * same kernels and bit-identical results, but the intermediate Z' (and the blocked-order copy of large
 * interleaved outputs) lives in a static device array of BLR_STATIC_SCRATCH_BYTES inside the library,
 * one copy per GPU, held from the moment the library is loaded on that GPU until the process ends. The
 * call allocates nothing and frees nothing. Its first call on a GPU looks the array's address up (the
 * current device must be the one `stream` belongs to).
 * BLR_ERR_WORKSPACE if blr_monarch_workspace_bytes(...) for these sizes exceeds BLR_STATIC_SCRATCH_BYTES
 * (e.g. 4096 x 4096, nblocks = 4, r = 1024 fits up to T = 8192); nothing is enqueued then.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams
 * or host threads) race on it and must be serialised by the caller; calls on one stream are ordered.
 * Nothing in the array has to be zero: every element a call reads was written by the same call.
 */
#define BLR_STATIC_SCRATCH_BYTES (64u << 20)
size_t     blr_static_scratch_bytes(void);
blr_status blr_monarch_forward_static(const void* X, const void* R, const void* L, void* Y,
                                      int64_t T, int n_in, int n_out, int nblocks, int r,
                                      blr_dtype dt, unsigned flags, blr_stream stream);

/*
 * Monarch forward with different block counts on the two sides (paper Section 2.1 "Monarch": the
 * weight is divided into b2 x b1 blocks W_{l,k} = V_{l,k} U_{l,k} of rank r', l < b1 input blocks of
 * p = n_in/b1 features, k < b2 output blocks of q = n_out/b2 features). With b1 = b_in, b2 = b_out,
 * r' = r_block:
 *   Z'[t][k][l*r'+rho] = sum_a X[t][l*p+a] * R[l][rho*b2+k][a]
 *   Y[t][o(k,j)]       = sum_m Z'[t][k][m] * L[k][j][m],   o = j*b2+k (default) or k*q+j (BLR_MONARCH_OUT_BLOCKED)
 * R[b1][r'*b2][p], L[b2][q][b1*r'] (the same two storage orders as blr_monarch_forward, which is the
 * case b1 = b2 = nblocks, r' = r/nblocks). b_in must divide n_in and b_out must divide n_out.
 * flags: BLR_MONARCH_OUT_BLOCKED, BLR_MONARCH_FUSED, BLR_MONARCH_TWO_KERNELS.
 * workspace: at least blr_monarch_rect_workspace_bytes(...) bytes (holds Z', T*b1*b2*r' elements).
 */
size_t     blr_monarch_rect_workspace_bytes(int64_t T, int n_in, int n_out, int b_in, int b_out, int r_block, blr_dtype dt);
blr_status blr_monarch_rect_forward(const void* X, const void* R, const void* L, void* Y,
                                    int64_t T, int n_in, int n_out, int b_in, int b_out, int r_block,
                                    blr_dtype dt, unsigned flags,
                                    void* workspace, size_t workspace_bytes, blr_stream stream);

/*
 * One-time re-layout of a first Monarch factor for BLR_MONARCH_IN_BLOCKED:
 *   Rp[l][c][k*(p/b) + jj] = R[l][c][jj*b + k],  p = n_in/nblocks, b = nblocks, jj < p/b, k < b.
 * R and Rp are [nblocks][r][p] device tensors of type dt and must not overlap.
 * BLR_ERR_INVALID_ARG if nblocks^2 does not divide n_in.
 */
blr_status blr_monarch_permute_first_factor(const void* R, void* Rp, int n_in, int nblocks, int r,
                                            blr_dtype dt, blr_stream stream);

/*
 * One-time re-layout that turns `members` Monarch layers of one shape (n_in, n_out, nblocks, r) which
 * read the same X into ONE layer with b_in = nblocks, b_out = members * nblocks, r_block = r / nblocks
 * for blr_monarch_rect_forward (paper Section 2.1 "Monarch": the general b2 x b1 block form; the q, k, v
 * or gate, up projections of a decoder layer, Section 5). With b = nblocks, r' = r / b:
 *   R_group[l][rho*(members*b) + m*b + k][:] = R_stack[m][l][rho*b + k][:],   m < members.
 * R_stack[members][b][r][p] holds the members' first factors one after the other, R_group is
 * [b][members*r][p]; they must not overlap. The second factors need no re-layout: the members' L one
 * after the other are L_group[members*b][q][r]. Output block m*b + k of the grouped layer is output
 * block k of member m, so with BLR_MONARCH_OUT_BLOCKED member m's result (in its own blocked order)
 * occupies columns m*n_out ... (m+1)*n_out - 1 of Y[T][members*n_out].
 */
blr_status blr_monarch_group_first_factor(const void* R_stack, void* R_group, int n_in, int nblocks, int r, int members,
                                          blr_dtype dt, blr_stream stream);

/*
 * Low-rank forward (paper Section 2.1 "Low-Rank (LR)": W = V U, Y = (X V) U; Section 3 uses it as the
 * compute-bound structured baseline; Appendix "Full Fusion" discusses its single-kernel form):
 *   Z[t][c] = sum_a X[t][a] * V[c][a],   Y[t][o] = sum_c Z[t][c] * U[o][c].
 * X[T][n_in]; V[r][n_in] and U[n_out][r] are the paper's factors stored transposed, so that both
 * contraction indices are contiguous (a one-time offline transposition of static weights);
 * Y[T][n_out]. workspace: at least blr_lowrank_workspace_bytes(...) bytes (holds Z, T*r elements).
 * flags: BLR_MONARCH_FUSED, BLR_MONARCH_TWO_KERNELS. Errors as for the other
 * forwards (BLR_ERR_INVALID_ARG for null factors, non-positive sizes, pointers not 16-byte aligned,
 * unknown flags; BLR_ERR_WORKSPACE; T == 0 returns BLR_OK without launching).
 */
size_t     blr_lowrank_workspace_bytes(int64_t T, int n_in, int n_out, int r, blr_dtype dt);
blr_status blr_lowrank_forward(const void* X, const void* V, const void* U, void* Y,
                               int64_t T, int n_in, int n_out, int r,
                               blr_dtype dt, unsigned flags,
                               void* workspace, size_t workspace_bytes, blr_stream stream);

/*
 * BLAST forward (paper Section 2.1 "BLAST"; Section 4 "BLAST", optimisations 4-5).
 * With q = n_in/b, p = n_out/b:
 *   Z[t][j][rho]  = sum_c X[t][j*q+c] * V[j][c][rho]
 *   A[t][i][rho]  = sum_j S[i][j][rho] * Z[t][j][rho]
 *   Y[t][i*p+a]   = sum_rho A[t][i][rho] * U[i][a][rho]
 * X[T][n_in]; U[b][p][r]; S[b][b][r] indexed [output block i][input block j]; V[b][q][r]; Y[T][n_out].
 * b must divide n_in and n_out. With BLR_BLAST_PACKED, `V` points to the buffer produced by
 * blr_blast_pack for the same (n_in, n_out, b, r), `S` is ignored (may be NULL), `U` is still the
 * canonical tensor (bf16 only). workspace: at least blr_blast_workspace_bytes(...) bytes with the
 * same flags (holds A where a kernel needs it; without BLR_BLAST_PACKED also the per-call re-layout).
 */
size_t     blr_blast_workspace_bytes(int64_t T, int n_in, int n_out, int b, int r, blr_dtype dt, unsigned flags);
blr_status blr_blast_forward(const void* X, const void* U, const void* S, const void* V, void* Y,
                             int64_t T, int n_in, int n_out, int b, int r,
                             blr_dtype dt, unsigned flags,
                             void* workspace, size_t workspace_bytes, blr_stream stream);

/*
 * `members` BLAST layers of one shape (n_in, n_out, b, r) that read the same X, as one call (q, k, v
 * or gate, up of a decoder layer; paper Section 2.1 "BLAST", Section 4 "BLAST"). Stages 1 and 2 of
 * the operator act on every rank index by itself, so the members' rank indices concatenate into one
 * layer of rank members*r there (one pass over X instead of `members`, larger launches); stage 3
 * contracts each member's own range:
 *   Z[t][j][m*r+rho]      = sum_c X[t][j*q+c] * V_m[j][c][rho]
 *   A[t][i][m*r+rho]      = sum_j S_m[i][j][rho] * Z[t][j][m*r+rho]
 *   Y[t][m*n_out+i*p+a]   = sum_rho A[t][i][m*r+rho] * U_m[i][a][rho]
 * X[T][n_in]; U[members][b][p][r]: the members' canonical U stacked; `packed`: the buffer written by
 * blr_blast_pack for (n_in, n_out, b, members*r) from S_g[b][b][members*r] and V_g[b][q][members*r],
 * the members' S and V concatenated along the rank index (U is not read by that call for such a shape:
 * pass the stacked U); Y[T][members*n_out], member m in columns m*n_out ... (m+1)*n_out - 1.
 * bf16 only, 8 | r. flags: BLR_BLAST_FUSED_STAGE12 or BLR_BLAST_THREE_KERNELS (default: the library
 * chooses as for a single layer of rank members*r). workspace: at least
 * blr_blast_group_workspace_bytes(...) bytes with the same flags.
 * BLR_ERR_UNSUPPORTED (workspace query: 0) where the concatenated layer has no matrix-core kernels
 * for stages 1 and 2 or is small enough for the single-kernel path, whose packed form holds no
 * separate stage-1 operand: run such members one by one with blr_blast_forward. Other errors as for
 * blr_blast_forward; T == 0 returns BLR_OK without launching.
 */
size_t     blr_blast_group_workspace_bytes(int64_t T, int n_in, int n_out, int b, int r, int members,
                                           blr_dtype dt, unsigned flags);
blr_status blr_blast_group_forward(const void* X, const void* U, const void* packed, void* Y,
                                   int64_t T, int n_in, int n_out, int b, int r, int members,
                                   blr_dtype dt, unsigned flags,
                                   void* workspace, size_t workspace_bytes, blr_stream stream);

/*
 * One-time re-layout of the static BLAST factors (paper Section 4: weights are static, so their
 * layout is changed once before inference). bf16 only, b <= 16. `packed` is an opaque buffer of
 * blr_blast_packed_bytes(...) bytes that holds
 *   S as one zero-padded 16x16 coupling tile per rank index, Sp[rho][i][j] = S[i][j][rho];
 *   V with the contraction index contiguous, Vt[j][rho][c] = V[j][c][rho]; or, for layers the
 *   single-kernel path serves (r <= 128, n_out/b <= 64), V and U in the register order of the
 *   matrix-core instructions that consume them, so that one load instruction of a wavefront reads
 *   one contiguous kilobyte.
 * The canonical tensors are not modified and are not needed afterwards, except U.
 */
size_t     blr_blast_packed_bytes(int n_in, int n_out, int b, int r, blr_dtype dt);
blr_status blr_blast_pack(const void* U, const void* S, const void* V, void* packed,
                          int n_in, int n_out, int b, int r, blr_dtype dt, blr_stream stream);

/*
 * Dense reference (paper Section 2.1 "Dense"): Y[t][o] = sum_a X[t][a] * W[o][a], W[n_out][n_in].
 * A hand-written GEMM of the same family as the BLR kernels; the denominator of every speed-up.
 */
blr_status blr_dense_reference_forward(const void* X, const void* W, void* Y,
                                       int64_t T, int n_in, int n_out, blr_dtype dt,
                                       unsigned flags, blr_stream stream);

/*
 * Glue between the BLR linears of a decoder-layer chain. The paper replaces the projections and the
 * MLP of Llama decoder layers with BLR linears (Section 5, Llama experiments) and leaves the rest of
 * the layer as it is; the chain benchmark of this library keeps, of that rest, a weightless RMS
 * normalisation, the residual additions and the SiLU gate, and puts the scaled sum of the q/k/v
 * branches where attention would be. All tensors are row-major [T][d] device memory in the storage
 * type dt (arithmetic in fp32), caller-owned; each call enqueues one kernel on `stream` and returns.
 * T == 0 returns BLR_OK without a launch; null pointers, d <= 0, T < 0, negative eps and the aliasings
 * named below return BLR_ERR_INVALID_ARG.
 *
 *   blr_rmsnorm:               N[t][:] = H[t][:] / sqrt(mean_c H[t][c]^2 + eps)          (N must not alias H)
 *   blr_residual_add_rmsnorm:  H += Y (stored back in dt), then N = rmsnorm(H) of the stored values;
 *                              N may be NULL, which leaves the plain residual addition (H, Y, N distinct)
 *   blr_sum3_scaled:           A = (Q + K + V) * scale                                   (A may alias an input)
 *   blr_silu_mul:              M = silu(G) * U, silu(x) = x / (1 + exp(-x))               (M may alias an input)
 */
blr_status blr_rmsnorm(const void* H, void* N, int64_t T, int d, float eps, blr_dtype dt, blr_stream stream);
blr_status blr_residual_add_rmsnorm(void* H, const void* Y, void* N, int64_t T, int d, float eps,
                                    blr_dtype dt, blr_stream stream);
blr_status blr_sum3_scaled(const void* Q, const void* K, const void* V, void* A, int64_t T, int d, float scale,
                           blr_dtype dt, blr_stream stream);
blr_status blr_silu_mul(const void* G, const void* U, void* M, int64_t T, int d, blr_dtype dt, blr_stream stream);
/* The same two operations on inputs whose rows are `ld >= d` elements apart (column slices of a wider
 * tensor: the outputs of several layers that one call computed side by side, see the general Monarch
 * form with b_out = layers * nblocks). The output has contiguous rows of d and must not alias an input. */
blr_status blr_sum3_scaled_ld(const void* Q, const void* K, const void* V, void* A, int64_t T, int d, int64_t ld,
                              float scale, blr_dtype dt, blr_stream stream);
blr_status blr_silu_mul_ld(const void* G, const void* U, void* M, int64_t T, int d, int64_t ld,
                           blr_dtype dt, blr_stream stream);

const char* blr_status_string(blr_status s);

#ifdef __cplusplus
}
#endif
#endif /* BLR_H */
