/*
 * fact.h - C ABI of the MI355X (gfx950) bf16 GEMM + fused-epilogue library
 *          (with the transformer block's fused attention, fact_attention).
 *
 * The library computes what the paper's synthesized kernels compute: dense
 * GEMMs (square, batched, large-K; paper Section 5.1 "Benchmark problems") and
 * the two-GEMM feed-forward patterns with fused activation epilogues (Section
 * 5.2.4 "MLP with GELU", Section 5.2.5 "SwiGLU MLP"), with reduced-precision
 * inputs and an fp32 accumulator (Listing 1: reduced-precision inputs with fp32
 * accumulator).  Here the inputs and outputs are bf16, or IEEE binary16 - the
 * paper's own precision - when fact_epilogue.f16 is set.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     allocates nothing, frees nothing and keeps no pointer after it returns.
 *   - Matrices are row-major; every leading dimension (ld*) and batch stride is
 *     in ELEMENTS, not bytes.
 *   - bf16 = upper 16 bits of IEEE binary32.  Products are accumulated in fp32;
 *     the result is rounded to bf16 once (nearest, ties to even) at the store.
 *   - trans_b == 0: B is [K][N]  (C = A B).
 *     trans_b == 1: B is [N][K]  (C = A B^T, the weight layout of a linear layer).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work
 *     is enqueued on it; the calls do not synchronise, allocate or clear memory, so
 *     they may be captured in a HIP graph and replayed (call each entry point once
 *     outside a capture first: a kernel's first launch on a device sets its LDS
 *     limit).  Two launches that share a workspace must not overlap in time.
 *   - Return value: FACT_OK or a negative fact_status.  Arguments are validated
 *     on the host before anything is launched; on error nothing is launched.  (The
 *     entry points made of several launches, fact_block_mlp and fact_block_forward,
 *     check every stage's arguments, limits and workspace before the first launch;
 *     only a HIP launch failure of a later stage, FACT_ERR_HIP, can leave earlier
 *     stages enqueued.)  No exception crosses the boundary and the library never aborts.
 *   - Aliasing: C may alias `residual` exactly (same pointer, same ld): each
 *     element is read before it is written by the same thread.  Any other overlap
 *     of an output with an input is undefined.
 *   - Shapes: any positive M, N, K.  The MFMA path needs 16-byte aligned A and B
 *     with lda, ldb and K multiples of 8 (and N a multiple of 8 when trans_b == 0);
 *     anything else runs a slower guarded kernel with the same results contract.
 */
#ifndef FACT_H
#define FACT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fact_status {
    FACT_OK = 0,
    FACT_ERR_NULL = -1,         /* a required pointer is NULL */
    FACT_ERR_DIM = -2,          /* a dimension is <= 0 or a leading dimension / stride is too small */
    FACT_ERR_ALIGN = -3,        /* a pointer is not 2-byte aligned (bf16) / workspace not 16-byte aligned */
    FACT_ERR_LAYOUT = -4,       /* trans_b is not 0 or 1, or the layout is not allowed with the epilogue */
    FACT_ERR_EPILOGUE = -5,     /* unknown activation, bias given with the gated epilogue, odd N with it */
    FACT_ERR_WORKSPACE = -6,    /* workspace missing or too small */
    FACT_ERR_UNSUPPORTED = -7,  /* unknown tile configuration id, split factor out of range */
    FACT_ERR_HIP = -8           /* a HIP call failed; text via fact_last_error() */
} fact_status;

typedef enum fact_act {
    FACT_ACT_NONE = 0,
    FACT_ACT_GELU_TANH = 1,     /* 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3)))  (Section 5.2.4: GELU epilogue) */
    FACT_ACT_SILU_GATE = 2      /* SiLU(gate) * up  (Section 5.2.5: gate projection with SiLU, times up projection) */
} fact_act;

/*
 * Fused epilogue, applied in registers in this order:
 *     z = acc + bias[n];  z = act(z);  z = z + residual[m][n];  C[m][n] = bf16(z)   (fp16(z) with f16 = 1)
 * bias     : bf16[Nout] device pointer or NULL.
 * residual : bf16[M][ldr] device pointer or NULL; ldr in elements, >= Nout.
 * act      : a fact_act.  With FACT_ACT_SILU_GATE the GEMM's B must be given with
 *            trans_b == 1 as [N][K] with N even: rows 0..N/2-1 are the gate
 *            weights, rows N/2..N-1 the up weights; the output then has
 *            Nout = N/2 columns and bias must be NULL.  Otherwise Nout = N.
 * In the batched call the residual of batch b starts stride_r elements after
 * that of batch b-1 (stride_r may be 0: one residual shared by all); bias is
 * shared by all batches.
 */
typedef struct fact_epilogue {
    const void *bias;
    const void *residual;
    int64_t ldr;
    int64_t stride_r;
    int32_t act;
    int32_t out_f32;        /* 1: C is fp32 [M][ldc] (ldc and stride_c in fp32 elements, C 4-byte aligned), written
                               without rounding: the paper's choice for its large-K problem (Section 5.2.3: fp32
                               accumulator AND output).  Every entry point takes it; with K whole the GEMM's own
                               epilogue writes the fp32 result, with K split (fact_gemm_splitk / fact_gemm_ex and
                               a workspace of fact_gemm_f32out_workspace_bytes()) the reduction pass does.
                               Shapes or pointers that only the guarded fallback kernel serves: FACT_ERR_UNSUPPORTED. */
    int32_t f16;            /* 1: A, B, bias, residual and C (unless out_f32) hold IEEE binary16 instead of bf16: the
                               precision the paper's own kernels compute in ("fp16 with fp32 accumulator", Listing 1;
                               Sections 5.2.3 - 5.2.5).  Same kernels with the fp16 matrix instruction, fp32
                               accumulation, one rounding to nearest even at the store (overflow gives infinity);
                               same layouts, alignment rules, tile table and error codes.  Taken by fact_gemm,
                               fact_gemm_batched, fact_gemm_splitk(_static) and fact_gemm_ex (and fact_block_mlp_f16
                               is fact_block_mlp with it); fact_attention, fact_norm, fact_rope and
                               fact_block_forward compute in bf16 only.
                               0 (and a NULL epilogue): bf16.  Other values: FACT_ERR_EPILOGUE. */
} fact_epilogue;

/* ---- entry points --------------------------------------------------------------------- */

/*
 * C[M][Nout] = epilogue(A[M][K] x B).  One data-parallel 2-D tiled launch (the paper's
 * "Data Parallel" grid schedule, Section 4.2 Action 2; Section 5.2.1).  ep may be NULL.
 * The tile configuration comes from the per-shape table (the shadow of the paper's
 * registry lookup, Section 4.2 Action 6).
 */
int fact_gemm(int64_t M, int64_t N, int64_t K,
              const void *A, int64_t lda,
              const void *B, int64_t ldb, int trans_b,
              void *C, int64_t ldc,
              const fact_epilogue *ep, void *stream);

/*
 * C[b] = epilogue(A[b] x B[b]) for b in [0, batch): one launch, grid.z = batch
 * (Section 5.1, Problem 3; Section 5.2.2).  Strides are in elements and may be 0 for
 * an operand shared by every batch (not for C).
 */
int fact_gemm_batched(int64_t batch, int64_t M, int64_t N, int64_t K,
                      const void *A, int64_t lda, int64_t stride_a,
                      const void *B, int64_t ldb, int64_t stride_b, int trans_b,
                      void *C, int64_t ldc, int64_t stride_c,
                      const fact_epilogue *ep, void *stream);

/*
 * Large-K GEMM (Section 5.1, Problem 6; Section 5.2.3): K is cut into split_k
 * contiguous ranges, each range's product is written as an fp32 partial into the
 * workspace (fp32 because reduced precision is not enough there, Section 5.2.3), and a
 * second kernel adds the partials in fp32 in a fixed order (the ranges in W consecutive
 * groups of ceil(split_k / W), ascending inside a group, then the W group sums in ascending
 * order; W is 1, 2, 4 or 8, the least that puts some 2048 waves to work on the M x N output
 * with at least four ranges each: a function of M, N and split_k alone), applies the epilogue
 * and rounds once.  split_k == 0 lets the table choose; split_k == 1 (or a
 * choice of 1) runs the plain kernel and needs no workspace.  Bit-reproducible: the
 * order of additions is fixed.
 * ws: device pointer, 16-byte aligned, at least
 * fact_gemm_splitk_workspace_bytes(M, N, K, split_k) bytes; contents are scratch.
 */
int fact_gemm_splitk(int64_t M, int64_t N, int64_t K,
                     const void *A, int64_t lda,
                     const void *B, int64_t ldb, int trans_b,
                     void *C, int64_t ldc,
                     const fact_epilogue *ep,
                     int split_k, void *ws, size_t ws_bytes, void *stream);

/*
 * fact_gemm_splitk for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  Same arguments, same results (bit for
 * bit) and same error codes as fact_gemm_splitk, without ws / ws_bytes: the fp32 partial sums (or
 * the hand-over tiles of a tail split) live in a static device array inside the library, of
 * fact_gemm_splitk_static_capacity() bytes (32 MiB: 128 K ranges of a 256 x 256 problem).  Every
 * GPU the library runs on holds its own copy of the array until the process ends.  The call
 * allocates nothing and frees nothing; a call that would need more than the array holds returns
 * FACT_ERR_WORKSPACE (fact_last_error says how much) and launches nothing.  All calls on one GPU
 * share that GPU's array and it keeps the last call's contents (every byte a call reads it has
 * written itself first, so nothing needs clearing): calls that overlap in time on one GPU, on
 * any streams, race.  The array's device address is looked up on the first call on a device (or
 * by fact_gemm_splitk_static_init with that device current, e.g. before a capture begins).
 */
int fact_gemm_splitk_static(int64_t M, int64_t N, int64_t K,
                            const void *A, int64_t lda,
                            const void *B, int64_t ldb, int trans_b,
                            void *C, int64_t ldc,
                            const fact_epilogue *ep,
                            int split_k, void *stream);
int fact_gemm_splitk_static_init(void);          /* FACT_OK, or FACT_ERR_HIP / FACT_ERR_UNSUPPORTED (device index >= 64) */
size_t fact_gemm_splitk_static_capacity(void);   /* bytes of the static array */

/* Bytes of workspace fact_gemm_splitk needs for this shape and split_k (0 = the table's
 * choice, which may also be a tail split, see fact_gemm_ex; negative = a forced tail split
 * of -split_k ranges, largest need over the tile configurations).  Returns 0 when no
 * workspace is needed or the arguments are invalid. */
size_t fact_gemm_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, int split_k);
/* Workspace of the same call with ep->out_f32 = 1: the fp32 partial planes when K is split
 * (split_k > 1, or 0 and the table splits this shape), else 0. */
size_t fact_gemm_f32out_workspace_bytes(int64_t M, int64_t N, int64_t K, int split_k);

/*
 * Two-GEMM feed-forward block (pattern p2 of Sections 5.2.4 and 5.2.5), two launches
 * on one stream:
 *     H = act(X W1^T + b1)      bf16 [T][d_ff], written to the caller's H buffer
 *     Y = H W2^T + b2 + R       bf16 [T][d_model]
 * X  : bf16 [T][d_model].        W1 : bf16 [d_ff][d_model].
 * W1u: with FACT_ACT_SILU_GATE, the up-projection weights bf16 [d_ff][d_model] and W1 is
 *      the gate projection; must be NULL otherwise.
 * b1 : bf16 [d_ff] or NULL (must be NULL with FACT_ACT_SILU_GATE).
 * W2 : bf16 [d_model][d_ff].     b2 : bf16 [d_model] or NULL.
 * R  : residual bf16 [T][d_model] or NULL (Y may alias R).
 * All matrices dense (leading dimension = row length).
 * ws : workspace for a split-K second GEMM or a tail split of either GEMM,
 *      fact_block_mlp_workspace_bytes() bytes (may be NULL when that returns 0).
 */
int fact_block_mlp(int64_t T, int64_t d_model, int64_t d_ff,
                   const void *X, const void *W1, const void *W1u, const void *b1, int act,
                   const void *W2, const void *b2, const void *R,
                   void *H, void *Y, void *ws, size_t ws_bytes, void *stream);

/* The same block with every 16-bit tensor (X, the weights and biases, R, H, Y) in IEEE binary16, the
 * precision the paper runs its two blocks in (Sections 5.2.4 and 5.2.5: fp16 compute, fp32 accumulator).
 * Same arguments, workspace size, launches and error codes as fact_block_mlp. */
int fact_block_mlp_f16(int64_t T, int64_t d_model, int64_t d_ff,
                       const void *X, const void *W1, const void *W1u, const void *b1, int act,
                       const void *W2, const void *b2, const void *R,
                       void *H, void *Y, void *ws, size_t ws_bytes, void *stream);

size_t fact_block_mlp_workspace_bytes(int64_t T, int64_t d_model, int64_t d_ff, int act);

/*
 * Fused multi-head self-attention (pattern p1 of Sections 5.2.4 and 5.2.5; tiled over keys so
 * that the score matrix stays on chip, Section 2.1), one launch:
 *     O[b,i,h,:] = sum_j softmax_j( scale * Q[b,i,h,:] . K[b,j,g,:] ) V[b,j,g,:],   g = h / (n_q_heads / n_kv_heads)
 * with j <= i only when causal == 1 (a query sees itself and earlier tokens) and all j < T when
 * causal == 0.  Grouped-query attention (n_kv_heads < n_q_heads, Section 5.2.5) is read in place:
 * consecutive query heads share a key/value head, nothing is expanded in memory.
 * Q, O : bf16 [batch][T][n_q_heads][head_dim];  K, V : bf16 [batch][T][n_kv_heads][head_dim].
 * Each tensor comes with three ELEMENT strides {batch entry, token, head} (host arrays of 3);
 * the head_dim elements of one (batch, token, head) row are contiguous.  This takes the output
 * of a fused QKV projection as it lies in memory: for rows of [q heads | k heads | v heads],
 * pass Q = base, K = base + n_q_heads*head_dim, V = K + n_kv_heads*head_dim, token stride =
 * (n_q_heads + 2 n_kv_heads) * head_dim, head stride = head_dim.
 * head_dim must be 64 or 128 (else FACT_ERR_UNSUPPORTED).  Q, K, V: 16-byte aligned, strides
 * multiples of 8, token stride >= head_dim, (T + 512) * token stride < 2^30; O: 8-byte aligned,
 * strides multiples of 4.  n_q_heads must be a multiple of n_kv_heads.
 * scale: the softmax scale; <= 0 selects 1 / sqrt(head_dim).
 * Arithmetic: scores and softmax in fp32 (base-2 exponentials), probabilities rounded to bf16
 * for the second contraction, fp32 accumulation, one rounding to bf16 at the store.
 * O must not overlap Q, K or V.
 */
int fact_attention(int64_t batch, int64_t T, int64_t n_q_heads, int64_t n_kv_heads, int64_t head_dim,
                   const void *Q, const int64_t *q_strides, const void *K, const int64_t *k_strides,
                   const void *V, const int64_t *v_strides, void *O, const int64_t *o_strides,
                   int causal, float scale, void *stream);

/*
 * Row normalisation, one memory-bound launch (the blocks of Section 5.1: LayerNorm in the GPT-style
 * block, RMSNorm in the Llama block):
 *   rms == 0 (LayerNorm): y = (x - mean(x)) / sqrt(var(x) + eps) * gamma + beta   (beta may be NULL)
 *   rms == 1 (RMSNorm):   y = x / sqrt(mean(x^2) + eps) * gamma                   (beta must be NULL)
 * X, Y: bf16 [T][d] with leading dimensions ldx, ldy (elements); gamma, beta: bf16 [d].  Statistics
 * in fp32 (two passes over the row held in registers), one rounding to bf16.  d must be a multiple
 * of 8 and <= 8192, pointers 16-byte aligned, leading dimensions multiples of 8
 * (FACT_ERR_UNSUPPORTED / FACT_ERR_ALIGN otherwise).  Y may alias X.
 */
int fact_norm(int64_t T, int64_t d, const void *X, int64_t ldx, const void *gamma, const void *beta, float eps, int rms,
              void *Y, int64_t ldy, void *stream);

/*
 * Rotary position embedding, in place, "rotate-half" pairing (the Llama block of Section 5.1):
 * for head width D, i < D/2 and token position t (0-based in its batch entry),
 *   angle = t * base^(-2 i / D),  (x_i, x_{i+D/2}) <- (x_i cos - x_{i+D/2} sin, x_{i+D/2} cos + x_i sin).
 * X: bf16 [batch][T][n_heads][head_dim] with element strides {batch, token, head} (host array of 3);
 * for a packed QKV buffer pass n_heads = query heads + key heads (they are adjacent).  head_dim a
 * multiple of 16, 16-byte aligned, strides multiples of 8, base > 1.  fp32 arithmetic, one rounding.
 */
int fact_rope(int64_t batch, int64_t T, int64_t n_heads, int64_t head_dim, void *X, const int64_t *strides, float base,
              void *stream);

/*
 * A whole pre-norm decoder block from this library's entry points (the composition step of
 * Section 4.3 applied to the two blocks of Section 5.1; every stage runs on the GPU):
 *     N1  = norm(X);  QKV = N1 Wqkv^T + bqkv;  rotary on the q and k heads (if rope);
 *     A   = causal attention(QKV);  X1 = A Wo^T + bo + X;
 *     N2  = norm(X1);  H = act(N2 W1^T + b1)  [or SiLU(N2 W1^T) * (N2 W1u^T)];  Y = H W2^T + b2 + X1.
 * X, Y: bf16 [batch * tokens][d_model], dense.  Wqkv: [(n_q_heads + 2 n_kv_heads) head_dim][d_model],
 * rows ordered query heads, key heads, value heads; Wo: [d_model][n_q_heads head_dim]; W1 (and
 * W1u with FACT_ACT_SILU_GATE): [d_ff][d_model]; W2: [d_model][d_ff].  Biases and norm1_b / norm2_b may
 * be NULL; norm_rms == 1 ignores them.  eps <= 0 selects 1e-5, rope_base <= 1 selects 500000.
 * Every intermediate is stored as bf16 in `scratch` (fact_block_scratch_bytes() bytes, 256-byte
 * aligned, contents scratch); fact_block_scratch_offsets() writes the byte offsets of
 * {N1, QKV (after the rotary step), A, X1, N2, H, GEMM workspace} for inspection.
 * Nine launches on `stream` (ten with the rotary step), no synchronisation.
 */
typedef struct fact_block {
    int64_t batch, tokens, d_model, n_q_heads, n_kv_heads, head_dim, d_ff;
    int32_t norm_rms;            /* 1: RMSNorm, 0: LayerNorm */
    int32_t act;                 /* FACT_ACT_GELU_TANH, FACT_ACT_SILU_GATE or FACT_ACT_NONE */
    int32_t rope;                /* 1: rotary embedding on q and k */
    float eps, rope_base;
    const void *norm1_g, *norm1_b, *Wqkv, *bqkv, *Wo, *bo, *norm2_g, *norm2_b, *W1, *W1u, *b1, *W2, *b2;
} fact_block;

size_t fact_block_scratch_bytes(const fact_block *blk);                  /* 0 if the description is invalid */
int fact_block_scratch_offsets(const fact_block *blk, size_t *offsets /* [7] */);
int fact_block_forward(const fact_block *blk, const void *X, void *Y, void *scratch, size_t scratch_bytes, void *stream);

/* ---- tile configurations: the auto-tuning surface (Section 4.2 Action 5) ---------------- */

/* Number of compiled tile configurations; ids are 0 .. fact_num_configs()-1. */
int fact_num_configs(void);

/* Describes configuration `id`: macro-tile rows/cols, waves along M and N, LDS bytes.
 * Any out pointer may be NULL.  Returns FACT_ERR_UNSUPPORTED for a bad id. */
int fact_config_info(int id, int *tile_m, int *tile_n, int *waves_m, int *waves_n, int *lds_bytes);

/* The table's choice for a shape (host logic only, no GPU needed): writes the tile
 * configuration id and the split-K factor (>= 1; -g for a tail split of g ranges, see
 * fact_gemm_ex).  batch >= 1.  Returns FACT_OK, or an
 * error if the shape is invalid.  config_id is -1 when the shape can only run on the
 * guarded fallback kernel (unaligned dimensions). */
int fact_select_config(int64_t batch, int64_t M, int64_t N, int64_t K, int trans_b, int act,
                       int *config_id, int *split_k);

/* ---- the persisted registry (Section 3: entries keyed by rule, data type and architecture;
 *      Section 4.2 Action 6: tuning results written back; Section 4.3: later lookups reuse them) -- */

/*
 * Loads tuning results from a registry file and consults them before the compiled-in table
 * (which is generated from the file shipped with the library).  Text, one entry per line:
 *
 *     # fact-registry 1
 *     gemm bf16 gfx950 <batch> <M> <N> <K> <kn|nk> <plain|gated> <config> <split_k> <group_m> [<ms> <TFLOP/s> <build> <name>]
 *
 * kn / nk: B as [K][N] (trans_b = 0) / as [N][K] (trans_b = 1); N counts the contraction's columns
 * (2 x d_ff when gated); split_k as in fact_gemm_ex (1, > 1, or -g); the trailing fields are
 * provenance and are not interpreted.  '#' lines other than the format line are comments.
 * Entries of another rule, data type or architecture, and entries naming a configuration this
 * build does not have (or one that cannot serve the layout), are skipped.  Of several entries for
 * one shape the first applies; a call that brings no workspace takes the first one with
 * split_k == 1.  Host only, callable from any thread; affects calls made after it returns.
 * path: host pointer to a NUL-terminated file name, read during the call, not kept.
 * Returns the number of entries taken (>= 0), FACT_ERR_NULL for a NULL path,
 * FACT_ERR_UNSUPPORTED if the file cannot be read or is not a version-1 registry.
 */
int fact_registry_load(const char *path);
void fact_registry_clear(void);               /* forgets every loaded entry; the compiled-in table stays */
int fact_registry_size(void);                 /* entries currently loaded */

#define FACT_CONFIG_TABLE   (-1)   /* config_id: the table's choice */
#define FACT_CONFIG_GUARDED (-2)   /* config_id: the guarded one-thread-per-element kernel, whatever the shape (no K split,
                                      no fp32 output): the product-side reference result of the on-device sweep */

/*
 * fact_gemm_batched with the tile configuration, split factor and tile-row group size
 * forced: the entry point the on-device sweep uses.  config_id == FACT_CONFIG_TABLE, split_k == 0 and
 * group_m <= 0 mean "table's choice".  split_k > 1 needs ws (see fact_gemm_splitk) and
 * batch == 1.
 * split_k = -g (g >= 2) asks for a tail split, this library's form of the paper's Stream-K
 * fix-up (Section 4.2 Action 2, Section 5.2.3): tiles are computed whole as long as they fill
 * all compute units; the tiles of the last, partly filled round are shared by g work-groups
 * each, one K range apiece, which hand their fp32 partial tiles to the one holding the last
 * range through ws; that one adds them in ascending range order (bit-reproducible) and runs
 * the epilogue.  Needs batch == 1 and fact_gemm_splitk_workspace_bytes(M, N, K, -g) bytes of
 * ws (contents are scratch and need no clearing).  FACT_ERR_UNSUPPORTED if the shape has no
 * partly filled round or too little K per range.  A configuration whose LDS or alignment needs the shape cannot meet
 * returns FACT_ERR_UNSUPPORTED (recorded by the sweep as a launch failure, as in
 * Section 5.1 "Auto-tuning methodology").
 */
int fact_gemm_ex(int64_t batch, int64_t M, int64_t N, int64_t K,
                 const void *A, int64_t lda, int64_t stride_a,
                 const void *B, int64_t ldb, int64_t stride_b, int trans_b,
                 void *C, int64_t ldc, int64_t stride_c,
                 const fact_epilogue *ep,
                 int config_id, int split_k, int group_m,
                 void *ws, size_t ws_bytes, void *stream);

/*
 * Tail split hand-over, failure reporting.  The work-group that finishes a shared tile waits for
 * its partners' partial sums (Section 5.2.3: the fix-up step of a K-partitioned tile).  Partners
 * are dispatched first and never wait, so the wait ends unless the GPU is shared with work that
 * keeps them from running; it is bounded all the same (about a third of a second).  A wait that
 * gives up is an error, never a quietly wrong tile: every element of that tile is written as NaN,
 * and the launch's identity is stored in the first word of the workspace (the workspace layout
 * is: a 256-byte status block, the partial tiles, the hand-over flags).
 * fact_tail_timeouts synchronizes `stream`, reads that word (a blocking device-to-host copy) and
 * sets *gave_up to 1 if any tail-split launch of this process that used `ws` gave up since the
 * word was last overwritten by other data, else to 0.  After a reported failure the hand-over
 * flags are in an undefined state: clear the workspace (or take a fresh one) before it serves a
 * captured graph again.  ws: the device pointer handed to fact_gemm_splitk / fact_gemm_ex /
 * fact_block_mlp (16-byte aligned); gave_up: host pointer.  Returns FACT_OK, FACT_ERR_NULL,
 * FACT_ERR_ALIGN or FACT_ERR_HIP.  Not capturable (it synchronizes).
 */
int fact_tail_timeouts(const void *ws, void *stream, int *gave_up);

/* Test hook: the number of polls a finishing work-group spends waiting (default 2^20); a negative
 * value makes it give up at once, which exercises the failure path above deterministically while
 * every kernel still runs to its end.  Process-wide, applies to launches made after the call. */
void fact_test_tail_poll_budget(int polls);

/*
 * Persistent launches (the grid-level schedule of Section 4.2 Action 2 next to "Data Parallel" and
 * "Split-K"; Section 5.2.3 describes the persistent Stream-K form).  With mode 1, a launch with K
 * whole and a 4-wave tile configuration that has more tiles (times batch entries) than the GPU holds
 * work-groups at once launches as many work-groups as fit, and each walks several tiles in the
 * XCD-aware order; the first operand stages of a work-group's next tile are requested before the
 * epilogue of the tile in hand runs.  Results are bit-identical either way.  Default: mode 0, one
 * work-group per tile everywhere - on this chip the persistent form measured 0.5-3 % slower on the
 * benchmark shapes (what the overlap saves per tile, the state carried from tile to tile costs).
 * Process-wide, applies to launches made after the call; returns the previous mode.
 */
int fact_tune_persistent(int mode);
/* Work-groups a launch of this problem with K whole uses when it is persistent, else 0 (config_id < 0:
 * the table's or the model's configuration; 0 as well when that choice splits K). */
int fact_persistent_grid(int64_t batch, int64_t M, int64_t N, int64_t K, int trans_b, int act, int config_id);

/* ---- misc ------------------------------------------------------------------------------- */

const char *fact_status_string(int status);   /* static string, never NULL */
const char *fact_last_error(void);            /* text of the last HIP failure on this thread, "" if none */
int fact_version(void);                       /* major*10000 + minor*100 + patch */

#ifdef __cplusplus
}
#endif
#endif /* FACT_H */
