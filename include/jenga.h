/*
 * jenga.h - C ABI of the MI355X (gfx950) attention-carving library.
 *
 * The library computes, for one attention layer of a video diffusion transformer, the
 * block-sparse self-attention of "Training-Free Efficient Video Generation via Dynamic Token
 * Carving" (Sec. 3.1 "Block-Wise Attention Carving", appendix Alg. 2-4):
 *
 *   jenga_curve_permute     z_blk = G(z_thw)                      Eq. 2
 *   jenga_select_blocks     B = B_top u B_cond u B_adja           Eq. 3, Alg. 3, appendix Eq. 5
 *   jenga_block_sparse_attn O = attention over the blocks of B    Alg. 4, Alg. 2, Eq. 1
 *   jenga_unpermute         z_thw = G^-1(z_blk)                   Eq. 2
 *   jenga_stage_switch      resolution switch between stages      Eq. 4
 *
 * Conventions
 *   - All tensor arguments are DEVICE pointers unless a comment says "host".  The caller owns
 *     every tensor and every workspace; the library owns only what is inside a jenga_plan.
 *   - bf16 tensors are raw 16-bit bfloat16 bit patterns.
 *   - "thw side" layout:   [batch][N_v + N_c][heads][head_dim]   vision tokens in (t,h,w)
 *     row-major order (w fastest) followed by the N_c text tokens.
 *   - "curve side" layout: [batch][heads][N_pad][head_dim]       sequence positions are
 *     [vision in curve order | pad to M_v*m | text | pad to M_c*m]; N_pad = M*m, M = M_v + M_c.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  The four hot calls
 *     only enqueue work: no allocation, no host synchronisation, no host<->device copies.
 *   - Every function returns JENGA_OK (0) or a negative jenga_status; nothing is thrown across
 *     the ABI and nothing is launched when validation fails.
 *   - One GPU: a plan belongs to the device that was current when it was created; a call that uses
 *     the plan's device tables with another device current returns JENGA_EINVAL.
 */
#ifndef JENGA_H_
#define JENGA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  JENGA_OK = 0,
  JENGA_EINVAL = -1,       /* null pointer, non-positive size, ratio out of range            */
  JENGA_EUNSUPPORTED = -2, /* head_dim / block / sequence length outside what is built       */
  JENGA_EWORKSPACE = -3,   /* workspace smaller than jenga_plan_info reports                 */
  JENGA_EHIP = -4,         /* a HIP runtime call or a kernel launch failed                   */
  JENGA_ENOMEM = -5        /* host or device allocation failed while creating a plan         */
} jenga_status;

enum {
  JENGA_FLAG_ADJACENCY = 1u, /* union with B_adja (Sec. 3.1 item 3)                          */
  JENGA_FLAG_CONDITION = 2u, /* union with B_cond: all text key blocks (Sec. 3.1 item 2)      */
  JENGA_FLAG_CURVE = 4u,     /* 1: generalized Hilbert order; 0: linear thw order (ablation)  */
  JENGA_FLAG_PACED_WALK = 8u /* attention with blocks of 128 tokens visits the selected key blocks in an
                                order paced by a chip-wide clock instead of list order, so that the
                                workgroups of an XCD share tiles in the L2 (Alg. 4 sums over a set: the
                                order is free).  Faster; the last bits of the output may differ between
                                runs; a block listed twice is visited once.  Ignored for other block sizes */
};

/* Problem statement of one layer (Sec. 3.1; Alg. 2 and Alg. 3 inputs). */
typedef struct {
  int32_t T, H, W;     /* latent grid, each >= 1; N_v = T*H*W vision tokens.  A layer without vision
                          tokens (the text-only branch of Alg. 2) is plain dense attention and is not
                          taken: JENGA_EINVAL                                                  */
  int32_t n_text;      /* N_c >= 0 condition tokens, stored behind the vision tokens           */
  int32_t batch;       /* >= 1                                                                 */
  int32_t heads;       /* >= 1                                                                 */
  int32_t head_dim;    /* d_k: 64 or 128                                                       */
  int32_t block;       /* m: 32, 64 or 128 tokens per block                                    */
  double topk_ratio;   /* k in (0, 1]: keep at least K_top = max(1, floor(k*M_v + 1e-6)) blocks */
  double cum_prob;     /* p in [0, 1): extend until the kept probability mass exceeds p         */
  float text_bias;     /* beta of the text-attention amplifier (Sec. 3.2), added to the scaled
                          logits of vision-query x text-key pairs; 0 switches it off; must be
                          finite (NaN or +-inf: JENGA_EINVAL)                                  */
  uint32_t flags;      /* JENGA_FLAG_*                                                         */
} jenga_config;

/* Sizes derived from a config (all counts in tokens or blocks, workspaces in bytes). */
typedef struct {
  int32_t N_v, M_v, M_c, M, N_pad, pad_v, pad_c, K_top;
  uint64_t select_workspace_bytes; /* for jenga_select_blocks                                  */
  uint64_t attn_workspace_bytes;   /* for jenga_block_sparse_attn                              */
} jenga_plan_info_t;

typedef struct jenga_plan jenga_plan; /* opaque, library-owned */

/*
 * Host precompute for one grid (Alg. 1 step "compute block reordering G, G^-1 and adjacency
 * masks"; Sec. 3.1: B_cond and B_adja depend only on the resolution and on G).  Builds the curve
 * permutation, the padded layout and the adjacency bit mask on the host, copies them to the
 * current device (synchronous) and returns the plan in *out.  cfg and out are host pointers.
 */
int jenga_plan_create(const jenga_config* cfg, jenga_plan** out);

/* Frees the device tables and the plan.  NULL is accepted. */
int jenga_plan_destroy(jenga_plan* plan);

/* Fills *info (host pointer). */
int jenga_plan_info(const jenga_plan* plan, jenga_plan_info_t* info);

/*
 * Copies the plan's tables to HOST arrays for inspection; any pointer may be NULL.
 *   perm[N_v]      thw index of the token at curve position i        (Eq. 2)
 *   inv_perm[N_v]  curve position of thw index n
 *   adja[M_v*M_v]  1 where blocks i and j hold tokens within Chebyshev distance 1 (Sec. 3.1)
 */
int jenga_plan_export(const jenga_plan* plan, int32_t* perm, int32_t* inv_perm, uint8_t* adja);

/*
 * Host-only form of create + info + export: computes the same tables without touching a device
 * (no plan is kept).  cfg and info are host pointers; perm, inv_perm, adja as in
 * jenga_plan_export, any of them may be NULL.  Same validation and status codes as create.
 */
int jenga_plan_tables(const jenga_config* cfg, jenga_plan_info_t* info, int32_t* perm, int32_t* inv_perm,
                      uint8_t* adja);

/*
 * Eq. 2, z_blk = G(z_thw), fused with the change of layout:
 *   dst_curve[b][h][i][:] = src_thw[b][src(i)][h][:]    for every valid position i, 0 for pads.
 * src_thw: bf16 thw side, read only.  dst_curve: bf16 curve side, fully overwritten.
 */
int jenga_curve_permute(const jenga_plan* plan, const void* src_thw, void* dst_curve, void* stream);

/*
 * Eq. 2 applied to a per-token table that has to follow the tokens into curve order, such as the
 * rotary position-embedding frequencies (appendix, implementation details, "Frequency re-ordering":
 * f_blk = G(f); Alg. 1, the step that remaps the positional frequencies once per stage):
 *   dst_rows[i][:] = src_rows[src(i)][:]   for every valid position i, 0 for pads.
 * src_rows: [N_v + N_c][row_bytes] bytes in thw order (text rows last), read only.
 * dst_rows: [N_pad][row_bytes], fully overwritten.  Both 16-byte aligned.
 * row_bytes: a power of two in [16, 4096] (e.g. 128 float32 = 512), else JENGA_EUNSUPPORTED.
 * The batch and heads of the plan play no part.
 */
int jenga_curve_permute_rows(const jenga_plan* plan, const void* src_rows, void* dst_rows, int32_t row_bytes,
                             void* stream);

/*
 * Alg. 3 with Alg. 2's rule for text queries.  For every (batch, head, query block i):
 *   i < M_v : mean-pool Q and K per block over their valid tokens (Eq. 3), R = softmax over all M
 *             key blocks of Q^.K^/sqrt(d_k); order by (R descending, index ascending);
 *             N_k = min(M, max(#{n : C_n <= p} + 1, K_top)) with C the running sum; keep the
 *             first N_k; union with the text key blocks and the adjacent blocks per the flags.
 *   i >= M_v: every block.
 * The arithmetic is float64 so that the integer decisions do not depend on summation order
 * beyond 1e-15 relative.
 *   q_curve, k_curve : bf16 curve side, read only (pad rows are ignored, not assumed zero)
 *   sel_count        : int32 [batch][heads][M]       number of selected key blocks
 *   sel_index        : int32 [batch][heads][M][M]    their indices, ascending; entries at and
 *                      beyond sel_count are left untouched
 *   mask_or_null     : uint8 [batch][heads][M][M]    dense 0/1 copy of B, or NULL
 *   workspace        : at least select_workspace_bytes, 256-byte aligned, contents undefined after
 */
int jenga_select_blocks(const jenga_plan* plan, const void* q_curve, const void* k_curve,
                        int32_t* sel_count, int32_t* sel_index, uint8_t* mask_or_null,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * jenga_select_blocks for callers that cannot allocate or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same computation, same outputs, same kernels; the
 * workspace is a static device array of JENGA_SELECT_STATIC_MAX_BYTES inside the library (one per GPU, resident
 * from module load until the process ends).  The call allocates nothing and frees nothing.
 *   - JENGA_EWORKSPACE when the plan's select_workspace_bytes exceeds JENGA_SELECT_STATIC_MAX_BYTES
 *     (nothing is launched); JENGA_EINVAL for null pointers or when the current device is not the plan's.
 *   - All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different
 *     streams, different threads) race on it and must be serialised by the caller.  The array keeps the
 *     last call's contents; the kernels overwrite everything they read, so no clearing is needed.
 */
#define JENGA_SELECT_STATIC_MAX_BYTES (64u << 20)
int jenga_select_blocks_static(const jenga_plan* plan, const void* q_curve, const void* k_curve,
                               int32_t* sel_count, int32_t* sel_index, uint8_t* mask_or_null, void* stream);

/*
 * Alg. 4 (and Alg. 2's dense rows for text queries, which simply carry a full index list).
 * For query block i of (batch, head): softmax attention of its valid rows over the valid keys of
 * the blocks sel_index[..][i][0 .. sel_count), logits q.k/sqrt(d_k) (+ text_bias for a vision
 * query block and a text key block), bf16 MFMA products with float32 accumulation and float32
 * online softmax.  Pad query rows produce zeros.
 *   q, k, v    : bf16 curve side, read only
 *   sel_count, sel_index : as written by jenga_select_blocks.  Counts are clamped to [0, M] and
 *                indices to [0, M) on the device, so a malformed list cannot cause an access
 *                out of range; a count of 0 gives zero rows.  The order of a list does not matter
 *                beyond rounding (any permutation of the same blocks is accepted)
 *   out_curve  : bf16 curve side, fully overwritten
 *   lse_or_null: float32 [batch][heads][N_pad] or NULL.  For every valid query row the natural
 *                logarithm of the sum of exp(logit) over the keys it visited (logits scaled and
 *                biased as above): Alg. 4's running maximum and running sum combined, the value a
 *                caller needs to merge this result with attention over other keys.  Pad query rows
 *                and rows of an empty list get -inf.  Fully overwritten when given
 *   workspace  : at least attn_workspace_bytes, 256-byte aligned (K and V re-tiled for the
 *                matrix cores, and 256 bytes of launch parameters), contents undefined after
 * Equivalent to jenga_pack_kv followed by jenga_block_sparse_attn_packed on the same workspace.
 */
int jenga_block_sparse_attn(const jenga_plan* plan, const void* q, const void* k, const void* v,
                            const int32_t* sel_count, const int32_t* sel_index, void* out_curve,
                            float* lse_or_null, void* workspace, size_t workspace_bytes, void* stream);

/*
 * First half of jenga_block_sparse_attn: re-tiles K and V of every block (Alg. 4's "load key-value
 * block") into the matrix-core fragment order inside `workspace`; pad rows of V are zeroed.
 * A caller that attends several times to the same K and V (a sweep of k or p) packs once.
 */
int jenga_pack_kv(const jenga_plan* plan, const void* k, const void* v, void* workspace,
                  size_t workspace_bytes, void* stream);

/*
 * Second half of jenga_block_sparse_attn: the block-sparse attention kernel itself, reading K and V
 * from a workspace filled by jenga_pack_kv for the same plan.  The packed tiles are only read; the last
 * 256 bytes of the workspace (launch parameters) may be written.  Other arguments as above.
 */
int jenga_block_sparse_attn_packed(const jenga_plan* plan, const void* q, void* packed_kv_workspace,
                                   size_t workspace_bytes, const int32_t* sel_count,
                                   const int32_t* sel_index, void* out_curve, float* lse_or_null,
                                   void* stream);

/*
 * Eq. 2, z_thw = G^-1(z_blk): dst_thw[b][src(i)][h][:] = src_curve[b][h][i][:] for every valid
 * position i; pad rows are dropped.  dst_thw is fully overwritten.
 */
int jenga_unpermute(const jenga_plan* plan, const void* src_curve, void* dst_thw, void* stream);

/*
 * Progressive-resolution stage switch (Sec. 3.2, Eq. 4), one fused elementwise pass:
 *   x_out = (1 - sigma_t) * U(x_t - sigma_t * eps_t) + sigma_t * eps_tilde
 * U is 3D area interpolation from (T_in, H_in, W_in) to (T_out, H_out, W_out): along each axis with I
 * input and O output cells, output cell o is the unweighted mean of input cells
 * floor(o*I/O) .. ceil((o+1)*I/O) - 1 (for integer factors: replication); any sizes >= 1 are accepted,
 * also smaller outputs.
 *   x_t, eps_t : float32 [channels][T_in][H_in][W_in]   latent and the model's prediction at step t (batch
 *                folded into channels), read only
 *   eps_tilde  : float32 [channels][T_out][H_out][W_out] standard-normal draw supplied by the caller
 *   x_out      : float32 [channels][T_out][H_out][W_out], fully overwritten; must not alias the inputs
 *   sigma_t    : scheduler noise level in [0, 1]
 * No plan is needed.  float32 arithmetic, window sums in (t, h, w) order.  Only enqueues work on `stream`.
 * JENGA_EINVAL for null pointers, sizes < 1 or sigma_t outside [0, 1] (NaN included); JENGA_EUNSUPPORTED
 * when an extent exceeds 2^14 or the output has more than 2^32 rows or 2^34 cells.
 */
int jenga_stage_switch(const float* x_t, const float* eps_t, const float* eps_tilde, float* x_out,
                       int32_t channels, int32_t T_in, int32_t H_in, int32_t W_in, int32_t T_out,
                       int32_t H_out, int32_t W_out, float sigma_t, void* stream);

/* Static, NUL-terminated description of a status code. */
const char* jenga_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* JENGA_H_ */
