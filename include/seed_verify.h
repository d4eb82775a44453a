/*
 * seed_verify.h -- C ABI of the MI355X (gfx950) library for the batched target-model verification
 * step of scheduled speculative decoding on a reasoning tree.
 *
 * What one verify step computes (paper Section 3.1 "Speculative Decoding", Section 3.4 Algorithm 1,
 * verification process, and Appendix "Batch Inference": one verified draft sequence per batch entry):
 *   for each of N draft branches, the target model scores the branch's gamma draft tokens in a single
 *   forward pass over (shared prefix + branch-private context + pending token + drafts), then every
 *   draft token is accepted with probability min(1, p_t/p_d) from left to right, and on the first
 *   rejection one replacement token is drawn from the normalised max(0, p_t - p_d).
 *
 * Conventions common to every entry point
 *   - All array arguments are DEVICE pointers owned by the caller (any allocator, e.g. a PyTorch
 *     tensor's data_ptr) unless the comment says "host".  Scalars and the argument structs themselves
 *     live on the host and are read before the call returns.
 *   - Calls only enqueue work on the HIP stream given at init (or passed explicitly); they never
 *     synchronise the device.  Outputs are valid once the caller has synchronised that stream.
 *   - Return value: SEED_OK (0) or a negative SEED_E_* code; seed_last_error() gives a thread-local
 *     human-readable message for the last failing call.  Argument errors are detected before any
 *     kernel is launched.  Nothing throws or aborts across this boundary.
 *   - Same inputs give bit-identical outputs from run to run (no floating-point atomics).
 *   - Matrices are row-major [out][in].  dtype 0: float32 weights and KV cache; dtype 1: bfloat16
 *     weights and KV cache; dtype 2: as 1, but the seven projection matrices of every layer and the LM head are
 *     given as OCP e4m3 codes (uint8: sign, 4 exponent bits of bias 7, 3 mantissa bits, no infinities; the code
 *     0x7f / 0xff is not a number and must not occur) with one float32 scale per output row, W[o][i] =
 *     scale[o] * value(code[o][i]): half the bytes of the weight stream that bounds a step.  Embedding, RMSNorm
 *     gains and the KV cache stay bfloat16.  Logits, probabilities and uniforms are always float32; token ids
 *     and lengths are int32.
 */
#ifndef SEED_VERIFY_H
#define SEED_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SEED_OK 0
#define SEED_E_INVALID_ARG (-1)
#define SEED_E_SHAPE (-2)
#define SEED_E_CAPACITY (-3)
#define SEED_E_NULL_PTR (-4)
#define SEED_E_UNSUPPORTED_DTYPE (-5)
#define SEED_E_NOT_INIT (-6)
#define SEED_E_HIP (-7)

#define SEED_DTYPE_F32 0
#define SEED_DTYPE_BF16 1
#define SEED_DTYPE_BF16_W8 2 /* as BF16, but the projection matrices are one byte per weight (see seed_layer_w) */
#define SEED_DTYPE_BF16_W4 3 /* as BF16, but the projection matrices are four bits per weight (see seed_layer_w) */

/* seed_accept_args.probs_kind */
#define SEED_KIND_LOGITS 0 /* p_or_logits holds raw logits; the kernel applies softmax(logits / temperature) */
#define SEED_KIND_PROBS 1  /* p_or_logits already holds the target probabilities p                          */

/* seed_step_args.flags / seed_draft_args.flags */
#define SEED_STEP_PREFILL_SHARED 1 /* rows are prefix tokens appended to the shared KV cache (n_branches = 1) */
#define SEED_STEP_GREEDY 2         /* temperature-0 verification: accept iff draft == argmax                  */
#define SEED_STEP_COMMIT_ALL 4     /* no accept step: every fed row becomes private context (private prefill) */

typedef struct seed_ctx seed_ctx; /* opaque; one per model instance */

typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ff, vocab;
    int32_t dtype;      /* SEED_DTYPE_F32, SEED_DTYPE_BF16, SEED_DTYPE_BF16_W8 or SEED_DTYPE_BF16_W4 */
    float rms_eps;      /* RMSNorm epsilon                    */
    float rope_theta;   /* rotary base; rotate-half pairing (i, i + head_dim/2) */
    int32_t max_branches;        /* largest N of any step (bf16: N * T <= 768 rows per step)  */
    int32_t max_rows_per_branch; /* largest T (= gamma, or gamma+1 with a bonus row)        */
    int32_t max_shared;          /* capacity of the shared-prefix KV cache, tokens          */
    int32_t max_private;         /* capacity of each branch's private context, tokens       */
} seed_model_cfg;

typedef struct {
    const void *wq, *wk, *wv, *wo;      /* [H*dh][d], [H*dh][d], [H*dh][d], [d][H*dh] */
    const void *wgate, *wup, *wdown;    /* [F][d], [F][d], [d][F]                     */
    const void *norm_attn, *norm_ffn;   /* [d] RMSNorm gains                          */
    /* The seven matrices by dtype (norm gains, embedding: bf16 in every BF16* dtype):
     *   SEED_DTYPE_BF16_W8: uint8 [rows][cols], OCP e4m3 codes; s* = float32 [rows], the weight is code * s[row];
     *   SEED_DTYPE_BF16_W4: uint8 [rows][cols/2], OCP MXFP4: E2M1 codes, column c in the low (c even) or high
     *     nibble of byte c/2; s* = uint8 [rows][cols/32], E8M0 block scales: the weight is code * 2^(s - 127) with s
     *     the byte of its row and of its block of 32 consecutive columns;
     *   otherwise s* are ignored and may be NULL. */
    const void *sq, *sk, *sv, *so, *sgate, *sup, *sdown;
} seed_layer_w;

typedef struct {
    const void *tok_emb;        /* [V][d]                                    */
    const void *norm_final;     /* [d]                                       */
    const void *lm_head;        /* [V][d] (untied)                           */
    const seed_layer_w *layers; /* HOST array of n_layers entries            */
    const void *lm_head_scale;  /* as the s* of seed_layer_w, for lm_head     */
} seed_weights;

/*
 * Candidate tree of a draft phase (paper Section 2.2 "Tree Attention"; Section 4.1: k_config; appendix
 * "Details of Tree Attention").  k_config = (k_1, ..., k_G): at position j every candidate of position j - 1 has
 * k_j candidate continuations, drawn independently from the draft distribution given the path to them; (2,2,1)
 * is 2 + 4 + 4 = 10 draft tokens.  Nodes are numbered in level order: node 0 is the root (the branch's pending
 * token), then the k_1 nodes of position 1, then the k_1 k_2 nodes of position 2 (children of a node consecutive,
 * in the order of their parents), and so on.  n_nodes = 1 + k_1 + k_1 k_2 + ... <= 64; n_par = the nodes that have
 * children = n_nodes minus the last position's.  All ones is the plain chain.
 */
typedef struct {
    int32_t depth;            /* G, 1..8                                   */
    const int32_t *k_config;  /* HOST array of G entries, each >= 1        */
} seed_tree;

/*
 * Accept / reject / resample (paper Section 3.1; Algorithm 1, inner loop of the verification process).
 *   Row j of branch b holds the target distribution that verifies draft token draft_tok[b][j].
 *   accept iff  fl32(u_acc[b][j] * q[b][j][x]) < p[b][j][x]  (x = draft_tok[b][j]; one float32
 *   multiply, strict comparison), left to right; a_b = number accepted.  At the first rejection one
 *   token is drawn from norm(max(0, p - q)) of that row with u_res[b], using an integer fixed-point
 *   inverse CDF (weights truncated to multiples of 2^-38, so the result does not depend on scan order).
 *   With n_target_rows == gamma + 1 and every draft accepted, a bonus token is drawn from row gamma.
 *   Uniforms must lie on the grid m * 2^-24, 0 <= m < 2^24.
 *   greedy != 0: accept iff x == argmax of the row (lowest index on ties), otherwise emit the argmax;
 *   q, u_acc, u_res and temperature are ignored and may be NULL; p_or_logits must hold logits.
 * Outputs: accept_len[b] = a_b; out_tok[b][0..gamma] = the a_b accepted drafts, then the new token if
 *   any, then -1 padding; n_out[b] = number of valid entries (a_b + 1, or gamma when all gamma drafts
 *   were accepted without a bonus row); p_tok[b][j] = p(draft_tok[b][j]) as used in the test (optional).
 *   private_len (optional, in/out): Algorithm 1's validated-length bookkeeping in cache terms,
 *   private_len[b] += min(a_b + 1, n_target_rows).
 * With a candidate tree (tree != NULL; gamma must equal tree->depth): target row r holds the distribution that
 *   follows the path to node r; n_target_rows = n_par, or n_nodes to also draw a bonus token after a fully
 *   accepted path; q is [N][n_par][V], row r the draft distribution from which node r's children were drawn;
 *   draft_tok, u_acc and p_tok are [N][n_nodes - 1], entry i - 1 belonging to node i (p_tok: the target
 *   probability at the node's parent of the node's token).  The walk starts at the root and tests the children of
 *   the current node in order: the first as above; after i rejections at a node the target becomes the normalised
 *   residual of the previous one minus q (fixed point, 2^-38; totals are integer sums) and candidate x is accepted
 *   iff fl64(fl32(u q(x))) * fl64(Z_i) < fl64(R_i[x]); an accepted child becomes the current node; when all
 *   children are rejected one token is drawn from the last residual with u_res and the walk ends.  The output law
 *   equals the target's.  accept_len = depth reached; out_tok as above; path_node (optional) [N][gamma] = the
 *   accepted node at each depth, then -1.  private_len[b] += number of rows kept: the root and the accepted
 *   nodes that were fed.
 */
typedef struct {
    int32_t n_branches;    /* N >= 0                                             */
    int32_t gamma;         /* draft tokens per branch (the paper's k), >= 1      */
    int32_t n_target_rows; /* gamma or gamma + 1                                 */
    int32_t vocab;         /* V >= 1                                             */
    int32_t probs_kind;    /* SEED_KIND_LOGITS or SEED_KIND_PROBS                */
    int32_t greedy;        /* 0 / 1                                              */
    float temperature;     /* > 0 unless greedy (LOGITS kind only)               */
    const float *p_or_logits; /* [N][n_target_rows][V]                           */
    const float *q;           /* [N][gamma][V]                                   */
    const int32_t *draft_tok; /* [N][gamma], each in [0, V); an id outside is never
                                 used as an index and counts as rejected          */
    const float *u_acc;       /* [N][gamma]                                      */
    const float *u_res;       /* [N]                                             */
    int32_t *accept_len;      /* [N]            out                              */
    int32_t *out_tok;         /* [N][gamma + 1] out                              */
    int32_t *n_out;           /* [N]            out                              */
    float *p_tok;             /* [N][gamma]     out, may be NULL                 */
    int32_t *private_len;     /* [N]            in/out, may be NULL              */
    const seed_tree *tree;    /* HOST, NULL = one candidate per position (chain)  */
    int32_t *path_node;       /* [N][gamma]     out, may be NULL (tree only)      */
} seed_accept_args;

/*
 * One target forward over N x T rows (paper Section 3.1: the context and the draft tokens go through the
 * target model together, which yields the distribution at every draft position in one pass), optionally
 * followed by accept / resample.
 *   row_tok[b][0] is the branch's pending token (validated, KV not yet cached); row_tok[b][j], j >= 1,
 *   is draft token j.  Row j sits at position shared_len + private_len[b] + j and attends to the shared
 *   prefix (read once for all branches), to the branch's private context and causally to rows 0..j of
 *   its own branch.  logits[b][j] is the distribution that verifies draft token j+1.  The K/V of the
 *   fed rows are appended after the branch's private context ("in flight"); committing a row is just
 *   the private_len update done by the accept step.
 *   flags: SEED_STEP_PREFILL_SHARED (n_branches must be 1; rows are appended to the shared cache at
 *   position shared_len; private_len is ignored), SEED_STEP_GREEDY, SEED_STEP_COMMIT_ALL.
 *   accept (optional): its p_or_logits / probs_kind / n_target_rows / n_branches / vocab fields are
 *   filled in by the library from this step's logits; the remaining fields are the caller's.
 *   branch_slot (optional, bf16 contexts): verify a SUBSET of the context's branches (Section 3.3: the
 *   target verifies whichever drafts are waiting in the queue).  Branch b of the call then is the context's
 *   branch branch_slot[b]: its private KV cache is slot branch_slot[b] (0 <= slot < max_branches, all
 *   different within a call) and its length is private_len[branch_slot[b]], i.e. private_len is the
 *   caller's array over ALL max_branches slots; row_tok, logits_out and the accept arrays stay dense over
 *   the call's N branches.  NULL = branch b is slot b.  An out-of-range slot is clamped and sets bit 1 of
 *   the status word.
 *   tree (optional, bf16 contexts): the rows of every branch are the first T nodes of this candidate tree
 *   (T = n_par, or n_nodes with bonus rows) instead of a chain: row j sits at position shared_len +
 *   private_len[b] + depth(j) and attends, among the rows of its branch, to itself and its ancestors only, i.e. it
 *   sees exactly the sequence context + root-to-itself path.  The accept step then walks the tree (accept->tree is
 *   taken from here) and, in every layer, moves the K/V of the rows that are kept (root + accepted path) to the
 *   front of the branch's in-flight region, so that committing stays a length update.
 * Errors: SEED_E_CAPACITY if N, T or shared_len + T exceed what the context was created for.  A branch
 *   whose private_len would overflow max_private + max_rows_per_branch is detected on the device:
 *   its out-of-range rows are dropped and bit 0 of the status word is set (seed_verify_status).
 */
typedef struct {
    int32_t n_branches;       /* N                                                */
    int32_t rows_per_branch;  /* T                                                */
    int32_t flags;
    int32_t shared_len;       /* S: valid tokens in the shared cache (host value) */
    const int32_t *row_tok;   /* [N][T]                                           */
    int32_t *private_len;     /* [N] in (out if accept / COMMIT_ALL)              */
    float *logits_out;        /* [N][T][V] out, may be NULL                       */
    const seed_accept_args *accept; /* host pointer, may be NULL                  */
    const int32_t *branch_slot; /* [N] device, may be NULL: see above              */
    const seed_tree *tree;      /* HOST, may be NULL: see above                    */
} seed_step_args;

/*
 * One autoregressive draft token for each of N branches (paper Section 3.1: drafts are sampled
 * autoregressively from p_d; Algorithm 1, drafting process).  Runs the same forward with one row per
 * branch (the pending token), writes q = softmax(logits / temperature) and draws the next token from
 * q with u[b] by the fixed-point inverse CDF; private_len[b] += 1.  GREEDY: token = argmax, q is
 * still written (with temperature 1).
 *   q_out row b starts at q_out + b * q_stride; tok_out entry b at tok_out + b * tok_stride, so the
 *   call can fill column j of q[N][gamma][V] and draft_tok[N][gamma] directly.
 */
typedef struct {
    int32_t n_branches;
    int32_t flags;
    int32_t shared_len;
    float temperature;
    const int32_t *row_tok; /* [N] pending tokens                 */
    int32_t *private_len;   /* [N] in/out                          */
    const float *u;         /* [N]                                 */
    float *q_out;           /* N rows of V, stride q_stride floats */
    int64_t q_stride;
    int32_t *tok_out;       /* N entries, stride tok_stride        */
    int64_t tok_stride;
    float *logits_out;      /* [N][V] out, may be NULL             */
    const int32_t *branch_slot; /* [N] device, may be NULL: as in seed_step_args (private_len is then indexed
                                   by slot; row_tok, u, q_out, tok_out, logits_out stay dense)  */
} seed_draft_args;

/* Bytes of device workspace a context needs: repacked weights + KV caches + activations. 0 on error. */
size_t seed_verify_workspace_bytes(const seed_model_cfg *cfg);

/*
 * Create a context.  Validates cfg, carves `workspace` (device memory, 256-byte aligned, at least
 * seed_verify_workspace_bytes(cfg)), repacks the weights into it (the caller's weight tensors may be
 * freed once the stream has been synchronised) and zeroes the KV caches.  hip_stream is a hipStream_t
 * (NULL = the default stream) used by every later call on this context.
 */
int seed_verify_init(seed_ctx **out, const seed_model_cfg *cfg, const seed_weights *weights,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

int seed_verify_step(seed_ctx *ctx, const seed_step_args *args);
int seed_draft_step(seed_ctx *ctx, const seed_draft_args *args);

/* Stateless, model-free accept / resample on `hip_stream`; see seed_accept_args. */
int seed_accept_resample(const seed_accept_args *args, void *hip_stream);

/*
 * The same accept / resample for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It runs the two-launch form
 * of the accept step (row statistics spread over the chip, then one workgroup per branch) that a verify step
 * runs out of its context's workspace, with the statistics in an array that is part of the library's device
 * image: this call allocates nothing and frees nothing.  At most 4096 target rows (n_branches *
 * n_target_rows), else SEED_E_CAPACITY; the array is 1 MiB per GPU, held until the process ends.  Arguments,
 * outputs and errors otherwise as seed_accept_resample; the probabilities of the LOGITS kind may differ from
 * that entry point's in the last bits (the statistics are summed slice by slice).  Every call on a GPU uses
 * that GPU's one array: calls that overlap on one GPU (two streams, two threads) race; calls on one stream
 * are ordered.  Nothing in the array has to be cleared between calls.
 */
int seed_accept_resample_static(const seed_accept_args *args, void *hip_stream);

/*
 * Stateless draw x ~ probs rows by the fixed-point inverse CDF (the draft-side sampler of Section 3.1).
 * probs: n_rows rows of V floats, row i at probs + i * row_stride; u: [n_rows]; tok_out: [n_rows].
 */
int seed_sample_probs(const float *probs, int64_t row_stride, const float *u, int32_t *tok_out,
                      int32_t n_rows, int32_t vocab, void *hip_stream);

/*
 * The uniforms u of the accept test, of the residual draw and of the draft sampler (Section 3.1) generated on
 * the device, so that they never cross the host link: out[i] (device, n floats) = (w >> 8) * 2^-24 in [0, 1),
 * where w is word i % 4 of the Philox4x32-10 block (Salmon et al., SC'11) with counter (i / 4, 0, stream, 0) and
 * key (seed, 0x5EED).  A pure function of (seed, stream, i): values are consumed by index, never "next from a
 * stream", and equal the host generator of the test harness bit for bit.  n <= 2^34.
 */
int seed_uniform_philox(uint32_t seed, uint32_t stream, float *out, int64_t n, void *hip_stream);

/*
 * Import externally produced KV for one layer (synthetic-KV protocol): k_shared / v_shared
 * [H][shared_len][dh] (keys already rotated), k_private / v_private [n_branches][H][private_len][dh],
 * all in the context's dtype, device pointers; private pointers may be NULL when private_len == 0.
 */
int seed_kv_load(seed_ctx *ctx, int32_t layer, const void *k_shared, const void *v_shared,
                 int32_t shared_len, const void *k_private, const void *v_private,
                 int32_t n_branches, int32_t private_len);

/* Synchronises the context's stream and returns the device status word in *host_status, then clears it.
 * 0 = clean; bit 0 = a branch overflowed its private capacity (its out-of-range rows were dropped); bit 1 = a
 * branch_slot entry was out of range (clamped); bit 2 = a draft token id of the accept step was outside
 * [0, vocab) (treated as rejected); bit 3 = a row token id was outside [0, vocab) (clamped). */
int seed_verify_status(seed_ctx *ctx, int32_t *host_status);

/*
 * Measurement aid for the weight-streaming projection kernel (the dominant kernel of a step).  While
 * enabled, every projection launch is bracketed by two HIP events on the context's stream.
 * seed_verify_profile_read synchronises the stream and returns, summed over the launches recorded since
 * the last read: their number, their total duration in milliseconds and the weight bytes they streamed
 * (2 bytes per parameter on the bf16 path, 4 on the fp32 path); then forgets them.  Any output pointer may
 * be NULL.  Profiling adds event packets between kernels, so step timings are taken with it disabled.
 */
int seed_verify_profile_enable(seed_ctx *ctx, int32_t enable);
int seed_verify_profile_read(seed_ctx *ctx, int64_t *launches, double *total_ms, double *weight_bytes);

/*
 * What a pair of timing events adds around a launch: brackets n_pairs launches of a one-wavefront kernel that
 * runs for about 20 microseconds by the device's constant-rate wall clock (and records how long it really ran)
 * the same way, synchronises, and returns (time between the events - time the kernel ran) per pair, in
 * milliseconds.  The bracketed time of a projection launch minus this figure is the kernel's own duration as a
 * kernel trace reports it.  The profile must have been read.
 */
int seed_verify_profile_overhead(seed_ctx *ctx, int32_t n_pairs, double *ms_per_pair);

/*
 * Measurement aid: one launch that reads `bytes` (multiple of 16) of device memory at `buf` (16-byte aligned)
 * once, with the access pattern of the weight-streaming projections and nothing else.  Timed by the caller
 * over a buffer much larger than the 256 MB last-level cache, its rate is the practical ceiling of an
 * HBM-bound kernel on this chip.  sink: NULL or 16 writable bytes (never written in practice).
 */
int seed_hbm_read_probe(const void *buf, size_t bytes, void *sink, void *hip_stream);

void seed_verify_destroy(seed_ctx *ctx);

const char *seed_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SEED_VERIFY_H */
