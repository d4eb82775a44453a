// Internal declarations shared by the translation units of libseed_verify (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/seed_verify.h"

namespace seedv {

void set_error(const char *fmt, ...);
}  // namespace seedv
struct seed_ctx;
namespace seedv {
// what the scheduler needs of a context
hipStream_t seed_ctx_stream(const seed_ctx *c);
const seed_model_cfg &seed_ctx_cfg(const seed_ctx *c);
int hip_fail(hipError_t e, const char *what);

// ---- candidate trees ----------------------------------------------------------------------------
constexpr int kMaxTreeDepth = 8;               // positions of a draft phase
constexpr int kMaxTreeNodes = 64;              // nodes of a branch's tree, root included (64-bit ancestor masks)
struct TreeInfo {                              // host-side expansion of a seed_tree
    int G, n_nodes, n_par;                     // positions; nodes (root included); nodes that have children
    int k[kMaxTreeDepth];
    int off[kMaxTreeDepth + 2];                // first node of each level; off[G + 1] = n_nodes
    int parent[kMaxTreeNodes], depth[kMaxTreeNodes];
    unsigned long long anc[kMaxTreeNodes];     // bit j: node j is the node itself or an ancestor
};
int expand_tree(const seed_tree *t, TreeInfo *out);   // validates; SEED_OK or an error code (message set)

// Most rows (branches x rows per branch) of one bf16 step: 48 row tiles, run as row shares of three or four
// tiles that share a weight pass.
constexpr int kMaxStepRows = 768;

// ---- accept.hip ------------------------------------------------------------------------------
size_t accept_scratch_bytes(int max_rows);
constexpr int kStaticAcceptRows = 4096;        // most target rows of a seed_accept_resample_static call
int accept_static_scratch(void **out);         // this GPU's statistics array for that entry point
int launch_accept(const seed_accept_args &a, void *scratch, const int32_t *branch_slot, int n_slots,
                  int32_t *status, hipStream_t st);   // scratch, branch_slot, status may be NULL
// commit_rows (optional, [n_branches][kMaxTreeDepth + 2] ints): per branch the number of rows that stay in the
// cache, then the accepted node at each depth (the root, row 0, is implied)
int launch_accept_tree(const seed_accept_args &a, const TreeInfo &t, void *scratch, const int32_t *branch_slot,
                       int n_slots, int32_t *status, int32_t *commit_rows, hipStream_t st);
int launch_softmax_sample(const float *logits, int64_t logits_stride, float temperature, int greedy,
                          const float *u, float *q_out, int64_t q_stride, int32_t *tok_out,
                          int64_t tok_stride, int32_t *private_len, int n_rows, int vocab, void *scratch,
                          int *counters, const int32_t *branch_slot, int n_slots, hipStream_t st);   // scratch, counters, slot may be NULL
int launch_sample_probs(const float *probs, int64_t row_stride, const float *u, int32_t *tok_out,
                        int n_rows, int vocab, hipStream_t st);

}  // namespace seedv

namespace seedv {
// ---- gemm_bf16.hip -----------------------------------------------------------------------------
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };
struct GemmArgs {
    const void *Wp;        // packed bf16 weights, NT x KT tiles of 1 KiB
    const void *Xp;        // packed hi/lo bf16 activations [m-tile][KT][hi|lo][64][8]
    int NT, KT, kt_per_split, SK, M;
    float *part;           // [SK][M][NT*16] split-K partial sums (SK > 1)
    size_t part_floats;    // capacity of `part` in floats (a split needs SK * M * NT * 16)
    int *counters;         // >= groups + 1 ints, zero on entry and left zero on exit
    float *out;            // STORE: out[row * ld_out + col]
    int ld_out;
    const float *ssq_in;   // STORE (optional) / SWIGLU: [M][NT_in] per-tile sums of squares of the input rows;
    int NT_in;             //   the epilogue scales row r by 1/sqrt(sum / (16 NT_in) + eps)
    float *x;              // RESID: fp32 residual stream [M][NT*16], updated in place
    const void *gain;      // RESID: bf16 gain [NT*16] of the norm that follows
    uint16_t *act_out;     // RESID / SWIGLU: packed hi/lo activation for the next projection
    int KT_out;            //   its k-tile count
    float *ssq;            // RESID: [M][NT] per-tile sums of squares of the new residual stream (out)
    float eps;
    const float *w_scale;  // 8-bit weights: one float per output feature, in packed tile order (NULL: bf16 weights)
    const uint8_t *w_mx;   // 4-bit weights: E8M0 block scales [n-tile][k-tile][16] (NULL otherwise)
    int rot;               // multiplier of the per-column-group rotation of the k walk (0: none)
    int MS;                // row splits: MS workgroups per column group, each with 1 / MS of the row tiles (0 or 1: none)
};
void gemm_bf16_pick(int NT, int KT, int epi, int m_tiles, int *wn, int *wk, int *tn, int *sk, int *wide, int *ms,
                    int w8);
int launch_gemm_bf16_cfg(const GemmArgs &a, int epi, int m_tiles, int wn, int wk, int tn, int wide, hipStream_t st);
int launch_gemm_bf16(GemmArgs a, int epi, int m_tiles, hipStream_t st);   // a.SK < 1: pick automatically
int launch_pack_weight(const void *W, void *dst, int n_rows, int K, int dst_tile0, int dst_tile_step,
                       hipStream_t st);
int launch_pack_weight8(const void *codes, const float *scale, void *dst, float *scale_dst, int n_rows, int K,
                        int dst_tile0, int dst_tile_step, hipStream_t st);
int launch_pack_weight4(const void *codes, const void *mx_scale, void *dst, void *scale_dst, int n_rows, int K,
                        int dst_tile0, int dst_tile_step, hipStream_t st);
// ---- rowops.hip ----------------------------------------------------------------------------------
int launch_rownorm(bool bf16, float *x, const float *part, int SK, int64_t split_stride, const int32_t *tok,
                   const void *emb, int vocab, const void *gain, float eps, void *act, int M, int Mp, int d,
                   int32_t *status, hipStream_t st);   // status may be NULL
int launch_swiglu(bool bf16, const float *part, int SK, int64_t split_stride, void *act, int M, int Mp, int F,
                  hipStream_t st);
int launch_embed_norm(const int32_t *tok, const void *emb, int vocab, const void *gain, float *x, void *act,
                      float *ssq, int M, int d, int32_t *status, hipStream_t st);
int launch_rope_table(float *table, int n_pos, int dh, float theta, hipStream_t st);
int launch_philox_uniform(uint32_t seed, uint32_t stream, float *out, int64_t n, hipStream_t st);
int launch_rope_kv(bool bf16, const float *qkv, const float *rope_table, void *q_out, size_t q_plane,
                   void *k_shared, void *v_shared, void *k_priv, void *v_priv,
                   const int32_t *private_len, int M, int Mq,
                   int T, int H, int dh, int S, int prefill_shared, int cap_shared, int cap_priv,
                   int max_private, int32_t *status, hipStream_t st);
int launch_kv_import(bool bf16, bool transpose, const void *src, void *dst, int heads, int len, int dh, int cap,
                     hipStream_t st);
int launch_hbm_read_probe(const void *buf, size_t bytes, void *sink, hipStream_t st);
int launch_calib_spin(unsigned long long ticks, unsigned long long *elapsed_total, hipStream_t st);
int launch_tree_tables(const TreeInfo &t, int n_rows, int32_t *depth_out, unsigned long long *anc_out, hipStream_t st);
int launch_kv_compact(void *k_priv, void *vt_priv, size_t layer_stride_bytes, int n_layers, const int32_t *commit_rows,
                      const int32_t *private_len, const int32_t *branch_slot, int n_slots, int n_branches, int H, int dh,
                      int cap_p, int max_private, hipStream_t st);
int launch_add_len(int32_t *len, int n, int delta, const int32_t *branch_slot, int n_slots, hipStream_t st);
// ---- attention_bf16.hip ----------------------------------------------------------------------------
void attn_bf16_plan(int M, int H, int N, int total_shared_keys, int cap_priv_keys, int prefill_shared,
                    int *ks_shared, int *keys_per_range, int *ks_priv, int *keys_per_range_priv);
// Verify / decode steps (prefill_shared == 0) run as one launch that reads qkv / rope directly, appends to the
// private cache, sets status bit 0 on a private-length overflow and merges through `counters` (n_heads ints,
// zero on entry, left zero); the shared-prefix prefill reads q (hi/lo planes) written by launch_rope_kv.
struct AttnBf16Args {
    int dh;
    const void *q; size_t q_plane;
    const float *qkv, *rope;
    const void *k_shared, *vt_shared;
    void *k_priv, *vt_priv;
    const int32_t *private_len;
    const int32_t *branch_slot;   // may be NULL; private_len and the private caches are indexed by slot
    int n_slots;                  // max_branches of the context (slots are clamped to it)
    float *o_part, *ml_part;
    int *counters;
    void *act;
    int32_t *status;
    const int32_t *row_depth;                // candidate trees: depth and ancestor mask of the T rows of a branch
    const unsigned long long *row_anc;       //   (both NULL: chain)
    int M, Mp, Mq, N, T, H, S, prefill_shared, cap_s, cap_p, max_private, ks_shared, keys_per_range, ks_priv,
        keys_per_range_priv;
};
int launch_attn_bf16(const AttnBf16Args &a, hipStream_t st);
// ---- fp32_path.hip -----------------------------------------------------------------------------------
int launch_gemm_f32(const void *W, const void *X, float *Y, int M, int Nout, int K, int ldy, hipStream_t st);
int launch_attn_f32(const void *q, const void *k_shared, const void *v_shared, const void *k_priv,
                    const void *v_priv, const int32_t *private_len, float *out, int M, int T, int H, int dh, int S,
                    int prefill_shared, int cap_s, int cap_p, int max_private, hipStream_t st);
}  // namespace seedv
