// C-ABI entry points: argument validation, workspace layout, weight repacking and the per-step
// sequence of kernel launches.  Every entry point validates on the host first and only then touches HIP.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "seed_internal.h"

namespace seedv {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int hip_fail(hipError_t e, const char *what) {
    if (e == hipSuccess) return SEED_OK;
    set_error("%s: %s", what, hipGetErrorString(e));
    return SEED_E_HIP;
}

int expand_tree(const seed_tree *t, TreeInfo *out) {
    if (t == nullptr || out == nullptr) { set_error("tree is NULL"); return SEED_E_NULL_PTR; }
    if (t->depth < 1 || t->depth > kMaxTreeDepth) { set_error("tree: depth must be 1..%d", kMaxTreeDepth); return SEED_E_CAPACITY; }
    if (t->k_config == nullptr) { set_error("tree: k_config is NULL"); return SEED_E_NULL_PTR; }
    TreeInfo ti{};
    ti.G = t->depth;
    ti.off[0] = 0;
    ti.off[1] = 1;
    long level = 1;
    for (int j = 1; j <= ti.G; ++j) {
        const int k = t->k_config[j - 1];
        if (k < 1) { set_error("tree: k_config[%d] = %d must be >= 1", j - 1, k); return SEED_E_INVALID_ARG; }
        level *= k;
        if (ti.off[j] + level > kMaxTreeNodes) { set_error("tree: more than %d nodes", kMaxTreeNodes); return SEED_E_CAPACITY; }
        ti.k[j - 1] = k;
        ti.off[j + 1] = ti.off[j] + (int)level;
    }
    for (int j = ti.G + 2; j < kMaxTreeDepth + 2; ++j) ti.off[j] = ti.off[ti.G + 1];
    ti.n_nodes = ti.off[ti.G + 1];
    ti.n_par = ti.off[ti.G];
    ti.parent[0] = -1;
    ti.depth[0] = 0;
    ti.anc[0] = 1ull;
    for (int j = 1; j <= ti.G; ++j)
        for (int i = ti.off[j]; i < ti.off[j + 1]; ++i) {
            ti.parent[i] = ti.off[j - 1] + (i - ti.off[j]) / ti.k[j - 1];
            ti.depth[i] = j;
            ti.anc[i] = ti.anc[ti.parent[i]] | (1ull << i);
        }
    *out = ti;
    return SEED_OK;
}

namespace {

constexpr int kMaxCounters = 4096;
constexpr int kMaxAttnSlots = 128;
constexpr int kMaxHeads = 1024;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int round_up(int v, int a) { return (v + a - 1) / a * a; }

struct Layout {
    size_t es;                    // bytes per weight / KV element
    int HD, M_cap, Mp_cap, Mq_cap, cap_s, cap_p;
    // weights
    size_t w_qkv, w_o, w_gu, w_d, s_qkv, s_o, s_gu, s_d, g_attn, g_ffn, layer_stride, layers0;
    size_t emb, g_final, lm, s_lm;
    // KV caches (per-layer strides)
    size_t ks, vs, kp, vp, ks_stride, kp_stride;
    // activations
    size_t x, act_d, act_hd, act_f, part, qkv, rinv, ssq, counters, attn_counters, rope, q, o_part, ml_part, logits, acc_stats, draft_counters, status,
        tree_depth, tree_anc, commit_rows;
    int n_pos;
    size_t part_floats;
    size_t total;
};

int validate_cfg(const seed_model_cfg *c) {
    if (c == nullptr) { set_error("cfg is NULL"); return SEED_E_NULL_PTR; }
    if (c->dtype != SEED_DTYPE_F32 && c->dtype != SEED_DTYPE_BF16 && c->dtype != SEED_DTYPE_BF16_W8 && c->dtype != SEED_DTYPE_BF16_W4) {
        set_error("unsupported dtype %d", c->dtype);
        return SEED_E_UNSUPPORTED_DTYPE;
    }
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->head_dim < 2 || c->d_ff < 1 || c->vocab < 1 ||
        c->max_branches < 1 || c->max_rows_per_branch < 1 || c->max_shared < 0 || c->max_private < 0) {
        set_error("model dimensions and capacities must be positive");
        return SEED_E_INVALID_ARG;
    }
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) {
        set_error("rms_eps must be >= 0 and rope_theta > 0");
        return SEED_E_INVALID_ARG;
    }
    const long HD = (long)c->n_heads * c->head_dim;
    if (c->head_dim % 2) { set_error("head_dim must be even"); return SEED_E_SHAPE; }
    if (c->dtype != SEED_DTYPE_F32) {
        if (c->d_model % 32 || c->d_ff % 32 || HD % 32 || c->vocab % 16) {
            set_error("bf16 path needs d_model, d_ff, n_heads*head_dim multiples of 32 and vocab a multiple of 16");
            return SEED_E_SHAPE;
        }
        if (c->head_dim != 64 && c->head_dim != 128) {
            set_error("bf16 path supports head_dim 64 or 128");
            return SEED_E_SHAPE;
        }
        if (c->n_heads > kMaxHeads) {
            set_error("bf16 path supports at most %d heads", kMaxHeads);
            return SEED_E_CAPACITY;
        }
        if ((long)c->max_branches * c->max_rows_per_branch > kMaxStepRows) {
            set_error("bf16 path supports at most %d rows per step (max_branches * max_rows_per_branch)", kMaxStepRows);
            return SEED_E_CAPACITY;
        }
    } else {
        if (c->d_model % 8 || c->d_ff % 8 || HD % 8) {
            set_error("fp32 path needs d_model, d_ff, n_heads*head_dim multiples of 8");
            return SEED_E_SHAPE;
        }
        const long keys = (long)round_up(c->max_shared, 32) + round_up(c->max_private + c->max_rows_per_branch, 32);
        if (keys * 4 > 60 * 1024) {
            set_error("fp32 path supports at most %d cached keys per row", 60 * 1024 / 4);
            return SEED_E_CAPACITY;
        }
        if ((long)c->max_branches * c->max_rows_per_branch > 4096) {
            set_error("fp32 path supports at most 4096 rows per step");
            return SEED_E_CAPACITY;
        }
    }
    return SEED_OK;
}

Layout make_layout(const seed_model_cfg &c) {
    Layout L{};
    const bool bf = c.dtype != SEED_DTYPE_F32;
    const bool w8 = c.dtype == SEED_DTYPE_BF16_W8, w4 = c.dtype == SEED_DTYPE_BF16_W4;
    L.es = bf ? 2 : 4;
    const size_t wbits = w4 ? 4 : w8 ? 8 : 8 * L.es;   // bits per projection weight
    const size_t d = c.d_model, F = c.d_ff, V = c.vocab, H = c.n_heads, dh = c.head_dim;
    L.HD = (int)(H * dh);
    const size_t HD = L.HD;
    L.M_cap = c.max_branches * c.max_rows_per_branch;
    L.Mp_cap = round_up(L.M_cap, 16);
    L.Mq_cap = round_up(L.M_cap, 32);
    L.cap_s = round_up(c.max_shared > 0 ? c.max_shared : 1, 32);
    L.cap_p = round_up(c.max_private + c.max_rows_per_branch, 32);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    // one layer's weights
    size_t lo = 0;
    auto ltake = [&](size_t bytes) { size_t o = lo; lo = align_up(lo + bytes, 256); return o; };
    L.w_qkv = ltake(3 * HD * d * wbits / 8);
    L.w_o = ltake(d * HD * wbits / 8);
    L.w_gu = ltake(2 * F * d * wbits / 8);
    L.w_d = ltake(d * F * wbits / 8);
    // (one-byte weights: per-output-row scales, in the order of the packed tiles; four-bit weights: one scale
    // byte per output row and 32 inputs)
    L.s_qkv = ltake(w8 ? 3 * HD * 4 : w4 ? 3 * HD * d / 32 : 0);
    L.s_o = ltake(w8 ? d * 4 : w4 ? d * HD / 32 : 0);
    L.s_gu = ltake(w8 ? 2 * F * 4 : w4 ? 2 * F * d / 32 : 0);
    L.s_d = ltake(w8 ? d * 4 : w4 ? d * F / 32 : 0);
    L.g_attn = ltake(d * L.es);
    L.g_ffn = ltake(d * L.es);
    L.layer_stride = lo;
    L.layers0 = take(L.layer_stride * c.n_layers);
    L.emb = take(V * d * L.es);
    L.g_final = take(d * L.es);
    L.lm = take(V * d * wbits / 8);
    L.s_lm = take(w8 ? V * 4 : w4 ? V * d / 32 : 256);
    L.ks_stride = align_up(H * L.cap_s * dh * L.es, 256);
    L.kp_stride = align_up((size_t)c.max_branches * H * L.cap_p * dh * L.es, 256);
    L.ks = take(L.ks_stride * c.n_layers);
    L.vs = take(L.ks_stride * c.n_layers);
    L.kp = take(L.kp_stride * c.n_layers);
    L.vp = take(L.kp_stride * c.n_layers);
    size_t widest = 3 * HD;
    if (2 * F > widest) widest = 2 * F;
    if (d > widest) widest = d;
    L.x = take((size_t)L.Mp_cap * d * 4);
    L.act_d = take((size_t)L.Mp_cap * d * 4);             // bf16 path: hi + lo halves; fp32 path: plain floats
    L.act_hd = take((size_t)L.Mp_cap * HD * 4);
    L.act_f = take((size_t)L.Mp_cap * F * 4);
    // split-K partials: SK * Nout stays near 384 workgroups * 128 columns; V covers an unsplit LM head
    L.part_floats = (size_t)L.M_cap * (bf ? (widest > 65536 ? widest : 65536) : widest);
    L.part = take(L.part_floats * 4);
    L.qkv = take((size_t)L.M_cap * 3 * HD * 4);
    L.rinv = take((size_t)L.Mp_cap * 4);
    L.ssq = take((size_t)L.M_cap * (d / 16 + 1) * 4);
    L.counters = take(4096 * 4);
    L.attn_counters = take(kMaxHeads * 4);
    L.n_pos = c.max_shared + c.max_private + c.max_rows_per_branch + 1;
    L.rope = take((size_t)L.n_pos * dh * 4);
    L.q = take((size_t)L.Mq_cap * HD * 4);   // bf16 path: hi and lo planes
    L.o_part = take(bf ? (size_t)kMaxAttnSlots * L.Mq_cap * HD * 4 : 256);
    L.ml_part = take(bf ? (size_t)kMaxAttnSlots * L.Mq_cap * H * 2 * 4 : 256);
    L.logits = take((size_t)L.M_cap * V * 4);
    L.acc_stats = take(accept_scratch_bytes(L.M_cap));
    L.draft_counters = take((size_t)L.M_cap * 4);
    L.status = take(256);
    L.tree_depth = take(kMaxTreeNodes * 4);
    L.tree_anc = take(kMaxTreeNodes * 8);
    L.commit_rows = take((size_t)c.max_branches * (kMaxTreeDepth + 2) * 4);
    L.total = off;
    return L;
}

}  // namespace
}  // namespace seedv

using namespace seedv;

struct seed_ctx {
    seed_model_cfg cfg;
    Layout L;
    char *ws;
    hipStream_t stream;
    bool bf16;
    bool w8;                             // projection matrices as e4m3 codes + per-row scales
    bool w4;                             // ... as MXFP4 codes + per-block scales
    // projection-kernel profiling (seed_verify_profile_*)
    bool profiling = false;
    std::vector<hipEvent_t> ev_pool;     // start/stop pairs, reused
    size_t ev_used = 0;
    double prof_bytes = 0.0;
};

namespace seedv {
hipStream_t seed_ctx_stream(const seed_ctx *c) { return c->stream; }
const seed_model_cfg &seed_ctx_cfg(const seed_ctx *c) { return c->cfg; }
}  // namespace seedv

namespace {

inline void *at(const seed_ctx *c, size_t off) { return c->ws + off; }
inline void *layer_w(const seed_ctx *c, int l, size_t off) { return c->ws + c->L.layers0 + c->L.layer_stride * l + off; }

int check_accept_args(const seed_accept_args *a) {
    if (a == nullptr) { set_error("accept args is NULL"); return SEED_E_NULL_PTR; }
    if (a->n_branches < 0 || a->gamma < 1 || a->vocab < 1) {
        set_error("accept: need n_branches >= 0, gamma >= 1, vocab >= 1");
        return SEED_E_INVALID_ARG;
    }
    if (a->tree != nullptr) {
        TreeInfo ti;
        const int rc = expand_tree(a->tree, &ti);
        if (rc) return rc;
        if (a->gamma != ti.G) { set_error("accept: gamma %d must equal the tree's depth %d", a->gamma, ti.G); return SEED_E_SHAPE; }
        if (a->n_target_rows != ti.n_par && a->n_target_rows != ti.n_nodes) {
            set_error("accept: n_target_rows must be %d (nodes with children) or %d (all nodes)", ti.n_par, ti.n_nodes);
            return SEED_E_SHAPE;
        }
    } else if (a->n_target_rows != a->gamma && a->n_target_rows != a->gamma + 1) {
        set_error("accept: n_target_rows must be gamma or gamma + 1");
        return SEED_E_SHAPE;
    }
    if (a->gamma > 1023) { set_error("accept: gamma must be < 1024"); return SEED_E_CAPACITY; }
    if (a->probs_kind != SEED_KIND_LOGITS && a->probs_kind != SEED_KIND_PROBS) {
        set_error("accept: probs_kind must be SEED_KIND_LOGITS or SEED_KIND_PROBS");
        return SEED_E_INVALID_ARG;
    }
    if (a->n_branches == 0) return SEED_OK;
    if (!a->p_or_logits || !a->draft_tok || !a->accept_len || !a->out_tok || !a->n_out) {
        set_error("accept: p_or_logits, draft_tok, accept_len, out_tok, n_out must be non-NULL");
        return SEED_E_NULL_PTR;
    }
    if (a->greedy) {
        if (a->probs_kind != SEED_KIND_LOGITS) {
            set_error("accept: greedy mode needs logits");
            return SEED_E_INVALID_ARG;
        }
    } else {
        if (!a->q || !a->u_acc || !a->u_res) {
            set_error("accept: q, u_acc, u_res must be non-NULL unless greedy");
            return SEED_E_NULL_PTR;
        }
        if (a->probs_kind == SEED_KIND_LOGITS && !(a->temperature > 0.f)) {
            set_error("accept: temperature must be > 0");
            return SEED_E_INVALID_ARG;
        }
    }
    return SEED_OK;
}

// Wraps one projection launch with the optional profiling events.
template <class F>
int profiled(seed_ctx *c, double weight_bytes, F &&launch) {
    if (!c->profiling) return launch();
    if (c->ev_used + 2 > c->ev_pool.size()) {
        for (int i = 0; i < 2; ++i) {
            hipEvent_t e;
            int rc = hip_fail(hipEventCreate(&e), "event create");
            if (rc) return rc;
            c->ev_pool.push_back(e);
        }
    }
    hipEvent_t e0 = c->ev_pool[c->ev_used], e1 = c->ev_pool[c->ev_used + 1];
    int rc = hip_fail(hipEventRecord(e0, c->stream), "event record");
    if (rc) return rc;
    rc = launch();
    if (rc) return rc;
    rc = hip_fail(hipEventRecord(e1, c->stream), "event record");
    if (rc) return rc;
    c->ev_used += 2;
    c->prof_bytes += weight_bytes;
    return SEED_OK;
}

struct KvPtrs { void *ks, *vs, *kp, *vp; };
KvPtrs kv_layer(const seed_ctx *c, int l) {
    const Layout &L = c->L;
    return {c->ws + L.ks + L.ks_stride * l, c->ws + L.vs + L.ks_stride * l, c->ws + L.kp + L.kp_stride * l,
            c->ws + L.vp + L.kp_stride * l};
}

// bf16 path: projections with fused epilogues (see gemm_bf16.hip); 5 launches per layer in a verify / decode
// step (6 above 16 rows), 7 in the shared-prefix prefill.
int run_forward_bf16(seed_ctx *c, int N, int T, int S, int prefill_shared, const int32_t *row_tok,
                     const int32_t *private_len, const int32_t *branch_slot, const TreeInfo *tree, float *logits) {
    const seed_model_cfg &g = c->cfg;
    const Layout &L = c->L;
    hipStream_t st = c->stream;
    const int M = N * T, Mp = round_up(M, 16), Mq = round_up(M, 32);
    const int d = g.d_model, F = g.d_ff, H = g.n_heads, dh = g.head_dim, HD = L.HD, V = g.vocab;
    const int m_tiles = Mp / 16;
    float *x = (float *)at(c, L.x);
    float *ssq = (float *)at(c, L.ssq);
    int32_t *status = (int32_t *)at(c, L.status);
    const size_t q_plane = (size_t)L.Mq_cap * HD;
    int rc;

    auto gemm = [&](int epi, const void *W, const void *scale, int Nout, int K, const void *Xp, GemmArgs a) -> int {
        a.Wp = W;
        a.w_scale = c->w8 ? (const float *)scale : nullptr;
        a.w_mx = c->w4 ? (const uint8_t *)scale : nullptr;
        a.Xp = Xp;
        a.NT = Nout / 16;
        a.KT = K / 32;
        a.M = M;
        a.part = (float *)at(c, L.part);
        a.part_floats = L.part_floats;
        a.counters = (int *)at(c, L.counters);
        a.eps = g.rms_eps;
        int wn, wk, tn, sk, wide, ms;
        gemm_bf16_pick(a.NT, a.KT, epi, m_tiles, &wn, &wk, &tn, &sk, &wide, &ms, c->w8 || c->w4);
        while (sk > 1 && (size_t)sk * M * Nout > L.part_floats) --sk;
        a.SK = sk;
        if (sk > 1 && (a.NT / (wn * tn) + 8) * ms + 2 > kMaxCounters) {
            set_error("projection with %d column groups exceeds the counter array", a.NT / (wn * tn));
            return SEED_E_CAPACITY;
        }
        return profiled(c, (double)Nout * K * (c->w4 ? 0.53125 : c->w8 ? 1.0 : 2.0), [&]() { return launch_gemm_bf16(a, epi, m_tiles, st); });
    };

    int ks_shared = 1, keys_per_range = 32, ks_priv = 0, keys_per_range_priv = 128;
    attn_bf16_plan(M, H, N, prefill_shared ? S + M : S, g.max_private, prefill_shared, &ks_shared, &keys_per_range,
                   &ks_priv, &keys_per_range_priv);
    if (ks_shared + ks_priv + 1 > kMaxAttnSlots) {
        set_error("attention plan needs %d partial slots (max %d)", ks_shared + ks_priv + 1, kMaxAttnSlots);
        return SEED_E_CAPACITY;
    }

    const int32_t *row_depth = nullptr;
    const unsigned long long *row_anc = nullptr;
    if (tree != nullptr) {
        // the per-row tables of the candidate tree: position offsets and who sees whom among a branch's rows
        rc = launch_tree_tables(*tree, T, (int32_t *)at(c, L.tree_depth), (unsigned long long *)at(c, L.tree_anc), st);
        if (rc) return rc;
        row_depth = (const int32_t *)at(c, L.tree_depth);
        row_anc = (const unsigned long long *)at(c, L.tree_anc);
    }
    rc = launch_embed_norm(row_tok, at(c, L.emb), V, layer_w(c, 0, L.g_attn), x, at(c, L.act_d), ssq, M, d, status, st);
    if (rc) return rc;
    for (int l = 0; l < g.n_layers; ++l) {
        GemmArgs a{};
        a.out = (float *)at(c, L.qkv);
        a.ld_out = 3 * HD;
        a.ssq_in = ssq;
        a.NT_in = d / 16;
        rc = gemm(EPI_STORE, layer_w(c, l, L.w_qkv), layer_w(c, l, L.s_qkv), 3 * HD, d, at(c, L.act_d), a);
        if (rc) return rc;
        const KvPtrs kv = kv_layer(c, l);
        if (prefill_shared) {
            rc = launch_rope_kv(true, (const float *)at(c, L.qkv), (const float *)at(c, L.rope), at(c, L.q), q_plane,
                                kv.ks, kv.vs, kv.kp, kv.vp, private_len, M, Mq, T, H, dh, S, prefill_shared, L.cap_s,
                                L.cap_p, g.max_private, status, st);
            if (rc) return rc;
        }
        AttnBf16Args at_{};
        at_.dh = dh;
        at_.q = at(c, L.q); at_.q_plane = q_plane;
        at_.qkv = (const float *)at(c, L.qkv); at_.rope = (const float *)at(c, L.rope);
        at_.k_shared = kv.ks; at_.vt_shared = kv.vs; at_.k_priv = kv.kp; at_.vt_priv = kv.vp;
        at_.private_len = private_len;
        at_.branch_slot = branch_slot;
        at_.n_slots = g.max_branches;
        at_.o_part = (float *)at(c, L.o_part); at_.ml_part = (float *)at(c, L.ml_part);
        at_.counters = (int *)at(c, L.attn_counters);
        at_.act = at(c, L.act_hd);
        at_.status = status;
        at_.row_depth = row_depth;
        at_.row_anc = row_anc;
        at_.M = M; at_.Mp = Mp; at_.Mq = Mq; at_.N = N; at_.T = T; at_.H = H; at_.S = S;
        at_.prefill_shared = prefill_shared;
        at_.cap_s = L.cap_s; at_.cap_p = L.cap_p; at_.max_private = g.max_private;
        at_.ks_shared = ks_shared; at_.keys_per_range = keys_per_range; at_.ks_priv = ks_priv;
        at_.keys_per_range_priv = keys_per_range_priv;
        rc = launch_attn_bf16(at_, st);
        if (rc) return rc;
        GemmArgs o{};
        o.x = x;
        o.gain = layer_w(c, l, L.g_ffn);
        o.act_out = (uint16_t *)at(c, L.act_d);
        o.KT_out = d / 32;
        o.ssq = ssq;
        rc = gemm(EPI_RESID, layer_w(c, l, L.w_o), layer_w(c, l, L.s_o), d, HD, at(c, L.act_hd), o);
        if (rc) return rc;
        GemmArgs gu{};
        gu.ssq_in = ssq;
        gu.NT_in = d / 16;
        gu.act_out = (uint16_t *)at(c, L.act_f);
        gu.KT_out = F / 32;
        rc = gemm(EPI_SWIGLU, layer_w(c, l, L.w_gu), layer_w(c, l, L.s_gu), 2 * F, d, at(c, L.act_d), gu);
        if (rc) return rc;
        GemmArgs dn = o;
        dn.gain = (l + 1 < g.n_layers) ? layer_w(c, l + 1, L.g_attn) : at(c, L.g_final);
        rc = gemm(EPI_RESID, layer_w(c, l, L.w_d), layer_w(c, l, L.s_d), d, F, at(c, L.act_f), dn);
        if (rc) return rc;
    }
    if (logits != nullptr) {
        GemmArgs a{};
        a.out = logits;
        a.ld_out = V;
        a.ssq_in = ssq;
        a.NT_in = d / 16;
        rc = gemm(EPI_STORE, at(c, L.lm), at(c, L.s_lm), V, d, at(c, L.act_d), a);
        if (rc) return rc;
    }
    return SEED_OK;
}

// fp32 path: plain kernels, one stage per launch.
int run_forward_f32(seed_ctx *c, int N, int T, int S, int prefill_shared, const int32_t *row_tok,
                    const int32_t *private_len, float *logits) {
    const seed_model_cfg &g = c->cfg;
    const Layout &L = c->L;
    hipStream_t st = c->stream;
    const int M = N * T;
    const int d = g.d_model, F = g.d_ff, H = g.n_heads, dh = g.head_dim, HD = L.HD, V = g.vocab;
    float *x = (float *)at(c, L.x);
    float *part = (float *)at(c, L.part);
    void *act_d = at(c, L.act_d), *act_hd = at(c, L.act_hd), *act_f = at(c, L.act_f);
    int32_t *status = (int32_t *)at(c, L.status);
    int rc;
    auto gemm = [&](const void *W, int Nout, int K, const void *X, float *out, int ld) -> int {
        return profiled(c, (double)Nout * K * 4.0, [&]() { return launch_gemm_f32(W, X, out, M, Nout, K, ld, st); });
    };
    rc = launch_rownorm(false, x, nullptr, 0, 0, row_tok, at(c, L.emb), V, layer_w(c, 0, L.g_attn), g.rms_eps, act_d, M,
                        M, d, status, st);
    if (rc) return rc;
    for (int l = 0; l < g.n_layers; ++l) {
        rc = gemm(layer_w(c, l, L.w_qkv), 3 * HD, d, act_d, part, 3 * HD);
        if (rc) return rc;
        const KvPtrs kv = kv_layer(c, l);
        rc = launch_rope_kv(false, part, (const float *)at(c, L.rope), at(c, L.q), 0, kv.ks, kv.vs, kv.kp, kv.vp,
                            private_len, M, M, T, H, dh, S, prefill_shared, L.cap_s, L.cap_p, g.max_private,
                            status, st);
        if (rc) return rc;
        rc = launch_attn_f32(at(c, L.q), kv.ks, kv.vs, kv.kp, kv.vp, private_len, (float *)act_hd, M, T, H, dh, S,
                             prefill_shared, L.cap_s, L.cap_p, g.max_private, st);
        if (rc) return rc;
        rc = gemm(layer_w(c, l, L.w_o), d, HD, act_hd, part, d);
        if (rc) return rc;
        rc = launch_rownorm(false, x, part, 1, 0, nullptr, nullptr, V, layer_w(c, l, L.g_ffn), g.rms_eps, act_d, M, M, d,
                            nullptr, st);
        if (rc) return rc;
        rc = gemm(layer_w(c, l, L.w_gu), 2 * F, d, act_d, part, 2 * F);
        if (rc) return rc;
        rc = launch_swiglu(false, part, 1, 0, act_f, M, M, F, st);
        if (rc) return rc;
        rc = gemm(layer_w(c, l, L.w_d), d, F, act_f, part, d);
        if (rc) return rc;
        const void *next_gain = (l + 1 < g.n_layers) ? layer_w(c, l + 1, L.g_attn) : at(c, L.g_final);
        rc = launch_rownorm(false, x, part, 1, 0, nullptr, nullptr, V, next_gain, g.rms_eps, act_d, M, M, d, nullptr, st);
        if (rc) return rc;
    }
    if (logits != nullptr) return gemm(at(c, L.lm), V, d, act_d, logits, V);
    return SEED_OK;
}

int run_forward(seed_ctx *c, int N, int T, int S, int prefill_shared, const int32_t *row_tok,
                const int32_t *private_len, const int32_t *branch_slot, const TreeInfo *tree, float *logits) {
    if ((branch_slot != nullptr || tree != nullptr) && (!c->bf16 || prefill_shared)) {
        set_error("branch_slot and candidate trees need a bf16 context and a verify / decode step");
        return SEED_E_UNSUPPORTED_DTYPE;
    }
    return c->bf16 ? run_forward_bf16(c, N, T, S, prefill_shared, row_tok, private_len, branch_slot, tree, logits)
                   : run_forward_f32(c, N, T, S, prefill_shared, row_tok, private_len, logits);
}

}  // namespace

extern "C" {

const char *seed_last_error(void) { return g_err; }

size_t seed_verify_workspace_bytes(const seed_model_cfg *cfg) {
    if (validate_cfg(cfg) != SEED_OK) return 0;
    return make_layout(*cfg).total;
}

int seed_verify_init(seed_ctx **out, const seed_model_cfg *cfg, const seed_weights *w, void *workspace,
                     size_t workspace_bytes, void *hip_stream) {
    if (out == nullptr) { set_error("out is NULL"); return SEED_E_NULL_PTR; }
    *out = nullptr;
    int rc = validate_cfg(cfg);
    if (rc) return rc;
    if (w == nullptr || workspace == nullptr) { set_error("weights / workspace is NULL"); return SEED_E_NULL_PTR; }
    if (!w->tok_emb || !w->norm_final || !w->lm_head || !w->layers) {
        set_error("weights: tok_emb, norm_final, lm_head, layers must be non-NULL");
        return SEED_E_NULL_PTR;
    }
    for (int l = 0; l < cfg->n_layers; ++l) {
        const seed_layer_w &lw = w->layers[l];
        if (!lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.wgate || !lw.wup || !lw.wdown || !lw.norm_attn ||
            !lw.norm_ffn) {
            set_error("weights: layer %d has a NULL tensor", l);
            return SEED_E_NULL_PTR;
        }
    }
    if (cfg->dtype == SEED_DTYPE_BF16_W8 || cfg->dtype == SEED_DTYPE_BF16_W4) {
        if (!w->lm_head_scale) { set_error("weights: lm_head_scale is NULL"); return SEED_E_NULL_PTR; }
        for (int l = 0; l < cfg->n_layers; ++l) {
            const seed_layer_w &lw = w->layers[l];
            if (!lw.sq || !lw.sk || !lw.sv || !lw.so || !lw.sgate || !lw.sup || !lw.sdown) {
                set_error("weights: layer %d has a NULL scale array", l);
                return SEED_E_NULL_PTR;
            }
        }
    }
    if (((uintptr_t)workspace & 255) != 0) { set_error("workspace must be 256-byte aligned"); return SEED_E_INVALID_ARG; }
    Layout L = make_layout(*cfg);
    if (workspace_bytes < L.total) {
        set_error("workspace too small: %zu < %zu", workspace_bytes, L.total);
        return SEED_E_CAPACITY;
    }
    seed_ctx *c = new (std::nothrow) seed_ctx;
    if (c == nullptr) { set_error("out of host memory"); return SEED_E_INVALID_ARG; }
    c->cfg = *cfg;
    c->L = L;
    c->ws = (char *)workspace;
    c->stream = (hipStream_t)hip_stream;
    c->bf16 = cfg->dtype != SEED_DTYPE_F32;
    c->w8 = cfg->dtype == SEED_DTYPE_BF16_W8;
    c->w4 = cfg->dtype == SEED_DTYPE_BF16_W4;
    hipStream_t st = c->stream;
    const size_t es = L.es, d = cfg->d_model, F = cfg->d_ff, V = cfg->vocab, HD = L.HD;
    auto copy = [&](void *dst, const void *src, size_t bytes) {
        return hip_fail(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st), "weight copy");
    };
#define SEEDV_TRY(expr) do { rc = (expr); if (rc) { delete c; return rc; } } while (0)
    for (int l = 0; l < cfg->n_layers; ++l) {
        const seed_layer_w &lw = w->layers[l];
        if (c->w8) {
            const int qt = (int)(HD / 16);
            float *sqkv = (float *)layer_w(c, l, L.s_qkv), *sgu = (float *)layer_w(c, l, L.s_gu);
            SEEDV_TRY(launch_pack_weight8(lw.wq, (const float *)lw.sq, layer_w(c, l, L.w_qkv), sqkv, (int)HD, (int)d, 0, 1, st));
            SEEDV_TRY(launch_pack_weight8(lw.wk, (const float *)lw.sk, layer_w(c, l, L.w_qkv), sqkv, (int)HD, (int)d, qt, 1, st));
            SEEDV_TRY(launch_pack_weight8(lw.wv, (const float *)lw.sv, layer_w(c, l, L.w_qkv), sqkv, (int)HD, (int)d, 2 * qt, 1, st));
            SEEDV_TRY(launch_pack_weight8(lw.wo, (const float *)lw.so, layer_w(c, l, L.w_o), (float *)layer_w(c, l, L.s_o), (int)d, (int)HD, 0, 1, st));
            SEEDV_TRY(launch_pack_weight8(lw.wgate, (const float *)lw.sgate, layer_w(c, l, L.w_gu), sgu, (int)F, (int)d, 0, 2, st));
            SEEDV_TRY(launch_pack_weight8(lw.wup, (const float *)lw.sup, layer_w(c, l, L.w_gu), sgu, (int)F, (int)d, 1, 2, st));
            SEEDV_TRY(launch_pack_weight8(lw.wdown, (const float *)lw.sdown, layer_w(c, l, L.w_d), (float *)layer_w(c, l, L.s_d), (int)d, (int)F, 0, 1, st));
        } else if (c->w4) {
            const int qt = (int)(HD / 16);
            void *sqkv = layer_w(c, l, L.s_qkv), *sgu = layer_w(c, l, L.s_gu);
            SEEDV_TRY(launch_pack_weight4(lw.wq, lw.sq, layer_w(c, l, L.w_qkv), sqkv, (int)HD, (int)d, 0, 1, st));
            SEEDV_TRY(launch_pack_weight4(lw.wk, lw.sk, layer_w(c, l, L.w_qkv), sqkv, (int)HD, (int)d, qt, 1, st));
            SEEDV_TRY(launch_pack_weight4(lw.wv, lw.sv, layer_w(c, l, L.w_qkv), sqkv, (int)HD, (int)d, 2 * qt, 1, st));
            SEEDV_TRY(launch_pack_weight4(lw.wo, lw.so, layer_w(c, l, L.w_o), layer_w(c, l, L.s_o), (int)d, (int)HD, 0, 1, st));
            SEEDV_TRY(launch_pack_weight4(lw.wgate, lw.sgate, layer_w(c, l, L.w_gu), sgu, (int)F, (int)d, 0, 2, st));
            SEEDV_TRY(launch_pack_weight4(lw.wup, lw.sup, layer_w(c, l, L.w_gu), sgu, (int)F, (int)d, 1, 2, st));
            SEEDV_TRY(launch_pack_weight4(lw.wdown, lw.sdown, layer_w(c, l, L.w_d), layer_w(c, l, L.s_d), (int)d, (int)F, 0, 1, st));
        } else if (c->bf16) {
            const int qt = (int)(HD / 16);
            SEEDV_TRY(launch_pack_weight(lw.wq, layer_w(c, l, L.w_qkv), (int)HD, (int)d, 0, 1, st));
            SEEDV_TRY(launch_pack_weight(lw.wk, layer_w(c, l, L.w_qkv), (int)HD, (int)d, qt, 1, st));
            SEEDV_TRY(launch_pack_weight(lw.wv, layer_w(c, l, L.w_qkv), (int)HD, (int)d, 2 * qt, 1, st));
            SEEDV_TRY(launch_pack_weight(lw.wo, layer_w(c, l, L.w_o), (int)d, (int)HD, 0, 1, st));
            SEEDV_TRY(launch_pack_weight(lw.wgate, layer_w(c, l, L.w_gu), (int)F, (int)d, 0, 2, st));
            SEEDV_TRY(launch_pack_weight(lw.wup, layer_w(c, l, L.w_gu), (int)F, (int)d, 1, 2, st));
            SEEDV_TRY(launch_pack_weight(lw.wdown, layer_w(c, l, L.w_d), (int)d, (int)F, 0, 1, st));
        } else {
            char *qkv = (char *)layer_w(c, l, L.w_qkv);
            SEEDV_TRY(copy(qkv, lw.wq, HD * d * es));
            SEEDV_TRY(copy(qkv + HD * d * es, lw.wk, HD * d * es));
            SEEDV_TRY(copy(qkv + 2 * HD * d * es, lw.wv, HD * d * es));
            SEEDV_TRY(copy(layer_w(c, l, L.w_o), lw.wo, d * HD * es));
            char *gu = (char *)layer_w(c, l, L.w_gu);
            SEEDV_TRY(copy(gu, lw.wgate, F * d * es));
            SEEDV_TRY(copy(gu + F * d * es, lw.wup, F * d * es));
            SEEDV_TRY(copy(layer_w(c, l, L.w_d), lw.wdown, d * F * es));
        }
        SEEDV_TRY(copy(layer_w(c, l, L.g_attn), lw.norm_attn, d * es));
        SEEDV_TRY(copy(layer_w(c, l, L.g_ffn), lw.norm_ffn, d * es));
    }
    SEEDV_TRY(copy(at(c, L.emb), w->tok_emb, V * d * es));
    SEEDV_TRY(copy(at(c, L.g_final), w->norm_final, d * es));
    if (c->w8) SEEDV_TRY(launch_pack_weight8(w->lm_head, (const float *)w->lm_head_scale, at(c, L.lm), (float *)at(c, L.s_lm), (int)V, (int)d, 0, 1, st));
    else if (c->w4) SEEDV_TRY(launch_pack_weight4(w->lm_head, w->lm_head_scale, at(c, L.lm), at(c, L.s_lm), (int)V, (int)d, 0, 1, st));
    else if (c->bf16) SEEDV_TRY(launch_pack_weight(w->lm_head, at(c, L.lm), (int)V, (int)d, 0, 1, st));
    else SEEDV_TRY(copy(at(c, L.lm), w->lm_head, V * d * es));
    // KV caches and scratch start at zero: chunked key loops may touch (masked) entries past the valid length
    SEEDV_TRY(hip_fail(hipMemsetAsync(at(c, L.ks), 0, L.total - L.ks, st), "workspace clear"));
    SEEDV_TRY(launch_rope_table((float *)at(c, L.rope), L.n_pos, cfg->head_dim, cfg->rope_theta, st));
#undef SEEDV_TRY
    *out = c;
    return SEED_OK;
}

void seed_verify_destroy(seed_ctx *ctx) {
    if (ctx == nullptr) return;
    for (hipEvent_t e : ctx->ev_pool) (void)hipEventDestroy(e);
    delete ctx;
}

int seed_verify_profile_enable(seed_ctx *c, int32_t enable) {
    if (c == nullptr) { set_error("context is NULL"); return SEED_E_NOT_INIT; }
    c->profiling = enable != 0;
    return SEED_OK;
}

int seed_verify_profile_read(seed_ctx *c, int64_t *launches, double *total_ms, double *weight_bytes) {
    if (c == nullptr) { set_error("context is NULL"); return SEED_E_NOT_INIT; }
    int rc = hip_fail(hipStreamSynchronize(c->stream), "stream sync");
    if (rc) return rc;
    double ms = 0.0;
    for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
        float t = 0.f;
        rc = hip_fail(hipEventElapsedTime(&t, c->ev_pool[i], c->ev_pool[i + 1]), "event elapsed");
        if (rc) return rc;
        ms += t;
    }
    if (launches) *launches = (int64_t)(c->ev_used / 2);
    if (total_ms) *total_ms = ms;
    if (weight_bytes) *weight_bytes = c->prof_bytes;
    c->ev_used = 0;
    c->prof_bytes = 0.0;
    return SEED_OK;
}

int seed_verify_profile_overhead(seed_ctx *c, int32_t n_pairs, double *ms_per_pair) {
    if (c == nullptr) { set_error("context is NULL"); return SEED_E_NOT_INIT; }
    if (n_pairs < 1 || n_pairs > 100000 || ms_per_pair == nullptr) { set_error("profile_overhead: need 1 <= n_pairs <= 100000 and an output pointer"); return SEED_E_INVALID_ARG; }
    if (c->ev_used != 0) { set_error("profile_overhead: read the recorded launches first"); return SEED_E_INVALID_ARG; }
    int dev = 0, khz = 0;
    int rc = hip_fail(hipGetDevice(&dev), "hipGetDevice");
    if (rc) return rc;
    rc = hip_fail(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev), "wall clock rate");
    if (rc) return rc;
    if (khz <= 0) { set_error("profile_overhead: the device reports no wall clock rate"); return SEED_E_HIP; }
    // the counter lives in the status block, past the status word
    unsigned long long *total = reinterpret_cast<unsigned long long *>((char *)at(c, c->L.status) + 64);
    rc = hip_fail(hipMemsetAsync(total, 0, 8, c->stream), "calibration clear");
    if (rc) return rc;
    const unsigned long long ticks = (unsigned long long)khz * 20 / 1000;        // 20 microseconds
    const bool was = c->profiling;
    c->profiling = true;
    for (int i = 0; i < n_pairs && rc == SEED_OK; ++i)
        rc = profiled(c, 0.0, [&]() { return launch_calib_spin(ticks, total, c->stream); });
    c->profiling = was;
    if (rc) return rc;
    int64_t n = 0;
    double ms = 0.0;
    rc = seed_verify_profile_read(c, &n, &ms, nullptr);      // synchronises the stream
    if (rc) return rc;
    unsigned long long spent = 0;
    rc = hip_fail(hipMemcpy(&spent, total, 8, hipMemcpyDeviceToHost), "calibration read");
    if (rc) return rc;
    *ms_per_pair = (ms - (double)spent / (double)khz) / (double)n;
    return SEED_OK;
}

int seed_hbm_read_probe(const void *buf, size_t bytes, void *sink, void *hip_stream) {
    if (buf == nullptr) { set_error("read probe: buffer is NULL"); return SEED_E_NULL_PTR; }
    if (bytes < 16 || ((uintptr_t)buf & 15) != 0) { set_error("read probe: need a 16-byte aligned buffer of at least 16 bytes"); return SEED_E_INVALID_ARG; }
    return launch_hbm_read_probe(buf, bytes, sink, (hipStream_t)hip_stream);
}

int seed_accept_resample(const seed_accept_args *args, void *hip_stream) {
    int rc = check_accept_args(args);
    if (rc) return rc;
    if (args->tree != nullptr) {
        TreeInfo ti;
        if ((rc = expand_tree(args->tree, &ti))) return rc;
        return launch_accept_tree(*args, ti, nullptr, nullptr, 0, nullptr, nullptr, (hipStream_t)hip_stream);
    }
    return launch_accept(*args, nullptr, nullptr, 0, nullptr, (hipStream_t)hip_stream);
}

int seed_accept_resample_static(const seed_accept_args *args, void *hip_stream) {
    int rc = check_accept_args(args);
    if (rc) return rc;
    if (args->n_branches == 0) return SEED_OK;
    const long rows = (long)args->n_branches * args->n_target_rows;
    if (rows > kStaticAcceptRows) {
        set_error("accept (static scratch): %ld target rows exceed the maximum of %d", rows, kStaticAcceptRows);
        return SEED_E_CAPACITY;
    }
    void *stats = nullptr;
    rc = accept_static_scratch(&stats);
    if (rc) return rc;
    if (args->tree != nullptr) {
        TreeInfo ti;
        if ((rc = expand_tree(args->tree, &ti))) return rc;
        return launch_accept_tree(*args, ti, stats, nullptr, 0, nullptr, nullptr, (hipStream_t)hip_stream);
    }
    return launch_accept(*args, stats, nullptr, 0, nullptr, (hipStream_t)hip_stream);
}

int seed_sample_probs(const float *probs, int64_t row_stride, const float *u, int32_t *tok_out, int32_t n_rows,
                      int32_t vocab, void *hip_stream) {
    if (n_rows < 0 || vocab < 1 || row_stride < vocab) {
        set_error("sample: need n_rows >= 0, vocab >= 1, row_stride >= vocab");
        return SEED_E_INVALID_ARG;
    }
    if (n_rows == 0) return SEED_OK;
    if (!probs || !u || !tok_out) { set_error("sample: NULL pointer"); return SEED_E_NULL_PTR; }
    return launch_sample_probs(probs, row_stride, u, tok_out, n_rows, vocab, (hipStream_t)hip_stream);
}

int seed_uniform_philox(uint32_t seed, uint32_t stream, float *out, int64_t n, void *hip_stream) {
    if (n < 0) { set_error("uniform: need n >= 0"); return SEED_E_INVALID_ARG; }
    if (n == 0) return SEED_OK;
    if (!out) { set_error("uniform: NULL pointer"); return SEED_E_NULL_PTR; }
    if ((n + 3) / 4 > ((int64_t)1 << 32)) { set_error("uniform: the block counter is 32 bits (n <= 2^34)"); return SEED_E_CAPACITY; }
    return launch_philox_uniform(seed, stream, out, n, (hipStream_t)hip_stream);
}

int seed_verify_step(seed_ctx *c, const seed_step_args *a) {
    if (c == nullptr) { set_error("context is NULL"); return SEED_E_NOT_INIT; }
    if (a == nullptr) { set_error("step args is NULL"); return SEED_E_NULL_PTR; }
    const seed_model_cfg &g = c->cfg;
    const int N = a->n_branches, T = a->rows_per_branch;
    const int prefill = (a->flags & SEED_STEP_PREFILL_SHARED) != 0;
    if (N < 0 || T < 1 || a->shared_len < 0) { set_error("step: need N >= 0, T >= 1, shared_len >= 0"); return SEED_E_INVALID_ARG; }
    if (a->flags & ~(SEED_STEP_PREFILL_SHARED | SEED_STEP_GREEDY | SEED_STEP_COMMIT_ALL)) {
        set_error("step: unknown flag bits 0x%x", a->flags);
        return SEED_E_INVALID_ARG;
    }
    if (N == 0) return SEED_OK;
    if (prefill) {
        if (N != 1) { set_error("step: PREFILL_SHARED needs n_branches == 1"); return SEED_E_SHAPE; }
        if (a->accept != nullptr || (a->flags & SEED_STEP_COMMIT_ALL)) {
            set_error("step: PREFILL_SHARED cannot be combined with accept or COMMIT_ALL");
            return SEED_E_INVALID_ARG;
        }
        if (T > c->L.M_cap) { set_error("step: %d prefill rows exceed the row capacity %d", T, c->L.M_cap); return SEED_E_CAPACITY; }
        if ((long)a->shared_len + T > g.max_shared) {
            set_error("step: shared_len %d + %d rows exceeds max_shared %d", a->shared_len, T, g.max_shared);
            return SEED_E_CAPACITY;
        }
    } else {
        if (N > g.max_branches || T > g.max_rows_per_branch) {
            set_error("step: N=%d, T=%d exceed capacity (%d, %d)", N, T, g.max_branches, g.max_rows_per_branch);
            return SEED_E_CAPACITY;
        }
        if (a->shared_len > g.max_shared) { set_error("step: shared_len exceeds max_shared"); return SEED_E_CAPACITY; }
        if (a->private_len == nullptr) { set_error("step: private_len is NULL"); return SEED_E_NULL_PTR; }
    }
    if (a->row_tok == nullptr) { set_error("step: row_tok is NULL"); return SEED_E_NULL_PTR; }
    TreeInfo tree;
    const bool has_tree = a->tree != nullptr;
    if (has_tree) {
        int rc = expand_tree(a->tree, &tree);
        if (rc) return rc;
        if (prefill || (a->flags & SEED_STEP_COMMIT_ALL)) { set_error("step: a candidate tree cannot be combined with PREFILL_SHARED or COMMIT_ALL"); return SEED_E_INVALID_ARG; }
        if (T != tree.n_par && T != tree.n_nodes) {
            set_error("step: with this tree rows_per_branch must be %d (nodes with children) or %d (all nodes), not %d", tree.n_par, tree.n_nodes, T);
            return SEED_E_SHAPE;
        }
    }
    seed_accept_args acc;
    if (a->accept != nullptr) {
        if (a->flags & SEED_STEP_COMMIT_ALL) { set_error("step: COMMIT_ALL cannot be combined with accept"); return SEED_E_INVALID_ARG; }
        acc = *a->accept;
        acc.n_branches = N;
        acc.n_target_rows = T;
        acc.vocab = g.vocab;
        acc.probs_kind = SEED_KIND_LOGITS;
        acc.greedy = (a->flags & SEED_STEP_GREEDY) ? 1 : acc.greedy;
        acc.tree = a->tree;
        acc.p_or_logits = a->logits_out ? a->logits_out : (const float *)at(c, c->L.logits);
        if (acc.private_len == nullptr) acc.private_len = a->private_len;
        int rc = check_accept_args(&acc);
        if (rc) return rc;
    }
    const bool want_logits = a->logits_out != nullptr || a->accept != nullptr;
    float *logits = want_logits ? (a->logits_out ? a->logits_out : (float *)at(c, c->L.logits)) : nullptr;
    int rc = run_forward(c, N, T, a->shared_len, prefill, a->row_tok, a->private_len, a->branch_slot,
                         has_tree ? &tree : nullptr, logits);
    if (rc) return rc;
    if (a->accept != nullptr && has_tree) {
        int32_t *commit_rows = (int32_t *)at(c, c->L.commit_rows);
        rc = launch_accept_tree(acc, tree, at(c, c->L.acc_stats), a->branch_slot, g.max_branches,
                                (int32_t *)at(c, c->L.status), commit_rows, c->stream);
        if (rc) return rc;
        if (acc.private_len == nullptr) return SEED_OK;      // nothing committed: nothing to move
        // the rows that are kept go to the front of each branch's in-flight region, in every layer
        return launch_kv_compact(c->ws + c->L.kp, c->ws + c->L.vp, c->L.kp_stride, g.n_layers, commit_rows, acc.private_len,
                                 a->branch_slot, g.max_branches, N, g.n_heads, g.head_dim, c->L.cap_p, g.max_private,
                                 c->stream);
    }
    if (a->accept != nullptr)
        return launch_accept(acc, at(c, c->L.acc_stats), a->branch_slot, g.max_branches, (int32_t *)at(c, c->L.status),
                             c->stream);
    if (a->flags & SEED_STEP_COMMIT_ALL)
        return launch_add_len(a->private_len, N, T, a->branch_slot, g.max_branches, c->stream);
    return SEED_OK;
}

int seed_draft_step(seed_ctx *c, const seed_draft_args *a) {
    if (c == nullptr) { set_error("context is NULL"); return SEED_E_NOT_INIT; }
    if (a == nullptr) { set_error("draft args is NULL"); return SEED_E_NULL_PTR; }
    const seed_model_cfg &g = c->cfg;
    const int N = a->n_branches;
    if (N < 0 || a->shared_len < 0) { set_error("draft: need N >= 0, shared_len >= 0"); return SEED_E_INVALID_ARG; }
    if (a->flags & ~SEED_STEP_GREEDY) { set_error("draft: unknown flag bits 0x%x", a->flags); return SEED_E_INVALID_ARG; }
    if (N == 0) return SEED_OK;
    if (N > g.max_branches) { set_error("draft: N=%d exceeds max_branches %d", N, g.max_branches); return SEED_E_CAPACITY; }
    if (a->shared_len > g.max_shared) { set_error("draft: shared_len exceeds max_shared"); return SEED_E_CAPACITY; }
    const int greedy = (a->flags & SEED_STEP_GREEDY) != 0;
    if (!a->row_tok || !a->private_len || !a->tok_out) { set_error("draft: row_tok, private_len, tok_out must be non-NULL"); return SEED_E_NULL_PTR; }
    if (!greedy && !a->u) { set_error("draft: u is NULL"); return SEED_E_NULL_PTR; }
    if (!(a->temperature > 0.f)) { set_error("draft: temperature must be > 0"); return SEED_E_INVALID_ARG; }
    if (a->q_out != nullptr && a->q_stride < g.vocab) { set_error("draft: q_stride < vocab"); return SEED_E_INVALID_ARG; }
    if (a->tok_stride < 1) { set_error("draft: tok_stride must be >= 1"); return SEED_E_INVALID_ARG; }
    float *logits = a->logits_out ? a->logits_out : (float *)at(c, c->L.logits);
    int rc = run_forward(c, N, 1, a->shared_len, 0, a->row_tok, a->private_len, a->branch_slot, nullptr, logits);
    if (rc) return rc;
    return launch_softmax_sample(logits, g.vocab, a->temperature, greedy, a->u, a->q_out, a->q_stride, a->tok_out,
                                 a->tok_stride, a->private_len, N, g.vocab, at(c, c->L.acc_stats),
                                 (int *)at(c, c->L.draft_counters), a->branch_slot, g.max_branches, c->stream);
}

int seed_kv_load(seed_ctx *c, int32_t layer, const void *k_shared, const void *v_shared, int32_t shared_len,
                 const void *k_private, const void *v_private, int32_t n_branches, int32_t private_len) {
    if (c == nullptr) { set_error("context is NULL"); return SEED_E_NOT_INIT; }
    const seed_model_cfg &g = c->cfg;
    if (layer < 0 || layer >= g.n_layers || shared_len < 0 || private_len < 0 || n_branches < 0) {
        set_error("kv_load: bad layer or negative length");
        return SEED_E_INVALID_ARG;
    }
    if (shared_len > g.max_shared || private_len > g.max_private || n_branches > g.max_branches) {
        set_error("kv_load: lengths exceed capacity");
        return SEED_E_CAPACITY;
    }
    if (shared_len > 0 && (!k_shared || !v_shared)) { set_error("kv_load: shared KV is NULL"); return SEED_E_NULL_PTR; }
    if (private_len > 0 && n_branches > 0 && (!k_private || !v_private)) { set_error("kv_load: private KV is NULL"); return SEED_E_NULL_PTR; }
    const Layout &L = c->L;
    const int H = g.n_heads, dh = g.head_dim;
    int rc = SEED_OK;
    if (shared_len > 0) {
        rc = launch_kv_import(c->bf16, false, k_shared, c->ws + L.ks + L.ks_stride * layer, H, shared_len, dh, L.cap_s, c->stream);
        if (rc) return rc;
        rc = launch_kv_import(c->bf16, c->bf16, v_shared, c->ws + L.vs + L.ks_stride * layer, H, shared_len, dh, L.cap_s, c->stream);
        if (rc) return rc;
    }
    if (private_len > 0 && n_branches > 0) {
        rc = launch_kv_import(c->bf16, false, k_private, c->ws + L.kp + L.kp_stride * layer, n_branches * H, private_len, dh, L.cap_p, c->stream);
        if (rc) return rc;
        rc = launch_kv_import(c->bf16, c->bf16, v_private, c->ws + L.vp + L.kp_stride * layer, n_branches * H, private_len, dh, L.cap_p, c->stream);
    }
    return rc;
}

int seed_verify_status(seed_ctx *c, int32_t *host_status) {
    if (c == nullptr) { set_error("context is NULL"); return SEED_E_NOT_INIT; }
    if (host_status == nullptr) { set_error("host_status is NULL"); return SEED_E_NULL_PTR; }
    int rc = hip_fail(hipMemcpyAsync(host_status, at(c, c->L.status), 4, hipMemcpyDeviceToHost, c->stream), "status copy");
    if (rc) return rc;
    rc = hip_fail(hipStreamSynchronize(c->stream), "stream sync");
    if (rc) return rc;
    return hip_fail(hipMemsetAsync(at(c, c->L.status), 0, 4, c->stream), "status clear");
}

}  // extern "C"
