// Tree-KV attention for the verify step (bf16 cache, MFMA).
//
// Every query row (branch b, draft position j) attends to three key segments: the shared prefix (the
// same for all branches -- the paper's Thought Generator runs all n branches from one prompt, Section
// 3.2, and its Limitations section proposes caching that common prefix), the branch's private context,
// and causally the in-flight rows 0..j of its own branch (the per-branch gamma-by-context causal mask;
// the tree-attention idea of Section 2.2 / Appendix "Details of Tree Attention" at branch granularity).
//
// The shared segment is the bulk of the bytes; it is processed for ALL N*gamma rows of a head at once, so
// each shared K/V byte is read from HBM once per step instead of once per branch.  Work is cut into
// independent wavefront tasks (head, group of <= 32 query rows, key range); each task runs a
// flash-decoding loop over 32-key chunks entirely in registers:
//   S^T = K . Q^T          v_mfma_f32_16x16x32_bf16, A = K fragment (16 keys x 32 dims), B = Q fragment
//   online softmax         per query row = per MFMA column: in-lane max/sum + two xor-shuffles across
//                          the four 16-lane groups
//   O^T += V^T . P^T       A = V^T fragment (16 dims x 32 keys; V is cached transposed so this is one
//                          16-byte load per lane), B = P^T built in registers from the S^T accumulators
// (q and P are carried as hi/lo bf16 pairs, two MFMAs each, so that rounding them does not dominate the
// error of the attention output) and writes an unnormalised partial (max, sum, O) per (row, head, key range); a small merge kernel
// combines the partials by log-sum-exp and emits the bf16 activation tile of the O projection.
//
// The two S^T tiles of a 32-key chunk use the key order key = 8*(i/4) + (i%4) (+4 for the second tile),
// which makes lane group g hold exactly keys 8g..8g+7 -- the B-operand layout the P.V MFMA wants.
#include "seed_internal.h"
#include "device_utils.h"

namespace seedv {
namespace {

struct AttnParams {
    const uint16_t *q;        // [2][Mq][H*DH] bf16: hi plane, then lo plane (q = hi + lo)
    size_t q_plane;           // elements between the planes
    const uint16_t *k_shared; // [H][cap_s][DH]
    const uint16_t *vt_shared;// [H][DH][cap_s]
    const uint16_t *k_priv;   // [Nmax][H][cap_p][DH]
    const uint16_t *vt_priv;  // [Nmax][H][DH][cap_p]
    const int32_t *private_len;
    const float *k_new;       // [M][H*DH] fp32: rotated keys of this step's rows (in flight)
    const float *v_new;       // [M][H*DH] fp32: values of this step's rows
    float *o_part;            // [P][Mq][H][DH]
    float *ml_part;           // [P][Mq][H][2]
    int M, Mq, N, T, H;
    int S;                    // shared keys visible to every row (prefill: keys before the chunk)
    int prefill_shared;       // rows additionally see shared keys S .. S+j (their own chunk, causal)
    int cap_s, cap_p, max_private;
    int n_groups;             // ceil(Mq / 32): query-row groups of the shared pass
    int ks_shared;            // key ranges of the shared pass
    int keys_per_range;       // multiple of 32
    int ks_priv;              // key ranges of the private pass (0 in prefill)
    int groups_priv;          // ceil(T / 32)
    float scale_log2e;
};

template <int DH>
__device__ void attn_task(const AttnParams &P, int h, int row0, int rows_hi, const uint16_t *kbase,
                          const uint16_t *vtbase, int cap, int kbeg, int kend, int lim0, int row_ref,
                          int inc, int part) {
    constexpr int KS = DH / 32;   // k-steps of the QK^T contraction
    constexpr int DT = DH / 16;   // d-tiles of the output
    const int lane = threadIdx.x & 63, g = lane >> 4, col = lane & 15;
    const int HD = P.H * DH;

    // query fragments: B operand, lane holds Q[row0 + t*16 + col][h*DH + ks*32 + 8g .. +8]
    bf16x8 qf[2][KS][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const uint16_t *qp = P.q + (size_t)min(row0 + t * 16 + col, P.Mq - 1) * HD + h * DH + ks * 32 + 8 * g;
            qf[t][ks][0] = *reinterpret_cast<const bf16x8 *>(qp);
            qf[t][ks][1] = *reinterpret_cast<const bf16x8 *>(qp + P.q_plane);
        }

    int limit[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int r = row0 + t * 16 + col;
        limit[t] = (r < rows_hi) ? lim0 + inc * (r - row_ref) : 0;
    }

    f32x4 o[DT][2];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int t = 0; t < 2; ++t) o[dt][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};

    const int krow = 8 * (col >> 2) + (col & 3);   // key (within the chunk) of A-operand row `col`, tile 0
    const int wv = threadIdx.x >> 6;                      // the 4 wavefronts of the workgroup interleave chunks
    for (int c = kbeg + 32 * wv; c < kend; c += 128) {
        f32x4 s[2][2];                              // [key tile][row tile]
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const uint16_t *kp = kbase + (size_t)(c + krow + 4 * kt) * DH + 8 * g;
            bf16x8 kf[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[ks] = *reinterpret_cast<const bf16x8 *>(kp + ks * 32);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qf[t][ks][1], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qf[t][ks][0], acc, 0, 0, 0);
                }
                s[kt][t] = acc;
            }
        }
        bf16x8 pf[2][2];   // [row tile][hi|lo]
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            // lane holds keys c + 8g + {0..3} (tile 0) and c + 8g + {4..7} (tile 1) of query row `col`
            float sv[8];
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int key = c + 8 * g + i;
                float v = s[i >> 2][t][i & 3] * P.scale_log2e;
                v = (key < limit[t] && key < kend) ? v : -INFINITY;
                sv[i] = v;
                mx = fmaxf(mx, v);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[t], mx);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run[t] - m_use);
            float psum = 0.f;
            float pv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                pv[i] = __builtin_amdgcn_exp2f(sv[i] - m_use);
                psum += pv[i];
            }
            l_run[t] = l_run[t] * alpha + psum;      // per-lane partial sum; groups are combined at the end
            m_run[t] = m_new;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt][t] *= alpha;
            u32x4 wh, wl;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint16_t h0, l0, h1, l1;
                split_bf16(pv[2 * i], h0, l0);
                split_bf16(pv[2 * i + 1], h1, l1);
                wh[i] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                wl[i] = (uint32_t)l0 | ((uint32_t)l1 << 16);
            }
            pf[t][0] = *reinterpret_cast<bf16x8 *>(&wh);
            pf[t][1] = *reinterpret_cast<bf16x8 *>(&wl);
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            // A operand: V^T[d = dt*16 + col][keys c + 8g .. +8]
            const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(vtbase + (size_t)(dt * 16 + col) * cap + c + 8 * g);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                o[dt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[t][1], o[dt][t], 0, 0, 0);
                o[dt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[t][0], o[dt][t], 0, 0, 0);
            }
        }
    }
    // ---- merge the four wavefronts' partial results through LDS, write ONE partial per workgroup ----
    // (fixed order: deterministic; cuts the partial traffic to global memory fourfold)
    __shared__ float sm_m[4][32], sm_l[4][32];
    __shared__ float sm_o[4][32][DH + 4];
    float scale[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        float l = l_run[t];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (g == 0) {
            sm_m[wv][t * 16 + col] = m_run[t];
            sm_l[wv][t * 16 + col] = l;
        }
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int rr = t * 16 + col;
        float mstar = sm_m[0][rr];
#pragma unroll
        for (int i = 1; i < 4; ++i) mstar = fmaxf(mstar, sm_m[i][rr]);
        scale[t] = (m_run[t] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run[t] - mstar);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const f32x4 v = o[dt][t] * scale[t];
            *reinterpret_cast<f32x4 *>(&sm_o[wv][rr][dt * 16 + 4 * g]) = v;
        }
    }
    __syncthreads();
    // wavefront wv finishes rows wv*8 .. wv*8+7: lanes own DH/64 consecutive dims
    constexpr int PERD = DH / 64;
    for (int rr = wv * 8; rr < wv * 8 + 8; ++rr) {
        const int r = row0 + rr;
        if (r >= rows_hi) continue;
        float mstar = sm_m[0][rr];
#pragma unroll
        for (int i = 1; i < 4; ++i) mstar = fmaxf(mstar, sm_m[i][rr]);
        float L = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            L += (sm_m[i][rr] == -INFINITY) ? 0.f : sm_l[i][rr] * __builtin_amdgcn_exp2f(sm_m[i][rr] - mstar);
        float *op = P.o_part + (((size_t)part * P.Mq + r) * P.H + h) * DH + lane * PERD;
#pragma unroll
        for (int i = 0; i < PERD; ++i) {
            const int d = lane * PERD + i;
            op[i] = ((sm_o[0][rr][d] + sm_o[1][rr][d]) + sm_o[2][rr][d]) + sm_o[3][rr][d];
        }
        if (lane == 0) {
            float *mp = P.ml_part + (((size_t)part * P.Mq + r) * P.H + h) * 2;
            mp[0] = mstar;
            mp[1] = L;
        }
    }
}

// In-flight segment: row j of a branch against rows 0..j of the same branch (the causal part of the tree
// mask).  At most T keys per row, so it runs in plain fp32 on the vector ALUs from an fp32 side copy of the
// new keys / values: the rows of one step see each other unrounded, while the cache keeps bf16.
// One wavefront per (row, head); lanes own DH/64 dims; dot products are wavefront-shuffle reductions.
template <int DH>
__device__ void inflight_task(const AttnParams &P, int itask) {
    constexpr int PER = DH / 64;
    const int lane = threadIdx.x & 63;
    const int r = itask / P.H, h = itask - r * P.H;
    if (r >= P.M) return;
    const int b = r / P.T, j = r - b * P.T;
    const int HD = P.H * DH;
    float qv[PER], o[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const size_t e = (size_t)r * HD + h * DH + lane * PER + i;
        qv[i] = bf2f(P.q[e]) + bf2f(P.q[e + P.q_plane]);
        o[i] = 0.f;
    }
    float m = -INFINITY, l = 0.f;
    for (int jj = 0; jj <= j; ++jj) {
        const size_t e = (size_t)(b * P.T + jj) * HD + h * DH + lane * PER;
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < PER; ++i) s = fmaf(qv[i], P.k_new[e + i], s);
        s = wave_reduce_sum(s) * P.scale_log2e;
        const float m_new = fmaxf(m, s);
        const float alpha = exp2f(m - m_new), p = exp2f(s - m_new);
        l = l * alpha + p;
#pragma unroll
        for (int i = 0; i < PER; ++i) o[i] = o[i] * alpha + p * P.v_new[e + i];
        m = m_new;
    }
    const int part = P.ks_shared + P.ks_priv;
    float *op = P.o_part + (((size_t)part * P.Mq + r) * P.H + h) * DH + lane * PER;
#pragma unroll
    for (int i = 0; i < PER; ++i) op[i] = o[i];
    if (lane == 0) {
        float *mp = P.ml_part + (((size_t)part * P.Mq + r) * P.H + h) * 2;
        mp[0] = m;
        mp[1] = l;
    }
}

template <int DH>
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnParams P) {
    // workgroup tasks: shared (head, row group, key range), private (branch, head, row group, key range);
    // then four in-flight (row, head) wavefront tasks per workgroup
    const int task = blockIdx.x;
    const int n_shared = P.H * P.n_groups * P.ks_shared;
    if (task < n_shared) {
        const int ks = task % P.ks_shared;
        const int grp = (task / P.ks_shared) % P.n_groups;
        const int h = task / (P.ks_shared * P.n_groups);
        const int total = P.prefill_shared ? P.S + P.M : P.S;
        const int kbeg = ks * P.keys_per_range;
        const int kend = min(total, kbeg + P.keys_per_range);
        // verify: every row sees all S shared keys; prefill: row j sees keys < S + j + 1
        attn_task<DH>(P, h, grp * 32, P.M, P.k_shared + (size_t)h * P.cap_s * DH,
                      P.vt_shared + (size_t)h * DH * P.cap_s, P.cap_s, kbeg, max(kbeg, kend),
                      P.prefill_shared ? P.S + 1 : P.S, 0, P.prefill_shared ? 1 : 0, ks);
        return;
    }
    const int ptask = task - n_shared;
    const int n_priv = P.prefill_shared ? 0 : P.N * P.H * P.groups_priv * P.ks_priv;
    if (ptask >= n_priv) {
        if (!P.prefill_shared) inflight_task<DH>(P, (ptask - n_priv) * 4 + (threadIdx.x >> 6));
        return;
    }
    const int ks = ptask % P.ks_priv;
    const int grp = (ptask / P.ks_priv) % P.groups_priv;
    const int h = (ptask / (P.ks_priv * P.groups_priv)) % P.H;
    const int b = ptask / (P.ks_priv * P.groups_priv * P.H);
    const int pl = min(max(P.private_len[b], 0), P.max_private);
    const int total = pl;                             // committed private context; in-flight rows are separate
    const int kbeg = ks * P.keys_per_range;
    const int kend = min(total, kbeg + P.keys_per_range);
    const int row_first = b * P.T;
    // every row of the branch sees all pl committed private keys
    attn_task<DH>(P, h, row_first + grp * 32, row_first + P.T,
                  P.k_priv + ((size_t)b * P.H + h) * P.cap_p * DH, P.vt_priv + ((size_t)b * P.H + h) * DH * P.cap_p,
                  P.cap_p, kbeg, max(kbeg, kend), pl, row_first, 0, P.ks_shared + ks);
}

// Combine the partials of one (row, head) by log-sum-exp and write the bf16 activation (fragment-packed,
// K = H*DH) that feeds the O projection.  One wavefront per (row, head).
template <int DH>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float *o_part, const float *ml_part, uint16_t *act,
                                                         int M, int Mq, int Mp, int H, int n_part_shared,
                                                         int n_part_total, int prefill_shared) {
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (w >= Mp * H) return;
    const int r = w / H, h = w - r * H;
    const int KT = (H * DH) >> 5;
    constexpr int PER = DH / 64;     // output dims per lane
    if (r >= M) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const size_t o = packed_offset(r, h * DH + lane * PER + i, KT);
            act[o] = 0;
            act[o + kActLoOffset] = 0;
        }
        return;
    }
    const int np = prefill_shared ? n_part_shared : n_part_total;
    float mmax = -INFINITY;
    for (int p = 0; p < np; ++p) mmax = fmaxf(mmax, ml_part[(((size_t)p * Mq + r) * H + h) * 2]);
    float acc[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) acc[i] = 0.f;
    float L = 0.f;
    for (int p = 0; p < np; ++p) {
        const size_t base = ((size_t)p * Mq + r) * H + h;
        const float m = ml_part[base * 2], l = ml_part[base * 2 + 1];
        if (l == 0.f) continue;                       // empty key range
        const float wgt = __builtin_amdgcn_exp2f(m - mmax);
        L += l * wgt;
#pragma unroll
        for (int i = 0; i < PER; ++i) acc[i] += o_part[base * DH + lane * PER + i] * wgt;
    }
    const float inv = L > 0.f ? 1.0f / L : 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const size_t o = packed_offset(r, h * DH + lane * PER + i, KT);
        split_bf16(acc[i] * inv, act[o], act[o + kActLoOffset]);
    }
}

}  // namespace

// Number of partial slots per (row, head) for a given configuration; also fills the split parameters.
void attn_bf16_plan(int Mq, int H, int N, int T, int total_shared_keys, int cap_priv_keys, int prefill_shared,
                    int *ks_shared, int *keys_per_range, int *ks_priv) {
    // aim for ~512 workgroups of four wavefronts; a key range is a multiple of 128 keys (one 32-key chunk per
    // wavefront and round), at least 128 keys
    const int n_groups = (Mq + 31) / 32;
    const int base_tasks = H * n_groups;
    const int want = (512 + base_tasks - 1) / base_tasks;
    int rounds = (total_shared_keys + 127) / 128;      // 128-key rounds in the shared segment
    if (rounds < 1) rounds = 1;
    int ks = want < rounds ? want : rounds;
    if (ks < 1) ks = 1;
    if (ks > 32) ks = 32;
    const int per = ((rounds + ks - 1) / ks) * 128;
    ks = (rounds * 128 + per - 1) / per;
    *ks_shared = ks;
    *keys_per_range = per;
    *ks_priv = (prefill_shared || cap_priv_keys <= 0) ? 0 : (cap_priv_keys + per - 1) / per;
    (void)N;
    (void)T;
}

int launch_attn_bf16(int dh, const void *q, size_t q_plane, const void *k_shared, const void *vt_shared, const void *k_priv,
                     const void *vt_priv, const int32_t *private_len, const float *k_new, const float *v_new,
                     float *o_part, float *ml_part, void *act,
                     int M, int Mp, int Mq, int N, int T, int H, int S, int prefill_shared, int cap_s, int cap_p,
                     int max_private, int ks_shared, int keys_per_range, int ks_priv, hipStream_t st) {
    AttnParams P;
    P.q = (const uint16_t *)q;
    P.q_plane = q_plane;
    P.k_shared = (const uint16_t *)k_shared;
    P.vt_shared = (const uint16_t *)vt_shared;
    P.k_priv = (const uint16_t *)k_priv;
    P.vt_priv = (const uint16_t *)vt_priv;
    P.private_len = private_len;
    P.k_new = k_new;
    P.v_new = v_new;
    P.o_part = o_part;
    P.ml_part = ml_part;
    P.M = M; P.Mq = Mq; P.N = N; P.T = T; P.H = H; P.S = S;
    P.prefill_shared = prefill_shared;
    P.cap_s = cap_s; P.cap_p = cap_p; P.max_private = max_private;
    P.n_groups = (Mq + 31) / 32;
    P.ks_shared = ks_shared;
    P.keys_per_range = keys_per_range;
    P.ks_priv = ks_priv;
    P.groups_priv = (T + 31) / 32;
    P.scale_log2e = 1.4426950408889634f / sqrtf((float)dh);
    const int blocks = H * P.n_groups * ks_shared + (prefill_shared ? 0 : N * H * P.groups_priv * ks_priv + (M * H + 3) / 4);
    const int n_total = ks_shared + ks_priv + 1;      // + the in-flight slot
    if (dh == 128) {
        hipLaunchKernelGGL(attn_partial_kernel<128>, dim3(blocks), dim3(256), 0, st, P);
        hipLaunchKernelGGL(attn_merge_kernel<128>, dim3((Mp * H + 3) / 4), dim3(256), 0, st, o_part, ml_part,
                           (uint16_t *)act, M, Mq, Mp, H, ks_shared, n_total, prefill_shared);
    } else if (dh == 64) {
        hipLaunchKernelGGL(attn_partial_kernel<64>, dim3(blocks), dim3(256), 0, st, P);
        hipLaunchKernelGGL(attn_merge_kernel<64>, dim3((Mp * H + 3) / 4), dim3(256), 0, st, o_part, ml_part,
                           (uint16_t *)act, M, Mq, Mp, H, ks_shared, n_total, prefill_shared);
    } else {
        set_error("bf16 attention supports head_dim 64 or 128, got %d", dh);
        return SEED_E_SHAPE;
    }
    return hip_fail(hipGetLastError(), "attention launch");
}

}  // namespace seedv
