// Tree-KV attention for the verify step (bf16 cache, MFMA).
//
// Every query row (branch b, draft position j) attends to three key segments: the shared prefix (the
// same for all branches -- the paper's Thought Generator runs all n branches from one prompt, Section
// 3.2, and its Limitations section proposes caching that common prefix), the branch's private context,
// and causally the in-flight rows 0..j of its own branch (the per-branch gamma-by-context causal mask;
// the tree-attention idea of Section 2.2 / Appendix "Details of Tree Attention" at branch granularity).
//
// The shared segment is the bulk of the bytes; it is processed for all N*gamma rows of a head together, so
// each shared K/V byte is read from HBM once per step instead of once per branch.  Work is cut into
// independent tasks (head, 16 query rows, key range of one segment); a task walks its range in 32-key chunks,
// flash-decoding style, with everything but K and V in registers:
//   S^T = K . Q^T          v_mfma_f32_16x16x32_bf16, A = K fragment (16 keys x 32 dims), B = Q fragment
//   online softmax         per query row = per MFMA column: in-lane max/sum + two xor-shuffles across
//                          the four 16-lane groups
//   O^T += V^T . P^T       A = V^T fragment (16 dims x 32 keys; V is cached transposed, chunk by chunk, so
//                          this is one 16-byte load per lane), B = P^T built in registers from S^T
// (q and P are carried as hi/lo bf16 pairs, two MFMAs each, so that rounding them does not dominate the
// error of the attention output) and leaves an unnormalised partial (max, sum, O) per (row, head, key range);
// the partials of a (row, head) are combined by log-sum-exp into the hi/lo bf16 activation tile of the O
// projection.  Two forms of a task:
//   attn_task      the four wavefronts of a workgroup interleave the chunks (K/V straight to registers, next
//                  chunk in flight) and merge through LDS: steps of at most 16 rows, and every private segment;
//   attn_task_lds  steps with several row groups: a workgroup walks one shared key range for up to four row
//                  groups, a wavefront each; every chunk is fetched once, staged through LDS in fragment order.
//
// Verify / decode steps run everything in ONE launch: the tasks read q, k, v straight from the fp32 output
// of the QKV projection and apply the rotary embedding on the fly; the task of a branch's private segment
// also runs its in-flight rows and appends their rotated keys and values to the private cache; with at most
// 16 rows the workgroup that finishes last for a head (a per-head arrival counter) merges that head's
// partials, otherwise a merge launch follows.  The shared-prefix prefill keeps the three-launch form (rotary
// + cache append, partials, merge): its rows read the keys of their own chunk from the cache.
// Steps with several row groups, at most eight rows per branch and short private contexts (the paper's shapes:
// many branches, a few draft tokens each) use a lighter form of the branch tasks: one WAVEFRONT per (branch,
// head) -- attn_task<SOLO> over the private keys, then inflight_solo for all in-flight rows of the head -- four
// heads per workgroup, dispatched ahead of the shared-segment workgroups, whose number is chosen so that the
// whole launch is resident at once (two workgroups per CU).
//
// The two S^T tiles of a 32-key chunk use the key order key = 8*(i/4) + (i%4) (+4 for the second tile),
// which makes lane group g hold exactly keys 8g..8g+7 -- the B-operand layout the P.V MFMA wants.
#include "seed_internal.h"
#include "device_utils.h"

namespace seedv {
namespace {

constexpr int kRowTiles = 1;   // 16-row query tiles per task

struct AttnParams {
    const uint16_t *q;        // [2][Mq][H*DH] bf16: hi plane, then lo plane (q = hi + lo)
    size_t q_plane;           // elements between the planes
    const uint16_t *k_shared; // [H][cap_s][DH]
    const uint16_t *vt_shared;// [H][cap_s/32][DH][32]  (vt_offset)
    const uint16_t *k_priv;   // [Nmax][H][cap_p][DH]
    const uint16_t *vt_priv;  // [Nmax][H][cap_p/32][DH][32]
    const int32_t *private_len;
    const int32_t *slot;      // branch -> cache slot (NULL: identity); private_len is indexed by slot
    int n_slots;
    float *o_part;            // [P][Mq][H][DH]
    float *ml_part;           // [P][Mq][H][2]
    // single-launch form only:
    const float *qkv;         // [M][3*H*DH] fp32: q | k | v of this step's rows, before the rotary embedding
    const float *rope;        // [pos][DH/2][cos, sin]
    uint16_t *k_priv_w, *vt_priv_w;   // the private cache again, for the append
    int *counters;            // [H] arrival counters, zero on entry and left zero
    uint16_t *act;            // merged output, fragment-packed hi/lo activation of the O projection
    int32_t *status;
    // candidate trees (NULL: the rows of a branch are a chain, row j at depth j seeing rows 0..j)
    const int32_t *row_depth;             // [T] depth of row j in its branch's tree = its position offset
    const unsigned long long *row_anc;    // [T] bit jj set: row jj is row j itself or one of its ancestors
    int Mp;
    int wave_tasks;           // several row groups: shared tasks are attn_task_lds workgroups
    int gpw, n_quads;         // row groups per such workgroup (<= 4), workgroups per (head, key range)
    int merge_in_launch;      // the last workgroup of a head merges its rows (few rows); else a second launch
    int pair_xcd;             // shared tasks of one (head, key range) on ids L, L+8, ...: one XCD, one L2
    int solo_branch;          // branch tasks: a wavefront per (branch, head), four heads per workgroup,
    int n_solo;               // ... which are the first n_solo workgroups of the launch
    int M, Mq, N, T, H;
    int S;                    // shared keys visible to every row (prefill: keys before the chunk)
    int prefill_shared;       // rows additionally see shared keys S .. S+j (their own chunk, causal)
    int cap_s, cap_p, max_private;
    int n_groups;             // query-row groups of the shared pass (32 rows each; 16 when M <= 16)
    int ks_shared;            // key ranges of the shared pass
    int keys_per_range;       // shared ranges: multiple of 32
    int keys_per_range_priv;  // private ranges: multiple of 128
    int ks_priv;              // key ranges of the private pass (0 in prefill)
    int groups_priv;          // row groups of one branch
    float scale_log2e;
};

// Position and validity of query row r in a verify / decode step: branch b = r / T continues its private
// context, so the row sits at S + private_len[b] + j.  An out-of-range length is clamped (and flagged by the
// in-flight task, which then drops the cache append).
// Cache slot of branch b of this call (an out-of-range entry is clamped; the in-flight task flags it).
__device__ __forceinline__ int slot_of(const AttnParams &P, int b) {
    return P.slot != nullptr ? min(max(P.slot[b], 0), P.n_slots - 1) : b;
}
__device__ __forceinline__ int clamped_private_len(const AttnParams &P, int b) {
    return min(max(P.private_len[slot_of(P, b)], 0), P.max_private);
}

// Query fragments (B operand, hi/lo) of row r, head h from the fp32 QKV output with the rotary embedding
// applied: lane group g holds dims ks*32 + 8g .. +8 of every k-step; a dim below DH/2 pairs with dim + DH/2,
// i.e. k-step ks with ks + KS/2 at the same in-lane offsets.  Two stages, so that the loads that depend on
// nothing (the branch's private length, the raw q values) are in flight before the K / V chunk is requested
// and only the angle table waits for the length.
template <int DH>
struct RawQ {
    float lo[DH / 64][8], hi[DH / 64][8];   // dims d0 .. d0+8 and d0 + DH/2 .. of each k-step pair
    int pl;                                  // private length of the row's branch, as loaded
};
template <int DH>
__device__ __forceinline__ void load_q_raw(const AttnParams &P, int r, int h, int g, RawQ<DH> &q) {
    constexpr int KS = DH / 32, HALF = DH / 2;
    const float *row = P.qkv + (size_t)r * 3 * P.H * DH + h * DH;
#pragma unroll
    for (int ks = 0; ks < KS / 2; ++ks) {
        const int d0 = ks * 32 + 8 * g;
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            *reinterpret_cast<f32x4 *>(&q.lo[ks][4 * v]) = *reinterpret_cast<const f32x4 *>(row + d0 + 4 * v);
            *reinterpret_cast<f32x4 *>(&q.hi[ks][4 * v]) = *reinterpret_cast<const f32x4 *>(row + d0 + HALF + 4 * v);
        }
    }
}
template <int DH, bool TREE>
__device__ __forceinline__ void rotate_q(const AttnParams &P, int r, int g, const RawQ<DH> &q,
                                         bf16x8 (&qf)[DH / 32][2]) {
    constexpr int KS = DH / 32;
    const int j = r % P.T;
    const int dj = TREE ? P.row_depth[j] : j;      // candidate tree: a row sits at its depth, not its index
    const int pos = P.S + min(max(q.pl, 0), P.max_private) + dj;
    const float *tb = P.rope + (size_t)pos * DH;
#pragma unroll
    for (int ks = 0; ks < KS / 2; ++ks) {
        const int d0 = ks * 32 + 8 * g;
        float cs[16];
#pragma unroll
        for (int v = 0; v < 4; ++v)
            *reinterpret_cast<f32x4 *>(&cs[4 * v]) = *reinterpret_cast<const f32x4 *>(tb + 2 * d0 + 4 * v);
        const float *a = q.lo[ks], *bb = q.hi[ks];
        u32x4 ah, al, bh, bl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint16_t h0, l0, h1, l1;
            split_bf16(a[2 * e] * cs[4 * e] - bb[2 * e] * cs[4 * e + 1], h0, l0);
            split_bf16(a[2 * e + 1] * cs[4 * e + 2] - bb[2 * e + 1] * cs[4 * e + 3], h1, l1);
            ah[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            al[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
            split_bf16(bb[2 * e] * cs[4 * e] + a[2 * e] * cs[4 * e + 1], h0, l0);
            split_bf16(bb[2 * e + 1] * cs[4 * e + 2] + a[2 * e + 1] * cs[4 * e + 3], h1, l1);
            bh[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            bl[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
        }
        qf[ks][0] = *reinterpret_cast<bf16x8 *>(&ah);
        qf[ks][1] = *reinterpret_cast<bf16x8 *>(&al);
        qf[ks + KS / 2][0] = *reinterpret_cast<bf16x8 *>(&bh);
        qf[ks + KS / 2][1] = *reinterpret_cast<bf16x8 *>(&bl);
    }
}

// One 32-key chunk for the RT row tiles of a task: S^T = K.Q^T, online softmax, O^T += V^T.P^T.
// kf / vf are the chunk's A operands (any source), c its first key.  full (uniform over the wavefront): every
// key of the chunk is visible to every row of the task, no mask.
// The loop around this runs on two wavefronts per SIMD and is bound by instruction issue and latency, not by
// the MFMAs or by memory, so the softmax is kept short (about half the vector instructions of the textbook
// form): the running maximum is a REFERENCE, not the exact maximum -- it moves (and O and the sum are rescaled)
// only when a chunk's maximum exceeds it by more than kRescaleStep in the exponent, so p <= 2^kRescaleStep and
// most chunks skip the rescale altogether (the partial (m, l, O) stays self-consistent, the merge divides by
// l); scores are scaled inside the fused multiply-add that feeds exp2; the hi/lo split uses the hardware
// bf16 conversion.
constexpr float kRescaleStep = 8.f;
template <int DH>
__device__ __forceinline__ void chunk_update(const bf16x8 (&kf)[2][DH / 32], const bf16x8 (&vf)[DH / 16],
                                             const bf16x8 (&qf)[kRowTiles][DH / 32][2],
                                             f32x4 (&o)[DH / 16][kRowTiles], float (&m_run)[kRowTiles],
                                             float (&l_run)[kRowTiles], const int (&limit)[kRowTiles], int c,
                                             int kend, float scale_log2e, bool full) {
    constexpr int RT = kRowTiles, KS = DH / 32, DT = DH / 16;
    const int g = (threadIdx.x & 63) >> 4;
    f32x4 s[2][RT];                             // [key tile][row tile]
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kt][ks], qf[t][ks][1], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kt][ks], qf[t][ks][0], acc, 0, 0, 0);
            }
            s[kt][t] = acc;
        }
    }
    bf16x8 pf[RT][2];  // [row tile][hi|lo]
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        // lane holds keys c + 8g + {0..3} (tile 0) and c + 8g + {4..7} (tile 1) of query row `col`
        float sv[8];
        float mx = -INFINITY;
        if (full) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                sv[i] = s[i >> 2][t][i & 3];
                mx = fmaxf(mx, sv[i]);
            }
        } else {
            const int lim = min(limit[t], kend) - (c + 8 * g);      // keys 0 .. lim-1 of this lane's eight
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                sv[i] = i < lim ? s[i >> 2][t][i & 3] : -INFINITY;
                mx = fmaxf(mx, sv[i]);
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        mx *= scale_log2e;                                           // (the scale is positive)
        const bool need = mx > m_run[t] + kRescaleStep;              // also the first visible key: m_run = -inf
        if (__builtin_amdgcn_ballot_w64(need) != 0) {
            const float alpha = need ? __builtin_amdgcn_exp2f(m_run[t] - mx) : 1.f;
            m_run[t] = need ? mx : m_run[t];
            l_run[t] *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt][t] *= alpha;
        }
        const float neg_m = (m_run[t] == -INFINITY) ? 0.f : -m_run[t];
        float psum = 0.f;
        float pv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            pv[i] = __builtin_amdgcn_exp2f(fmaf(sv[i], scale_log2e, neg_m));
            psum += pv[i];
        }
        l_run[t] += psum;                        // per-lane partial sum; groups are combined at the end
        u32x4 wh, wl;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t h2, l2;
            split_bf16_x2(pv[2 * i], pv[2 * i + 1], h2, l2);
            wh[i] = h2;
            wl[i] = l2;
        }
        pf[t][0] = *reinterpret_cast<bf16x8 *>(&wh);
        pf[t][1] = *reinterpret_cast<bf16x8 *>(&wl);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            o[dt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pf[t][1], o[dt][t], 0, 0, 0);
            o[dt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pf[t][0], o[dt][t], 0, 0, 0);
        }
    }
}

// A wavefront's own partial, straight from the accumulators: lane (col, g) holds dims dt*16 + 4g .. +4 of row
// t*16 + col.  (Plain stores: the merge is a later launch whenever this is used.  Merging in this launch, by
// the workgroup that completes a (head, 16-row group), was measured slower: the last arrivals queue a 75 KB
// read of partials behind their own task, +6 us against a 5.9 us merge launch at full occupancy.)
template <int DH>
__device__ __forceinline__ void store_partial_direct(const AttnParams &P, int h, int row0, int rows_hi, int part,
                                                     const f32x4 (&o)[DH / 16][kRowTiles],
                                                     const float (&m_run)[kRowTiles],
                                                     const float (&l_run)[kRowTiles]) {
    constexpr int RT = kRowTiles, DT = DH / 16;
    const int lane = threadIdx.x & 63, g = lane >> 4, col = lane & 15;
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        float l = l_run[t];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const int r = row0 + t * 16 + col;
        if (r < rows_hi) {
            const size_t base = ((size_t)part * P.Mq + r) * P.H + h;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                *reinterpret_cast<f32x4 *>(P.o_part + base * DH + dt * 16 + 4 * g) = o[dt][t];
            if (g == 0) *reinterpret_cast<float2 *>(P.ml_part + base * 2) = make_float2(m_run[t], l);
        }
    }
}

// One task: a tile of 16 query rows against the keys [kbeg, kend) of one segment.  (The loops over RT row
// tiles are kept general; 32-row tasks were measured no faster: they leave no registers for the second K/V
// buffer and halve the number of workgroups per CU.)
// The four wavefronts of the workgroup interleave the 32-key chunks of the range and merge through LDS into one
// partial (every barrier is reached by all four).  Used for every task of a step with one row group and for
// the private segment; the shared segment of steps with several row groups goes through attn_task_lds.
// SOLO: the wavefront walks the whole range alone, chunk after chunk, and stores its own partial (no LDS, no
// barrier): four such tasks, one per head, share a workgroup (branch tasks of steps with several row groups).
template <int DH, bool FUSED, bool TREE, bool SOLO = false>
__device__ void attn_task(const AttnParams &P, int h, int row0, int rows_hi, const uint16_t *kbase,
                          const uint16_t *vtbase, int cap, int kbeg, int kend, int lim0, int row_ref,
                          int inc, int part, char *smem) {
    constexpr int RT = kRowTiles;
    constexpr int KS = DH / 32;   // k-steps of the QK^T contraction
    constexpr int DT = DH / 16;   // d-tiles of the output
    const int lane = threadIdx.x & 63, g = lane >> 4, col = lane & 15;
    const int HD = P.H * DH;

    // K and V^T fragments of a 32-key chunk (A operands): K rows in the key order described above, two
    // 16-key tiles x KS k-steps; V^T[d = dt*16 + col][keys c + 8g .. +8].  The first chunk is requested before
    // anything else and chunk i+1 while chunk i is computed: their addresses depend on nothing loaded here.
    const int krow = 8 * (col >> 2) + (col & 3);   // key (within the chunk) of A-operand row `col`, tile 0
    const int wv = threadIdx.x >> 6;               // the 4 wavefronts interleave chunks
    auto load_kv = [&](int c, bf16x8 (&kf)[2][KS], bf16x8 (&vf)[DT]) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kf[kt][ks] = *reinterpret_cast<const bf16x8 *>(kbase + (size_t)(c + krow + 4 * kt) * DH + 8 * g + ks * 32);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            vf[dt] = *reinterpret_cast<const bf16x8 *>(vtbase + vt_offset(dt * 16 + col, c + 8 * g, DH));
    };
    const int c0 = SOLO ? kbeg : kbeg + 32 * wv;
    constexpr int CSTEP = SOLO ? 32 : 128;
    // Issue order: the private lengths (oldest, so they can be waited for alone), the K / V chunk, the raw q
    // values; straight-line code, or the compiler drains the load queue at the join of a branch.  Rows past the
    // task's rows are clamped to a valid row and masked later.
    RawQ<DH> qraw[RT];
    if (FUSED) {
#pragma unroll
        for (int t = 0; t < RT; ++t) qraw[t].pl = P.private_len[slot_of(P, min(row0 + t * 16 + col, P.M - 1) / P.T)];
    }
    bf16x8 kf[2][KS], vf[DT];
    load_kv(c0 < kend ? c0 : 0, kf, vf);           // (a wavefront without a chunk reads chunk 0 and drops it)
    if (FUSED) {
#pragma unroll
        for (int t = 0; t < RT; ++t) load_q_raw<DH>(P, min(row0 + t * 16 + col, P.M - 1), h, g, qraw[t]);
        __builtin_amdgcn_sched_barrier(0);
    }

    // query fragments: B operand, lane holds Q[row0 + t*16 + col][h*DH + ks*32 + 8g .. +8]
    bf16x8 qf[RT][KS][2];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        if (FUSED) {
            rotate_q<DH, TREE>(P, min(row0 + t * 16 + col, P.M - 1), g, qraw[t], qf[t]);
        } else {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const uint16_t *qp = P.q + (size_t)min(row0 + t * 16 + col, P.Mq - 1) * HD + h * DH + ks * 32 + 8 * g;
                qf[t][ks][0] = *reinterpret_cast<const bf16x8 *>(qp);
                qf[t][ks][1] = *reinterpret_cast<const bf16x8 *>(qp + P.q_plane);
            }
        }
    }

    int limit[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const int r = row0 + t * 16 + col;
        limit[t] = (r < rows_hi) ? lim0 + inc * (r - row_ref) : 0;
    }

    f32x4 o[DT][RT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int t = 0; t < RT; ++t) o[dt][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m_run[RT], l_run[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        m_run[t] = -INFINITY;
        l_run[t] = 0.f;
    }
    // chunks that end at or below lim_full need no mask: the smallest limit among the task's rows (rows past
    // rows_hi are never stored)
    const int lim_full = min(kend, lim0 + inc * (row0 - row_ref));
    for (int c = c0; c < kend; c += CSTEP) {
        // the next chunk is requested while this one is computed
        bf16x8 kf_next[2][KS], vf_next[DT];
        const bool more = c + CSTEP < kend;           // (uniform)
        if (more) load_kv(c + CSTEP, kf_next, vf_next);
        chunk_update<DH>(kf, vf, qf, o, m_run, l_run, limit, c, kend, P.scale_log2e, __builtin_amdgcn_readfirstlane(c + 32 <= lim_full) != 0);
        if (more) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kf[kt][ks] = kf_next[kt][ks];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) vf[dt] = vf_next[dt];
        }
    }
    if (SOLO) {
        store_partial_direct<DH>(P, h, row0, rows_hi, part, o, m_run, l_run);
        return;
    }
    // ---- merge the four wavefronts' partial results through LDS, write ONE partial per workgroup ----
    // (fixed order: deterministic; cuts the partial traffic to global memory fourfold)
    float (*sm_m)[16 * RT] = reinterpret_cast<float (*)[16 * RT]>(smem);
    float (*sm_l)[16 * RT] = sm_m + 4;
    float (*sm_o)[16 * RT][DH + 4] = reinterpret_cast<float (*)[16 * RT][DH + 4]>(sm_l + 4);
    float scale[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
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
    for (int t = 0; t < RT; ++t) {
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
    // wavefront wv finishes 4*RT of the rows: lanes own DH/64 consecutive dims.  All LDS reads first, no
    // branch but the one around the stores (a wavefront is alone on its SIMD here: every dependent wait shows).
    constexpr int PERD = DH / 64, RW = 4 * RT;
    float mm[RW][4], ll[RW][4], ov[RW][PERD];
#pragma unroll
    for (int q = 0; q < RW; ++q) {
        const int rr = wv * RW + q;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            mm[q][i] = sm_m[i][rr];
            ll[q][i] = sm_l[i][rr];
        }
#pragma unroll
        for (int e = 0; e < PERD; ++e) {
            const int d = lane * PERD + e;
            ov[q][e] = ((sm_o[0][rr][d] + sm_o[1][rr][d]) + sm_o[2][rr][d]) + sm_o[3][rr][d];
        }
    }
#pragma unroll
    for (int q = 0; q < RW; ++q) {
        const int r = row0 + wv * RW + q;
        const float mstar = fmaxf(fmaxf(mm[q][0], mm[q][1]), fmaxf(mm[q][2], mm[q][3]));
        const float mu = (mstar == -INFINITY) ? 0.f : mstar;       // an empty wavefront has l = 0 and m = -inf
        float L = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) L += ll[q][i] * __builtin_amdgcn_exp2f(mm[q][i] - mu);
        if (r < rows_hi) {
            float *op = P.o_part + (((size_t)part * P.Mq + r) * P.H + h) * DH + lane * PERD;
            if (PERD == 2) {
                store2_agent(op, ov[q][0], ov[q][PERD - 1]);
            } else {
#pragma unroll
                for (int e = 0; e < PERD; ++e) store_agent(op + e, ov[q][e]);
            }
            if (lane == 0) store2_agent(P.ml_part + (((size_t)part * P.Mq + r) * P.H + h) * 2, mstar, L);
        }
    }
}

// Shared-segment task of a step with SEVERAL row groups: the workgroup walks one key range for up to four
// row groups at once, a wavefront per group.  Every 32-key chunk is fetched from global memory ONCE per
// workgroup (each thread a few 16-byte pieces, two chunks ahead in registers), stored to LDS in MFMA-fragment
// order (two stages) and read from there by all wavefronts; one barrier per chunk.  The wavefronts write
// their partials straight from the accumulators.  Wavefronts without a row group (n_grp < 4) only help load.
template <int DH, bool FUSED, bool TREE>
__device__ void attn_task_lds(const AttnParams &P, int h, int grp0, int n_grp, const uint16_t *kbase,
                              const uint16_t *vtbase, int kbeg, int kend, int lim0, int inc, int part,
                              char *smem) {
    constexpr int RT = kRowTiles, KS = DH / 32, DT = DH / 16;
    constexpr int PPT = (32 * DH / 8) / 256;       // 16-byte pieces of a K (or V) chunk per thread
    static_assert(RT == 1 && PPT >= 1, "one row tile per wavefront; head_dim >= 64");
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, g = lane >> 4, col = lane & 15;
    const bool active = wv < n_grp;
    const int row0 = (grp0 + (active ? wv : 0)) * 16;
    const int HD = P.H * DH;
    bf16x8 (*kst)[2 * KS * 64] = reinterpret_cast<bf16x8 (*)[2 * KS * 64]>(smem);                       // [2]
    bf16x8 (*vst)[DT * 64] = reinterpret_cast<bf16x8 (*)[DT * 64]>(smem + 2 * sizeof(bf16x8) * 2 * KS * 64);

    // this thread's pieces: where they come from in the chunk and which fragment slot they fill.
    // K chunk [32 keys][DH]: piece (key, dp) is lane (col, g) of fragment (kt, ks) with key = 8*(col/4) + col%4
    // + 4*kt, dp = 4*ks + g.  V chunk [DH][32 keys] (chunk-tiled cache): piece (d, kp) is lane (d%16, kp) of
    // fragment dt = d/16.  Within its 16-lane group a piece sits at col ^ dp (K) or col ^ 4*kp (V): the threads
    // that store one key's (one dim's) pieces would otherwise all hit the same four LDS banks (the counters
    // showed 61 % of the LDS cycles of this kernel as bank conflicts); the reads undo the same exchange.
    int k_src[PPT], k_dst[PPT], v_src[PPT], v_dst[PPT];
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
        const int j = tid + 256 * i;
        const int key = j / (DH / 8), dp = j % (DH / 8);
        k_src[i] = key * DH + dp * 8;
        k_dst[i] = ((((key >> 2) & 1) * KS + (dp >> 2)) * 64) + (dp & 3) * 16 + ((((key >> 3) << 2) | (key & 3)) ^ (dp & 15));
        const int d = j >> 2, kp = j & 3;
        v_src[i] = d * 32 + kp * 8;
        v_dst[i] = (d >> 4) * 64 + kp * 16 + ((d & 15) ^ (4 * kp));
    }
    const int nch = (kend - kbeg + 31) >> 5;        // chunks of the range
    auto gload = [&](int i, bf16x8 (&kr)[PPT], bf16x8 (&vr)[PPT]) {
        const int c = kbeg + 32 * max(min(i, nch - 1), 0);     // past the end: the last chunk again (dropped)
#pragma unroll
        for (int u = 0; u < PPT; ++u) {
            kr[u] = *reinterpret_cast<const bf16x8 *>(kbase + (size_t)c * DH + k_src[u]);
            vr[u] = *reinterpret_cast<const bf16x8 *>(vtbase + (size_t)(c >> 5) * DH * 32 + v_src[u]);
        }
    };
    auto lstore = [&](int stage, const bf16x8 (&kr)[PPT], const bf16x8 (&vr)[PPT]) {
#pragma unroll
        for (int u = 0; u < PPT; ++u) {
            kst[stage][k_dst[u]] = kr[u];
            vst[stage][v_dst[u]] = vr[u];
        }
    };

    // issue order as in attn_task: private lengths, the first two chunks, the raw q values; no branches
    const int qrow = min(row0 + col, P.M - 1);
    RawQ<DH> qraw;
    if (FUSED) qraw.pl = P.private_len[slot_of(P, qrow / P.T)];
    bf16x8 kr0[PPT], vr0[PPT], kr1[PPT], vr1[PPT];
    gload(0, kr0, vr0);
    gload(1, kr1, vr1);
    bf16x8 qf[RT][KS][2];
    if (FUSED) {
        load_q_raw<DH>(P, qrow, h, g, qraw);
        __builtin_amdgcn_sched_barrier(0);
        rotate_q<DH, TREE>(P, qrow, g, qraw, qf[0]);
    } else {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const uint16_t *qp = P.q + (size_t)min(row0 + col, P.Mq - 1) * HD + h * DH + ks * 32 + 8 * g;
            qf[0][ks][0] = *reinterpret_cast<const bf16x8 *>(qp);
            qf[0][ks][1] = *reinterpret_cast<const bf16x8 *>(qp + P.q_plane);
        }
    }
    int limit[RT];
    limit[0] = (active && row0 + col < P.M) ? lim0 + inc * (row0 + col) : 0;
    f32x4 o[DT][RT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt][0] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m_run[RT] = {-INFINITY}, l_run[RT] = {0.f};

    const int lim_full = min(kend, lim0 + inc * row0);     // (see attn_task)
    auto compute = [&](int stage, int c) {
        bf16x8 kf[2][KS], vf[DT];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[kt][ks] = kst[stage][(kt * KS + ks) * 64 + (lane & 48) + (col ^ ((4 * ks + g) & 15))];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) vf[dt] = vst[stage][dt * 64 + (lane & 48) + (col ^ (4 * g))];
        chunk_update<DH>(kf, vf, qf, o, m_run, l_run, limit, c, kend, P.scale_log2e, __builtin_amdgcn_readfirstlane(c + 32 <= lim_full) != 0);
    };

    lstore(0, kr0, vr0);
    gload(2, kr0, vr0);
    lds_barrier();
    for (int i = 0; i < nch; i += 2) {
        if (active) compute(0, kbeg + 32 * i);
        lstore(1, kr1, vr1);                         // chunk i+1 (stage 1 was last read before the previous barrier)
        gload(i + 3, kr1, vr1);
        lds_barrier();
        if (active && i + 1 < nch) compute(1, kbeg + 32 * (i + 1));
        lstore(0, kr0, vr0);                         // chunk i+2
        gload(i + 4, kr0, vr0);
        lds_barrier();
    }
    if (active) store_partial_direct<DH>(P, h, row0, P.M, part, o, m_run, l_run);
}

// In-flight segment: row j of a branch against rows 0..j of the same branch (the causal part of the tree
// mask).  At most T keys per row, so it runs in plain fp32 on the vector ALUs from unrounded keys / values:
// the rows of one step see each other unrounded, while the cache keeps bf16.  One wavefront per (row, head);
// lanes own DH/64 dims; dot products are wavefront-shuffle reductions.  q and the keys are rotated on the
// fly from the fp32 QKV output, and the wavefront of row r appends that row's rotated key and its value to
// the private cache.
template <int DH, bool TREE>
__device__ void inflight_task_fused(const AttnParams &P, int h, int r, int r2) {
    // r2: a second, later row of the same branch handled by this wavefront (-1: none).  Its keys are a
    // superset of row r's, so every key is loaded and rotated once and scored against both rows: a branch of up
    // to eight rows is one pass of the workgroup's four wavefronts, not two.
    constexpr int PER = DH / 64, HALF = DH / 2;
    const int lane = threadIdx.x & 63;
    if (r >= P.M) return;
    const bool two = r2 >= 0 && r2 < P.M;              // (uniform)
    const int b = r / P.T;
    const int jr[2] = {r - b * P.T, two ? r2 - b * P.T : r - b * P.T};
    const int jmax = jr[1];
    const int HD = P.H * DH;
    const int sb = slot_of(P, b);
    if (P.slot != nullptr && P.slot[b] != sb && lane == 0 && h == 0) atomicOr(P.status, 2);   // slot out of range
    int pl = P.private_len[sb];
    bool store_kv = true;
    if (pl < 0 || pl > P.max_private) {              // capacity overflow: drop the append, flag it
        if (lane == 0 && h == 0) atomicOr(P.status, 1);
        pl = min(max(pl, 0), P.max_private);
        store_kv = false;
    }
    // lane's dims d = lane*PER + i; the rotation partner of d is d ^ HALF, the angle index d % HALF
    int dl[PER];
    bool upper[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int d = lane * PER + i;
        dl[i] = d & (HALF - 1);
        upper[i] = d >= HALF;
    }
    auto rotated = [&](const float *vec, const float *tb, int i) {
        const int d = lane * PER + i;
        const float x = vec[d], y = vec[d ^ HALF], c = tb[2 * dl[i]], s_ = tb[2 * dl[i] + 1];
        return upper[i] ? x * c + y * s_ : x * c - y * s_;
    };
    const float *tb0 = P.rope + (size_t)(P.S + pl) * DH;
    // candidate trees (Section 2.2 "Tree Attention"; appendix): row j sees, among the rows of its branch, only
    // itself and its ancestors, and every row sits at the position of its depth
    unsigned long long anc[2];
    auto depth_of = [&](int jj) { return TREE ? P.row_depth[jj] : jj; };
    float qv[2][PER], o[2][PER], m[2], l[2];
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        anc[w] = TREE ? P.row_anc[jr[w]] : ~0ull;
        const int rw = b * P.T + jr[w];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            qv[w][i] = rotated(P.qkv + (size_t)rw * 3 * HD + h * DH, tb0 + (size_t)depth_of(jr[w]) * DH, i);
            o[w][i] = 0.f;
        }
        m[w] = -INFINITY;
        l[w] = 0.f;
    }
    constexpr int kB = 8;
    for (int j0 = 0; j0 <= jmax; j0 += kB) {            // kB keys per pass: their loads overlap
        float kk[kB][PER], vv[kB][PER], sc[2][kB];
#pragma unroll
        for (int u = 0; u < kB; ++u) {
            const int jj = min(j0 + u, jmax);
            const float *krow = P.qkv + (size_t)(b * P.T + jj) * 3 * HD + HD + h * DH;
            sc[0][u] = sc[1][u] = 0.f;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                kk[u][i] = rotated(krow, tb0 + (size_t)depth_of(jj) * DH, i);
                vv[u][i] = krow[HD + lane * PER + i];
                sc[0][u] = fmaf(qv[0][i], kk[u][i], sc[0][u]);
                sc[1][u] = fmaf(qv[1][i], kk[u][i], sc[1][u]);
            }
        }
#pragma unroll
        for (int u = 0; u < kB; ++u) {
            const int jj = j0 + u;
            if (jj > jmax) continue;                                               // (uniform over the wavefront)
#pragma unroll
            for (int w = 0; w < 2; ++w) {
                if (w == 1 && !two) continue;
                if (jj > jr[w] || (TREE && !((anc[w] >> (jj & 63)) & 1ull))) continue;
                const float s = wave_reduce_sum_dpp(sc[w][u]) * P.scale_log2e;   // (DPP: the keys of a row are a dependent chain)
                const float m_new = fmaxf(m[w], s);
                const float alpha = exp2f(m[w] - m_new), p = exp2f(s - m_new);
                l[w] = l[w] * alpha + p;
#pragma unroll
                for (int i = 0; i < PER; ++i) o[w][i] = o[w][i] * alpha + p * vv[u][i];
                m[w] = m_new;
            }
            if ((jj == jr[0] || (two && jj == jr[1])) && store_kv) {   // a row's own key / value: append to the cache
                const size_t head = (size_t)sb * P.H + h;
                const int idx = pl + jj;
#pragma unroll
                for (int i = 0; i < PER; ++i) {
                    const int d = lane * PER + i;
                    P.k_priv_w[(head * P.cap_p + idx) * DH + d] = f2bf(kk[u][i]);
                    P.vt_priv_w[head * DH * P.cap_p + vt_offset(d, idx, DH)] = f2bf(vv[u][i]);
                }
            }
        }
    }
    const int part = P.ks_shared + P.ks_priv;
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        if (w == 1 && !two) continue;
        const int rw = b * P.T + jr[w];
        float *op = P.o_part + (((size_t)part * P.Mq + rw) * P.H + h) * DH + lane * PER;
        if (PER == 2) {
            store2_agent(op, o[w][0], o[w][PER - 1]);
        } else {
#pragma unroll
            for (int i = 0; i < PER; ++i) store_agent(op + i, o[w][i]);
        }
        if (lane == 0) store2_agent(P.ml_part + (((size_t)part * P.Mq + rw) * P.H + h) * 2, m[w], l[w]);
    }
}

// The in-flight segment of ALL rows (at most eight) of branch b, head h in ONE wavefront (branch tasks that give a
// wavefront a whole head).  Row after row on the whole wavefront would be a chain of 21 dependent 64-lane
// reductions for six rows (measured 9.4 us); here the rotated q and k rows go through this wavefront's corner of
// LDS (rows padded by four floats: eight rows on distinct banks), lane (r, u) forms the one score q_r . k_u, a
// row's softmax is three xor-shuffles inside its eight lanes, and lanes go back to owning dims for P . V with the
// weights read lane by lane.  Also appends the rows' rotated keys and their values to the private cache.
template <int DH, bool TREE>
__device__ void inflight_solo(const AttnParams &P, int h, int b, float *lds) {
    constexpr int PER = DH / 64, HALF = DH / 2, R = 8, LD = DH + 4;
    const int lane = threadIdx.x & 63;
    const int n = P.T;                                   // 1 .. R rows
    const int HD = P.H * DH;
    const int sb = slot_of(P, b);
    if (P.slot != nullptr && P.slot[b] != sb && lane == 0 && h == 0) atomicOr(P.status, 2);   // slot out of range
    int pl = P.private_len[sb];
    bool store_kv = true;
    if (pl < 0 || pl > P.max_private) {              // capacity overflow: drop the append, flag it
        if (lane == 0 && h == 0) atomicOr(P.status, 1);
        pl = min(max(pl, 0), P.max_private);
        store_kv = false;
    }
    const int r = lane >> 3, u = lane & 7;              // this lane's (row, key) pair
    const unsigned long long anc = TREE ? P.row_anc[min(r, n - 1)] : ~0ull;
    int dl[PER];
    bool upper[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int d = lane * PER + i;
        dl[i] = d & (HALF - 1);
        upper[i] = d >= HALF;
    }
    auto rotated = [&](const float *vec, const float *tb, int i) {
        const int d = lane * PER + i;
        const float x = vec[d], y = vec[d ^ HALF], c = tb[2 * dl[i]], s_ = tb[2 * dl[i] + 1];
        return upper[i] ? x * c + y * s_ : x * c - y * s_;
    };
    const float *tb0 = P.rope + (size_t)(P.S + pl) * DH;
    float kr[R][PER], vv[R][PER];
    float *Qs = lds, *Ks = lds + R * LD;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int jj = min(j, n - 1);                    // (rows past the last repeat it; masked below)
        const float *row = P.qkv + (size_t)(b * P.T + jj) * 3 * HD + h * DH;
        const float *tb = tb0 + (size_t)(TREE ? P.row_depth[jj] : jj) * DH;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            Qs[j * LD + lane * PER + i] = rotated(row, tb, i);
            kr[j][i] = rotated(row + HD, tb, i);
            vv[j][i] = row[2 * HD + lane * PER + i];
            Ks[j * LD + lane * PER + i] = kr[j][i];
        }
    }
    // (LDS operations of one wavefront execute in program order: the reads below see the rows)
    float sc = 0.f;
#pragma unroll
    for (int d4 = 0; d4 < DH / 4; ++d4) {
        const f32x4 qa = *reinterpret_cast<const f32x4 *>(Qs + r * LD + 4 * d4);
        const f32x4 kb = *reinterpret_cast<const f32x4 *>(Ks + u * LD + 4 * d4);
        sc = fmaf(qa[0], kb[0], sc);
        sc = fmaf(qa[1], kb[1], sc);
        sc = fmaf(qa[2], kb[2], sc);
        sc = fmaf(qa[3], kb[3], sc);
    }
    // row r sees rows 0 .. r of its branch (candidate trees: itself and its ancestors)
    const bool vis = r < n && u <= r && ((anc >> u) & 1ull);
    const float s = vis ? sc * P.scale_log2e : -INFINITY;
    float m = s;
    m = fmaxf(m, __shfl_xor(m, 1));
    m = fmaxf(m, __shfl_xor(m, 2));
    m = fmaxf(m, __shfl_xor(m, 4));
    const float p = __builtin_amdgcn_exp2f(s - (m == -INFINITY ? 0.f : m));      // 0 where masked
    float l = p;
    l += __shfl_xor(l, 1);
    l += __shfl_xor(l, 2);
    l += __shfl_xor(l, 4);
    const int pbits = __builtin_bit_cast(int, p), mbits = __builtin_bit_cast(int, m), lbits = __builtin_bit_cast(int, l);
    const int part = P.ks_shared + P.ks_priv;
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        if (rr >= n) break;                              // (uniform)
        float o[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) o[i] = 0.f;
#pragma unroll
        for (int uu = 0; uu <= rr; ++uu) {
            const float w = __builtin_bit_cast(float, __builtin_amdgcn_readlane(pbits, rr * 8 + uu));
#pragma unroll
            for (int i = 0; i < PER; ++i) o[i] = fmaf(w, vv[uu][i], o[i]);
        }
        const int rw = b * P.T + rr;
        float *op = P.o_part + (((size_t)part * P.Mq + rw) * P.H + h) * DH + lane * PER;
        if (PER == 2) {
            store2_agent(op, o[0], o[PER - 1]);
        } else {
#pragma unroll
            for (int i = 0; i < PER; ++i) store_agent(op + i, o[i]);
        }
        const float mr = __builtin_bit_cast(float, __builtin_amdgcn_readlane(mbits, rr * 8));
        const float lr = __builtin_bit_cast(float, __builtin_amdgcn_readlane(lbits, rr * 8));
        if (lane == 0) store2_agent(P.ml_part + (((size_t)part * P.Mq + rw) * P.H + h) * 2, mr, lr);
        if (store_kv) {                                  // the row's own key / value: append to the cache
            const size_t head = (size_t)sb * P.H + h;
            const int idx = pl + rr;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int d = lane * PER + i;
                P.k_priv_w[(head * P.cap_p + idx) * DH + d] = f2bf(kr[rr][i]);
                P.vt_priv_w[head * DH * P.cap_p + vt_offset(d, idx, DH)] = f2bf(vv[rr][i]);
            }
        }
    }
}

// Combine the np partials of head h for the RB rows r0, r0 + rstep, ... by log-sum-exp and write the hi/lo bf16
// activation (fragment-packed, K = H*DH) that feeds the O projection; rows >= M of the tile are zero.  One
// wavefront; the loads of all RB rows and of up to eight partials are issued before the first is used (a
// load that crosses workgroups costs a trip to memory).
// ACROSS: the partials were written by other workgroups of the same launch (agent-scope loads).
template <int DH, bool ACROSS, int RB>
__device__ __forceinline__ void merge_rows(const float *o_part, const float *ml_part, uint16_t *act, int r0, int rstep,
                                           int h, int M, int Mp, int Mq, int H, int np) {
    const int lane = threadIdx.x & 63;
    const int KT = (H * DH) >> 5;
    constexpr int PER = DH / 64;     // output dims per lane
    constexpr int NPB = 6;                               // partials per pass (register budget of the fused kernel)
    auto ld = [](const float *p) { return ACROSS ? load_agent(p) : *p; };
    auto ld2 = [](const float *p, float &x, float &y) {      // two adjacent floats, 8-byte aligned
        if (ACROSS) {
            load2_agent(p, x, y);
        } else {
            const float2 w = *reinterpret_cast<const float2 *>(p);
            x = w.x;
            y = w.y;
        }
    };
    float mrun[RB], Lrun[RB], acc[RB][PER];
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        mrun[i] = -INFINITY;
        Lrun[i] = 0.f;
#pragma unroll
        for (int e = 0; e < PER; ++e) acc[i][e] = 0.f;
    }
    for (int p0 = 0; p0 < np; p0 += NPB) {
        float m[RB][NPB], l[RB][NPB], v[RB][NPB][PER];
#pragma unroll
        for (int k = 0; k < NPB; ++k) {
            if (p0 + k >= np) break;                      // (uniform)
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int r = min(r0 + i * rstep, M - 1);
                const size_t base = ((size_t)(p0 + k) * Mq + r) * H + h;
                ld2(ml_part + base * 2, m[i][k], l[i][k]);
                if (PER == 2) {
                    ld2(o_part + base * DH + lane * 2, v[i][k][0], v[i][k][PER - 1]);
                } else {
#pragma unroll
                    for (int e = 0; e < PER; ++e) v[i][k][e] = ld(o_part + base * DH + lane * PER + e);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            float mx = mrun[i];
#pragma unroll
            for (int k = 0; k < NPB; ++k)
                if (p0 + k < np && l[i][k] != 0.f) mx = fmaxf(mx, m[i][k]);
            const float sc = (mrun[i] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mrun[i] - mx);
            Lrun[i] *= sc;
#pragma unroll
            for (int e = 0; e < PER; ++e) acc[i][e] *= sc;
#pragma unroll
            for (int k = 0; k < NPB; ++k) {
                if (p0 + k >= np || l[i][k] == 0.f) continue;     // past the end / empty key range
                const float wgt = __builtin_amdgcn_exp2f(m[i][k] - mx);
                Lrun[i] += l[i][k] * wgt;
#pragma unroll
                for (int e = 0; e < PER; ++e) acc[i][e] += v[i][k][e] * wgt;
            }
            mrun[i] = mx;
        }
    }
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        const int r = r0 + i * rstep;
        if (r >= Mp) continue;
        const float inv = (r < M && Lrun[i] > 0.f) ? 1.0f / Lrun[i] : 0.f;
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const size_t o = packed_offset(r, h * DH + lane * PER + e, KT);
            split_bf16(acc[i][e] * inv, act[o], act[o + kActLoOffset]);
        }
    }
}

template <int DH, bool FUSED, bool TREE>
__global__ __launch_bounds__(256, 2) void attn_partial_kernel(AttnParams P) {
    constexpr int RT = kRowTiles;
    // workgroup tasks: first the shared segment, then one per (branch, head, row group, private key range)
    // all kernel arguments in one batch of scalar loads (each separate one is a round trip to memory)
    asm volatile("" ::"s"(P.q), "s"(P.q_plane), "s"(P.k_shared), "s"(P.vt_shared), "s"(P.k_priv), "s"(P.vt_priv),
                 "s"(P.private_len), "s"(P.slot), "s"(P.n_slots), "s"(P.o_part), "s"(P.ml_part), "s"(P.qkv),
                 "s"(P.rope), "s"(P.counters), "s"(P.act), "s"(P.status), "s"(P.row_depth), "s"(P.row_anc));
    asm volatile("" ::"s"(P.Mp), "s"(P.merge_in_launch), "s"(P.wave_tasks), "s"(P.gpw), "s"(P.n_quads), "s"(P.M), "s"(P.Mq), "s"(P.N),
                 "s"(P.T), "s"(P.H), "s"(P.S), "s"(P.prefill_shared), "s"(P.cap_s), "s"(P.cap_p), "s"(P.max_private),
                 "s"(P.n_groups), "s"(P.ks_shared), "s"(P.keys_per_range), "s"(P.keys_per_range_priv), "s"(P.ks_priv), "s"(P.groups_priv),
                 "s"(P.scale_log2e));
    // LDS: merge buffers of attn_task or the two K/V stages of attn_task_lds
    constexpr int kMergeBytes = 2 * 4 * 16 * RT * 4 + 4 * 16 * RT * (DH + 4) * 4;
    constexpr int kStageBytes = 2 * (2 * (DH / 32) + DH / 16) * 64 * 16;
    __shared__ __attribute__((aligned(16))) char smem[kMergeBytes > kStageBytes ? kMergeBytes : kStageBytes];
    const int task = (int)blockIdx.x - P.n_solo;          // (n_solo = 0 unless the branch tasks go first)
    const int wv = threadIdx.x >> 6;
    // steps with several row groups and short private contexts: a branch task is one WAVEFRONT -- the private
    // keys of (branch, head) walked chunk by chunk, then all in-flight rows of that head -- and a workgroup holds
    // four heads.  These workgroups come first in launch order and the shared pass gets the remaining slots of
    // the chip, so that every task of the launch is resident from the start: the launch is bound by the sum of
    // workgroup latencies over the slots (two workgroups per CU), not by throughput.
    if (FUSED && P.solo_branch && blockIdx.x < P.n_solo) {
        const int nr = max(P.ks_priv, 1);
        const int hq_n = (P.H + 3) >> 2;
        const int ks = (int)blockIdx.x % nr;
        const int hq = ((int)blockIdx.x / nr) % hq_n;
        const int b = (int)blockIdx.x / (nr * hq_n);
        const int h = hq * 4 + wv;
        if (h >= P.H) return;                              // (uniform over the wavefront; no barriers below)
        if (P.ks_priv > 0) {
            const int pl = clamped_private_len(P, b);
            const int kbeg = ks * P.keys_per_range_priv;
            const int kend = min(pl, kbeg + P.keys_per_range_priv);
            const size_t sb = (size_t)slot_of(P, b);
            attn_task<DH, FUSED, TREE, true>(P, h, b * P.T, (b + 1) * P.T, P.k_priv + (sb * P.H + h) * P.cap_p * DH,
                                             P.vt_priv + (sb * P.H + h) * DH * P.cap_p, P.cap_p, kbeg, max(kbeg, kend),
                                             pl, b * P.T, 0, P.ks_shared + ks, smem);
        }
        if (ks == 0) inflight_solo<DH, TREE>(P, h, b, reinterpret_cast<float *>(smem) + wv * (2 * 8 * (DH + 4)));
        return;                                            // (the merge is a launch of its own in this mode)
    }
    // shared segment: (head, row group, key range) tasks, or, when the step has several row groups,
    // (head, key range, up to four row groups) tasks that share the key range through LDS
    const int n_shared = P.wave_tasks ? P.H * P.ks_shared * P.n_quads : P.H * P.n_groups * P.ks_shared;
    int h;
    if (task < n_shared && P.wave_tasks) {
        // consecutive workgroup ids go round the 8 XCDs: the workgroups of one (head, key range) take ids
        // 8 apart, so they run on one XCD at about the same time and the second reads the keys from its L2
        int unit, quad;
        const int paired = P.pair_xcd ? (P.H * P.ks_shared / 8) * 8 * P.n_quads : 0;
        if (task < paired) {
            const int rem = task % (8 * P.n_quads);
            quad = rem >> 3;
            unit = (task / (8 * P.n_quads)) * 8 + (rem & 7);
        } else {
            quad = (task - paired) % P.n_quads;
            unit = paired / P.n_quads + (task - paired) / P.n_quads;
        }
        const int ks = unit % P.ks_shared;
        h = unit / P.ks_shared;
        const int total = P.prefill_shared ? P.S + P.M : P.S;
        const int kbeg = ks * P.keys_per_range;
        const int kend = min(total, kbeg + P.keys_per_range);
        const int grp0 = quad * P.gpw;
        attn_task_lds<DH, FUSED, TREE>(P, h, grp0, min(P.gpw, P.n_groups - grp0), P.k_shared + (size_t)h * P.cap_s * DH,
                                 P.vt_shared + (size_t)h * DH * P.cap_s, kbeg, max(kbeg, kend),
                                 P.prefill_shared ? P.S + 1 : P.S, P.prefill_shared ? 1 : 0, ks, smem);
        return;                                           // (the merge is a launch of its own in this mode)
    }
    if (task < n_shared) {
        const int ks = task % P.ks_shared;
        const int grp = (task / P.ks_shared) % P.n_groups;
        h = task / (P.ks_shared * P.n_groups);
        const int total = P.prefill_shared ? P.S + P.M : P.S;
        const int kbeg = ks * P.keys_per_range;
        const int kend = min(total, kbeg + P.keys_per_range);
        // verify: every row sees all S shared keys; prefill: row j sees keys < S + j + 1
        attn_task<DH, FUSED, TREE>(P, h, grp * 16 * RT, P.M, P.k_shared + (size_t)h * P.cap_s * DH,
                             P.vt_shared + (size_t)h * DH * P.cap_s, P.cap_s, kbeg, max(kbeg, kend),
                             P.prefill_shared ? P.S + 1 : P.S, 0, P.prefill_shared ? 1 : 0, ks, smem);
    } else {
        // branch task (verify / decode only): one key range of the branch's private context for one group of
        // its rows; the task of range 0 also runs the in-flight segment of those rows, a wavefront per row
        const int ptask = task - n_shared;
        const int nr = max(P.ks_priv, 1);
        const int ks = ptask % nr;
        const int grp = (ptask / nr) % P.groups_priv;
        h = (ptask / (nr * P.groups_priv)) % P.H;
        const int b = ptask / (nr * P.groups_priv * P.H);
        const int row_first = b * P.T + grp * 16 * RT, row_end = min((b + 1) * P.T, row_first + 16 * RT);
        if (P.ks_priv > 0) {
            const int pl = clamped_private_len(P, b);   // committed private context
            const int kbeg = ks * P.keys_per_range_priv;
            const int kend = min(pl, kbeg + P.keys_per_range_priv);
            // every row of the branch sees all pl committed private keys
            const size_t sb = (size_t)slot_of(P, b);
            attn_task<DH, FUSED, TREE>(P, h, row_first, row_end, P.k_priv + (sb * P.H + h) * P.cap_p * DH,
                                 P.vt_priv + (sb * P.H + h) * DH * P.cap_p, P.cap_p, kbeg, max(kbeg, kend),
                                 pl, b * P.T, 0, P.ks_shared + ks, smem);
        }
        if (FUSED && ks == 0)
            for (int r = row_first + wv; r < row_end; r += 8)
                inflight_task_fused<DH, TREE>(P, h, r, r + 4 < row_end ? r + 4 : -1);
    }
    if (FUSED && P.merge_in_launch) {
        // every task of head h has left its partial: the workgroup that arrives last merges the head's rows
        __shared__ int s_last;
        const int expected = P.n_groups * P.ks_shared + P.N * P.groups_priv * max(P.ks_priv, 1);
        if (!arrive_last(P.counters + h, expected, &s_last)) return;
        const int np = P.ks_shared + P.ks_priv + 1;
        for (int r = threadIdx.x >> 6; r < P.Mp; r += 16)     // rows r, r+4, r+8, r+12 per pass
            merge_rows<DH, true, 4>(P.o_part, P.ml_part, P.act, r, 4, h, P.M, P.Mp, P.Mq, P.H, np);
    }
}

// Merge as a launch of its own (shared-prefix prefill).  One wavefront per (row, head).
template <int DH>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float *o_part, const float *ml_part, uint16_t *act,
                                                         int M, int Mq, int Mp, int H, int np) {
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= Mp * H) return;
    merge_rows<DH, false, 1>(o_part, ml_part, act, w / H, 1, w % H, M, Mp, Mq, H, np);
}

}  // namespace

// Key ranges of the shared and the private segment for a step of M rows.
// One row group (M <= 16): workgroup tasks whose four wavefronts interleave 32-key chunks: ranges of whole
// 128-key rounds, about 512 workgroups.  Several row groups: workgroups that walk a range for up to four row
// groups (attn_task_lds): ranges of an even number of 32-key chunks (chunks are processed in pairs), about 450
// workgroups, fewer when the branch tasks are many.  Private ranges are always of the first kind.
void attn_bf16_plan(int M, int H, int N, int total_shared_keys, int cap_priv_keys, int prefill_shared,
                    int *ks_shared, int *keys_per_range, int *ks_priv, int *keys_per_range_priv) {
    const int n_groups = (M + 15) / 16;
    const bool lds_tasks = n_groups > 1;
    if (prefill_shared || cap_priv_keys <= 0) {
        *ks_priv = 0;
        *keys_per_range_priv = 128;
    } else {
        const int rounds = (cap_priv_keys + 127) / 128;
        // about one branch workgroup per CU: with 8 branches x 32 heads of up to 1024 private keys, one range
        // each (256 workgroups) was measured faster than two (512) and much faster than four or eight (every
        // range adds a partial to write, read back and merge)
        int kp = 256 / (N * H > 0 ? N * H : 1);
        if (kp < 1) kp = 1;
        if (kp > rounds) kp = rounds;
        if (kp > 32) kp = 32;
        const int per_rounds = (rounds + kp - 1) / kp;
        *ks_priv = (rounds + per_rounds - 1) / per_rounds;
        *keys_per_range_priv = per_rounds * 128;
    }
    const int unit = lds_tasks ? 64 : 128;
    int units = (total_shared_keys + unit - 1) / unit;
    if (units < 1) units = 1;
    const int base_tasks = lds_tasks ? H * ((n_groups + 3) / 4) : H;
    // workgroups of the shared pass.  Two fit on a CU (512 at once) and every one pays ~3.5 us of prologue and
    // partial store, so when the branch tasks alone fill the chip the shared pass gets fewer, longer ranges
    // (16 branches x 32 heads: 192 against 448 workgroups, -2 us; flat with 8 x 40)
    const int T = M / (N > 0 ? N : 1);
    const bool solo = lds_tasks && !prefill_shared && T <= 8 && *keys_per_range_priv <= 256;   // (as in the launcher)
    const int branch_tasks = prefill_shared ? 0 : (solo ? N * ((H + 3) / 4) : N * H * ((T + 15) / 16)) * (*ks_priv > 0 ? *ks_priv : 1);
    // (branch tasks of one wavefront per head go first and the shared pass takes the slots they leave, so that
    // the whole launch is resident at once)
    const int left = 512 - branch_tasks > 192 ? 512 - branch_tasks : 192;
    const int target = !lds_tasks ? 512 : solo ? left : branch_tasks >= 256 ? 192 : 448;
    const int want = solo ? (target / base_tasks > 0 ? target / base_tasks : 1) : (target + base_tasks - 1) / base_tasks;
    int ks = want < units ? want : units;
    if (lds_tasks && ks < (units + 15) / 16) ks = (units + 15) / 16;    // at most 32 chunks per workgroup
    if (ks < 1) ks = 1;
    if (ks > 32) ks = 32;
    const int per_units = (units + ks - 1) / ks;
    *ks_shared = (units + per_units - 1) / per_units;
    *keys_per_range = per_units * unit;
}

int launch_attn_bf16(const AttnBf16Args &a, hipStream_t st) {
    AttnParams P{};
    P.q = (const uint16_t *)a.q;
    P.q_plane = a.q_plane;
    P.k_shared = (const uint16_t *)a.k_shared;
    P.vt_shared = (const uint16_t *)a.vt_shared;
    P.k_priv = (const uint16_t *)a.k_priv;
    P.vt_priv = (const uint16_t *)a.vt_priv;
    P.k_priv_w = (uint16_t *)a.k_priv;
    P.vt_priv_w = (uint16_t *)a.vt_priv;
    P.private_len = a.private_len;
    P.slot = a.branch_slot;
    P.n_slots = a.n_slots;
    P.o_part = a.o_part;
    P.ml_part = a.ml_part;
    P.qkv = a.qkv;
    P.rope = a.rope;
    P.counters = a.counters;
    P.act = (uint16_t *)a.act;
    P.status = a.status;
    P.row_depth = a.row_depth;
    P.row_anc = a.row_anc;
    P.M = a.M; P.Mp = a.Mp; P.Mq = a.Mq; P.N = a.N; P.T = a.T; P.H = a.H; P.S = a.S;
    P.prefill_shared = a.prefill_shared;
    P.cap_s = a.cap_s; P.cap_p = a.cap_p; P.max_private = a.max_private;
    constexpr int rt = kRowTiles;
    P.n_groups = (a.M + 16 * rt - 1) / (16 * rt);
    P.wave_tasks = P.n_groups > 1;
    P.n_quads = (P.n_groups + 3) / 4;
    P.gpw = (P.n_groups + P.n_quads - 1) / P.n_quads;
    P.keys_per_range_priv = a.keys_per_range_priv;
    P.ks_shared = a.ks_shared;
    P.keys_per_range = a.keys_per_range;
    P.ks_priv = a.ks_priv;
    P.groups_priv = (a.T + 16 * rt - 1) / (16 * rt);
    P.scale_log2e = 1.4426950408889634f / sqrtf((float)a.dh);
    const bool fused = !a.prefill_shared;
    P.solo_branch = fused && P.wave_tasks && a.T <= 8 && a.keys_per_range_priv <= 256;
    const int branch_units = P.solo_branch ? a.N * ((a.H + 3) / 4) : a.N * a.H * P.groups_priv;
    const int n_branch = fused ? branch_units * (a.ks_priv > 0 ? a.ks_priv : 1) : 0;
    P.n_solo = P.solo_branch ? n_branch : 0;
    const int blocks = (P.wave_tasks ? a.H * a.ks_shared * P.n_quads : a.H * P.n_groups * a.ks_shared) + n_branch;
    if (a.dh != 128 && a.dh != 64) {
        set_error("bf16 attention supports head_dim 64 or 128, got %d", a.dh);
        return SEED_E_SHAPE;
    }
    // up to 16 rows the last workgroup of a head merges them in one pass; more rows would queue up behind its
    // four wavefronts, so they get a merge launch with a wavefront per (row, head)
    P.merge_in_launch = fused && !P.wave_tasks;
    P.pair_xcd = P.n_quads > 1;
    const int np = fused ? a.ks_shared + a.ks_priv + 1 : a.ks_shared;   // prefill: shared partials only
    const bool tree = fused && a.row_depth != nullptr && a.row_anc != nullptr;
#define SEEDV_ATTN(DHv, FUSEDv, TREEv) \
    hipLaunchKernelGGL((attn_partial_kernel<DHv, FUSEDv, TREEv>), dim3(blocks), dim3(256), 0, st, P)
    if (a.dh == 128) {
        if (tree) SEEDV_ATTN(128, true, true); else if (fused) SEEDV_ATTN(128, true, false); else SEEDV_ATTN(128, false, false);
        if (!P.merge_in_launch)
            hipLaunchKernelGGL(attn_merge_kernel<128>, dim3((a.Mp * a.H + 3) / 4), dim3(256), 0, st, a.o_part,
                               a.ml_part, (uint16_t *)a.act, a.M, a.Mq, a.Mp, a.H, np);
    } else {
        if (tree) SEEDV_ATTN(64, true, true); else if (fused) SEEDV_ATTN(64, true, false); else SEEDV_ATTN(64, false, false);
        if (!P.merge_in_launch)
            hipLaunchKernelGGL(attn_merge_kernel<64>, dim3((a.Mp * a.H + 3) / 4), dim3(256), 0, st, a.o_part,
                               a.ml_part, (uint16_t *)a.act, a.M, a.Mq, a.Mp, a.H, np);
    }
#undef SEEDV_ATTN
    return hip_fail(hipGetLastError(), "attention launch");
}

}  // namespace seedv
