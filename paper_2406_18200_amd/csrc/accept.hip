// Fused accept / reject / resample and the draft-side softmax + draw.
//
// Rule (paper Section 3.1; Algorithm 1, inner loop of the verification process): draft token x_j is
// accepted with probability min(1, p_t(x_j)/p_d(x_j)), checked left to right; the first rejection ends
// the check and one replacement token is returned by the target model.  The replacement is drawn from
// norm(max(0, p_t - p_d)), the distribution that keeps the output law equal to the target's.
//
// One workgroup (16 wavefronts) per branch.  Softmax statistics are wavefront-shuffle reductions; the
// draw is an integer fixed-point inverse CDF: weights are truncated to multiples of 2^-38 and summed
// as 64-bit integers, so the parallel scan gives the same token as a serial one.
#include <mutex>
#include "seed_internal.h"

namespace seedv {
namespace {

constexpr int kBlock = 1024;
constexpr int kWaves = kBlock / 64;
constexpr int kMaxSlices = 16;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

struct Shared {
    float red[kWaves];
    unsigned long long tot[kWaves];
    int idx[kWaves];
    int tok;
};

__device__ float block_max(float v, Shared &sm) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm.red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sm.red[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) r = fmaxf(r, sm.red[i]);
    return r;
}
__device__ float block_sum(float v, Shared &sm) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm.red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sm.red[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) r += sm.red[i];   // fixed order: deterministic
    return r;
}

// argmax with the lowest index on ties
__device__ int block_argmax(const float *row, int V, Shared &sm) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int v = threadIdx.x; v < V; v += kBlock) {
        float x = row[v];
        if (x > bv) { bv = x; bi = v; }               // strided ascending: first max kept
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        float ov = __shfl_xor(bv, off);
        int oi = __shfl_xor(bi, off);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sm.red[threadIdx.x >> 6] = bv; sm.idx[threadIdx.x >> 6] = bi; }
    __syncthreads();
    float rv = sm.red[0];
    int ri = sm.idx[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) {
        float ov = sm.red[i];
        int oi = sm.idx[i];
        if (ov > rv || (ov == rv && oi < ri)) { rv = ov; ri = oi; }
    }
    return ri;
}

// exp((x - mx) / temperature) with the hardware exp2: a few instructions instead of ~70 for the IEEE
// division + libm exp (the kernel runs on as few CUs as there are branches, so it is ALU-bound); relative
// error ~1e-6, far inside the tolerance of the LOGITS mode.  Every use of p goes through the same function,
// so the accept test and the residual draw see the same bits.
__device__ __forceinline__ float exp_scaled(float x, float mx, float inv_temp) {
    return __builtin_amdgcn_exp2f((x - mx) * inv_temp * 1.4426950408889634f);
}

// A row of target probabilities, either given or defined by softmax(logits / temperature).
struct TargetRow {
    const float *src;
    int is_logits;
    float mx, inv_sum, inv_temp;
    __device__ __forceinline__ float p(int v) const {
        if (!is_logits) return src[v];
        return exp_scaled(src[v], mx, inv_temp) * inv_sum;
    }
};

__device__ TargetRow make_row(const float *src, int is_logits, float temp, int V, Shared &sm) {
    TargetRow r{src, is_logits, 0.f, 1.f, 1.f / temp};
    if (!is_logits) return r;
    float m = -INFINITY;
#pragma unroll 8
    for (int v = threadIdx.x; v < V; v += kBlock) m = fmaxf(m, src[v]);
    r.mx = block_max(m, sm);
    float s = 0.f;
#pragma unroll 8
    for (int v = threadIdx.x; v < V; v += kBlock) s += exp_scaled(src[v], r.mx, r.inv_temp);
    r.inv_sum = 1.0f / block_sum(s, sm);
    return r;
}

__device__ __forceinline__ unsigned long long to_fixed(float w) {
    // w in [0, 1]: scaling by 2^38 is exact, the conversion truncates
    return (unsigned long long)(__fmul_rn(w, 274877906944.0f));
}

// weight of token v: residual max(0, p - q) (one float32 subtraction) or p itself
template <int RESIDUAL>
__device__ __forceinline__ unsigned long long weight_of(float p, const float *q, int v) {
    if (RESIDUAL) {
        float r = __fsub_rn(p, q[v]);
        return r > 0.f ? to_fixed(r) : 0ull;
    }
    return to_fixed(p);
}
template <int RESIDUAL>
__device__ __forceinline__ unsigned long long weight_fixed(const TargetRow &row, const float *q, int v) {
    float p = row.p(v);
    if (RESIDUAL) {
        float r = __fsub_rn(p, q[v]);
        return r > 0.f ? to_fixed(r) : 0ull;
    }
    return to_fixed(p);
}

// Fixed-point inverse CDF over [0, V): token = min{v : sum_{w<=v} k_w > (m * Z) >> 24}, u = m 2^-24.
// Returns -1 if every weight truncates to zero.  Uniform control flow: every thread of the block calls.
// The integer sums make the result independent of the order of summation, so the two phases are free to
// use different ones: totals per wavefront segment with coalesced strided loads, then the one wavefront whose
// segment holds the target walks it in blocks of 2048 tokens, 32 CONSECUTIVE tokens per lane (one batch of
// loads, one wavefront scan over the lane sums, a register walk in the lane that holds the target).
// store (optional): the row of probabilities is also written there, in the same pass that sums the weights.
template <int RESIDUAL>
__device__ int draw_fixed(const TargetRow &row, const float *q, float u, int V, Shared &sm, float *store = nullptr) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int per = (((V + kWaves - 1) / kWaves) + 63) & ~63;
    const int base = wave * per;
    const int end = min(V, base + per);
    unsigned long long local = 0;
    if (store != nullptr) {
#pragma unroll 16
        for (int v = base + lane; v < end; v += 64) {
            const float p = row.p(v);
            store[v] = p;
            local += weight_of<RESIDUAL>(p, q, v);
        }
    } else {
#pragma unroll 16
        for (int v = base + lane; v < end; v += 64) local += weight_fixed<RESIDUAL>(row, q, v);
    }
    local = wave_sum_u64(local);
    __syncthreads();
    if (lane == 0) sm.tot[wave] = local;
    if (threadIdx.x == 0) sm.tok = -1;
    __syncthreads();
    unsigned long long Z = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) Z += sm.tot[i];
    if (Z == 0) return -1;
    const unsigned long long m24 = (unsigned long long)(__fmul_rn(u, 16777216.0f));
    const unsigned long long t = (m24 * Z) >> 24;
    unsigned long long run = 0;
    int target = 0;
    for (int i = 0; i < kWaves; ++i) {
        unsigned long long nx = run + sm.tot[i];
        if (t < nx) { target = i; break; }
        run = nx;
    }
    if (wave == target) {
        constexpr int kPerLane = 32;
        for (int blk = base; blk < end; blk += 64 * kPerLane) {
            const int v0 = blk + lane * kPerLane;
            unsigned long long k[kPerLane];
            unsigned long long mine = 0;
#pragma unroll
            for (int e = 0; e < kPerLane; ++e) {
                const int v = v0 + e;
                k[e] = v < end ? weight_fixed<RESIDUAL>(row, q, min(v, end - 1)) : 0ull;
                mine += k[e];
            }
            unsigned long long incl = mine;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                unsigned long long o = __shfl_up(incl, off);
                if (lane >= off) incl += o;
            }
            const unsigned long long hit = __ballot(run + incl > t);
            if (hit) {
                const int src = __ffsll((long long)hit) - 1;          // first lane whose prefix passes t
                if (lane == src) {
                    unsigned long long c = run + incl - mine;
                    int tok = v0;
#pragma unroll
                    for (int e = 0; e < kPerLane; ++e) {
                        c += k[e];
                        if (c > t) { tok = v0 + e; break; }
                    }
                    sm.tok = tok;
                }
                break;
            }
            run += __shfl(incl, 63);
        }
    }
    __syncthreads();
    return sm.tok;
}

// Statistics of one slice of a row of logits, written by row_stats_kernel: the maximum, its lowest index, and
// the sum of exp((x - that maximum) / temperature) over the slice.
struct SliceStats {
    float mx;
    int idx;
    float sum;
    int pad;
};

// Softmax statistics of every target row, spread over the whole chip: grid (rows, slices), 256 threads.  The
// accept kernel has one workgroup per BRANCH (the accept chain is sequential within a branch), far too few
// to read N*T rows of V logits quickly; here each workgroup reads V / slices of them.
__global__ __launch_bounds__(256) void row_stats_kernel(const float *logits, int V, int per, float inv_temp,
                                                        SliceStats *stats) {
    __shared__ float s_m[4];
    __shared__ int s_i[4];
    __shared__ float s_s[4];
    const int row = blockIdx.x, sl = blockIdx.y;
    const float *src = logits + (size_t)row * V;
    const int base = sl * per, end = min(V, base + per);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float mv = -INFINITY;
    int mi = 0x7fffffff;
#pragma unroll 8
    for (int v = base + threadIdx.x; v < end; v += 256) {
        const float x = src[v];
        if (x > mv) { mv = x; mi = v; }                     // ascending per thread: first maximum kept
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(mv, off);
        const int oi = __shfl_xor(mi, off);
        if (ov > mv || (ov == mv && oi < mi)) { mv = ov; mi = oi; }
    }
    if (lane == 0) { s_m[wave] = mv; s_i[wave] = mi; }
    __syncthreads();
    mv = s_m[0];
    mi = s_i[0];
#pragma unroll
    for (int i = 1; i < 4; ++i) {
        const float ov = s_m[i];
        const int oi = s_i[i];
        if (ov > mv || (ov == mv && oi < mi)) { mv = ov; mi = oi; }
    }
    float sv = 0.f;
#pragma unroll 8
    for (int v = base + threadIdx.x; v < end; v += 256) sv += exp_scaled(src[v], mv, inv_temp);   // (L2 hits)
    sv = wave_sum(sv);
    if (lane == 0) s_s[wave] = sv;
    __syncthreads();
    if (threadIdx.x == 0) {
        SliceStats o;
        o.mx = mv;
        o.idx = mi;
        o.sum = ((s_s[0] + s_s[1]) + s_s[2]) + s_s[3];
        o.pad = 0;
        stats[(size_t)row * gridDim.y + sl] = o;
    }
}

// Per-row results of the parallel first phase
struct RowInfo {
    float mx[16], sum[16];
    int ok[16], best[16];
    float wm[kWaves];
    int wi[kWaves];
};

// One workgroup per branch.  Phase 1: the (up to 16) target rows of the branch are handled concurrently, each
// by a group of 16 / rows wavefronts: softmax statistics (or argmax in greedy mode), p(x) and the accept test.
// Phase 2: the whole workgroup draws the replacement / bonus token for the one row that needs it.
__global__ __launch_bounds__(kBlock) void accept_resample_kernel(seed_accept_args a, const SliceStats *stats,
                                                                int n_slices, const int32_t *slot, int n_slots,
                                                                int32_t *status) {
    __shared__ Shared sm;
    __shared__ RowInfo ri;
    const int b = blockIdx.x;
    const int G = a.gamma, Tp = a.n_target_rows, V = a.vocab;
    const int is_logits = a.probs_kind == SEED_KIND_LOGITS;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int acc = 0, new_tok = -1;
    bool rejected = false;
    int rej_row = -1;
    for (int r0 = 0; r0 < Tp; r0 += 16) {
        const int rows = min(16, Tp - r0);
        int wpr = 1;                                       // wavefronts per row: power of two <= 16 / rows
        while (wpr * 2 * rows <= kWaves) wpr *= 2;
        const int r = wave / wpr, sub = wave - r * wpr;    // this wavefront's row (if r < rows) and slice
        const bool has_row = r < rows;
        const float *src = a.p_or_logits + ((size_t)b * Tp + r0 + (has_row ? r : 0)) * V;
        // pass 1: maximum (and its lowest index) of the row
        float mv = -INFINITY;
        int mi = 0x7fffffff;
        float slice_sum = 0.f;
        if (stats != nullptr) {
            // the slices' statistics are there already: lane i takes slice i (one load per lane instead of a
            // chain of them); slices ascend, so the lowest lane holding the maximum has the lowest index
            if (has_row) {
                const SliceStats *st = stats + ((size_t)b * Tp + r0 + r) * n_slices;
                float lm = -INFINITY;
                int li = 0x7fffffff;
                if (lane < n_slices) {
                    const SliceStats e = st[lane];
                    lm = e.mx;
                    li = e.idx;
                    slice_sum = e.sum;
                }
                mv = lm;
                mi = li;
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    const float ov = __shfl_xor(mv, off);
                    const int oi = __shfl_xor(mi, off);
                    if (ov > mv || (ov == mv && oi < mi)) { mv = ov; mi = oi; }
                }
                // this lane's slice, rescaled to the row maximum (0 for lanes without a slice)
                slice_sum = lane < n_slices ? slice_sum * exp_scaled(lm, mv, a.greedy ? 1.0f : 1.0f / a.temperature) : 0.f;
            }
        } else if (has_row && (is_logits || a.greedy)) {
#pragma unroll 8
            for (int v = sub * 64 + lane; v < V; v += wpr * 64) {
                const float x = src[v];
                if (x > mv) { mv = x; mi = v; }
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const float ov = __shfl_xor(mv, off);
                const int oi = __shfl_xor(mi, off);
                if (ov > mv || (ov == mv && oi < mi)) { mv = ov; mi = oi; }
            }
        }
        if (lane == 0) { ri.wm[wave] = mv; ri.wi[wave] = mi; }
        __syncthreads();
        if (has_row) {
            mv = ri.wm[r * wpr];
            mi = ri.wi[r * wpr];
            for (int i = 1; i < wpr; ++i) {
                const float ov = ri.wm[r * wpr + i];
                const int oi = ri.wi[r * wpr + i];
                if (ov > mv || (ov == mv && oi < mi)) { mv = ov; mi = oi; }
            }
        }
        __syncthreads();
        // pass 2: sum of exp((x - max) / temperature)
        float sv = 0.f;
        if (stats != nullptr) {
            if (has_row && sub == 0 && is_logits && !a.greedy)
                for (int i = 0; i < n_slices; ++i) sv += __shfl(slice_sum, i);          // fixed order
        } else if (has_row && is_logits && !a.greedy) {
            const float inv_t = 1.0f / a.temperature;
#pragma unroll 8
            for (int v = sub * 64 + lane; v < V; v += wpr * 64) sv += exp_scaled(src[v], mv, inv_t);
            sv = wave_sum(sv);
        }
        if (lane == 0) ri.wm[wave] = sv;
        __syncthreads();
        if (has_row && sub == 0 && lane == 0) {
            float tot = ri.wm[r * wpr];
            for (int i = 1; i < wpr; ++i) tot += ri.wm[r * wpr + i];       // fixed order
            const int j = r0 + r;
            ri.mx[r] = mv;
            ri.sum[r] = (is_logits && !a.greedy) ? 1.0f / tot : 1.f;          // stored as 1 / sum
            ri.best[r] = mi;
            int ok = 0;
            if (j < G) {
                // a draft id outside [0, V) is never used as an index: it reads as token 0, counts as rejected
                // and raises bit 2 of the status word
                const int x_raw = a.draft_tok[b * G + j];
                const bool x_ok = (unsigned)x_raw < (unsigned)V;
                const int x = x_ok ? x_raw : 0;
                if (!x_ok && status != nullptr) atomicOr(status, 4);
                if (a.greedy) {
                    ok = x_ok && (x == mi);
                    if (a.p_tok != nullptr) a.p_tok[b * G + j] = 0.f;
                } else {
                    const TargetRow row{src, is_logits, mv, ri.sum[r], 1.0f / a.temperature};
                    const float pj = x_ok ? row.p(x) : 0.f;
                    if (a.p_tok != nullptr) a.p_tok[b * G + j] = pj;
                    ok = x_ok && __fmul_rn(a.u_acc[b * G + j], a.q[((size_t)b * G + j) * V + x]) < pj;
                }
            }
            ri.ok[r] = ok;
        }
        __syncthreads();
        // left-to-right scan of this batch (uniform over the workgroup)
        for (int r2 = 0; r2 < rows && !rejected; ++r2) {
            const int j = r0 + r2;
            if (j >= G) break;
            if (ri.ok[r2]) { ++acc; continue; }
            rejected = true;
            rej_row = r2;
        }
        const bool bonus_here = !rejected && Tp == G + 1 && G >= r0 && G < r0 + rows;
        if (rej_row >= 0 || bonus_here) {
            const int r2 = rej_row >= 0 ? rej_row : G - r0;
            const int j = r0 + r2;
            const float *rsrc = a.p_or_logits + ((size_t)b * Tp + j) * V;
            if (a.greedy) {
                new_tok = ri.best[r2];
            } else {
                const TargetRow row{rsrc, is_logits, ri.mx[r2], ri.sum[r2], 1.0f / a.temperature};
                if (rej_row >= 0) {
                    const float *q = a.q + ((size_t)b * G + j) * V;
                    new_tok = draw_fixed<1>(row, q, a.u_res[b], V, sm);
                    if (new_tok < 0) new_tok = draw_fixed<0>(row, q, a.u_res[b], V, sm);
                } else {
                    new_tok = draw_fixed<0>(row, nullptr, a.u_res[b], V, sm);
                }
            }
            rej_row = -1;
        }
        __syncthreads();
        if (rejected && (a.p_tok == nullptr || a.greedy)) break;     // later rows only matter for p_tok
    }
    if (a.greedy && a.p_tok != nullptr)
        for (int j = threadIdx.x; j < G; j += kBlock) a.p_tok[b * G + j] = 0.f;
    for (int j = threadIdx.x; j <= G; j += kBlock) {
        int t = -1;
        if (j < acc) t = a.draft_tok[b * G + j];
        else if (j == acc) t = new_tok;
        a.out_tok[b * (G + 1) + j] = t;
    }
    if (threadIdx.x == 0) {
        a.accept_len[b] = acc;
        a.n_out[b] = acc + (new_tok >= 0 ? 1 : 0);
        if (a.private_len != nullptr) {
            // (a verify step of a subset of branches keeps the lengths by cache slot)
            const int sb = slot != nullptr ? min(max(slot[b], 0), n_slots - 1) : b;
            a.private_len[sb] += min(acc + 1, Tp);
        }
    }
}

// Draft side: q = softmax(logits / temperature) written out, one token drawn from it (or the argmax).
// stats (optional): slice statistics of the rows from row_stats_kernel; without them the workgroup makes its
// own two passes over the row.
__global__ __launch_bounds__(kBlock) void softmax_sample_kernel(
        const float *logits, int64_t logits_stride, float temperature, int greedy, const float *u,
        float *q_out, int64_t q_stride, int32_t *tok_out, int64_t tok_stride, int32_t *private_len, int V,
        const SliceStats *stats, int n_slices, const int32_t *slot, int n_slots) {
    __shared__ Shared sm;
    const int b = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const float *src = logits + (size_t)b * logits_stride;
    TargetRow row{src, 1, 0.f, 1.f, 1.f / temperature};
    int best = -1;
    if (stats != nullptr) {
        // lane i takes slice i; slices ascend, so the lowest lane holding the maximum has the lowest index
        float lm = -INFINITY, ls = 0.f;
        int li = 0x7fffffff;
        if (lane < n_slices) {
            const SliceStats e = stats[(size_t)b * n_slices + lane];
            lm = e.mx;
            li = e.idx;
            ls = e.sum;
        }
        float mv = lm;
        int mi = li;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const float ov = __shfl_xor(mv, off);
            const int oi = __shfl_xor(mi, off);
            if (ov > mv || (ov == mv && oi < mi)) { mv = ov; mi = oi; }
        }
        ls = lane < n_slices ? ls * exp_scaled(lm, mv, row.inv_temp) : 0.f;
        float tot = 0.f;
        for (int i = 0; i < n_slices; ++i) tot += __shfl(ls, i);          // fixed order
        row.mx = mv;
        row.inv_sum = 1.0f / tot;
        best = mi;
    } else {
        row = make_row(src, 1, temperature, V, sm);
    }
    float *dst = q_out != nullptr ? q_out + (size_t)b * q_stride : nullptr;
    int tok;
    if (greedy) {
        if (dst != nullptr)
            for (int v = threadIdx.x; v < V; v += kBlock) dst[v] = row.p(v);
        tok = best >= 0 ? best : block_argmax(src, V, sm);
    } else {
        tok = draw_fixed<0>(row, nullptr, u[b], V, sm, dst);
    }
    if (threadIdx.x == 0) {
        tok_out[(size_t)b * tok_stride] = tok;
        if (private_len != nullptr) private_len[slot != nullptr ? min(max(slot[b], 0), n_slots - 1) : b] += 1;
    }
}

// The same over the whole chip: grid (rows, slices), behind row_stats_kernel.  One workgroup per row is a chain of
// memory round trips on 32000 logits (16 us for eight rows); here a workgroup combines the row's slice statistics
// itself (the same arithmetic in every workgroup, so all agree on max and sum), writes its slice of q and leaves
// the slice's fixed-point weight sum; the workgroup that arrives last for a row (arrival counter, zero on entry and
// left zero) picks the slice that holds the target from those integer sums and scans it.  Same token as the
// one-workgroup form: the sums are integers.
__global__ __launch_bounds__(256) void softmax_sample_slices_kernel(
        const float *logits, int V, int per, float temperature, int greedy, const float *u, float *q_out,
        int64_t q_stride, int32_t *tok_out, int64_t tok_stride, int32_t *private_len, const SliceStats *stats,
        unsigned long long *slice_sums, int *counters, const int32_t *slot, int n_slots) {
    __shared__ unsigned long long s_tot[4];
    __shared__ int s_last, s_tok;
    const int row = blockIdx.x, sl = blockIdx.y, n_slices = gridDim.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const float *src = logits + (size_t)row * V;
    TargetRow r{src, 1, 0.f, 1.f, 1.f / temperature};
    // the row's statistics from its slices (as in softmax_sample_kernel)
    float lm = -INFINITY, ls = 0.f;
    int li = 0x7fffffff;
    if (lane < n_slices) {
        const SliceStats e = stats[(size_t)row * n_slices + lane];
        lm = e.mx;
        li = e.idx;
        ls = e.sum;
    }
    float mv = lm;
    int mi = li;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(mv, off);
        const int oi = __shfl_xor(mi, off);
        if (ov > mv || (ov == mv && oi < mi)) { mv = ov; mi = oi; }
    }
    ls = lane < n_slices ? ls * exp_scaled(lm, mv, r.inv_temp) : 0.f;
    float tot = 0.f;
    for (int i = 0; i < n_slices; ++i) tot += __shfl(ls, i);          // fixed order
    r.mx = mv;
    r.inv_sum = 1.0f / tot;
    // this slice: q values out, fixed-point weights summed
    const int base = sl * per, end = min(V, base + per);
    float *dst = q_out != nullptr ? q_out + (size_t)row * q_stride : nullptr;
    unsigned long long local = 0;
#pragma unroll 4
    for (int v = base + threadIdx.x; v < end; v += 256) {
        const float p = r.p(v);
        if (dst != nullptr) dst[v] = p;
        local += to_fixed(p);
    }
    local = wave_sum_u64(local);
    if (lane == 0) s_tot[wave] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long sum = (s_tot[0] + s_tot[1]) + (s_tot[2] + s_tot[3]);
        __hip_atomic_store(slice_sums + (size_t)row * n_slices + sl, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0);
        const int old = __hip_atomic_fetch_add(counters + row, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = old == n_slices - 1;
        if (s_last) __hip_atomic_store(counters + row, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // re-arm
        s_tok = -1;
    }
    __syncthreads();
    if (!s_last) return;
    int tok = mi;                                         // greedy: the argmax (lowest index on ties)
    if (!greedy) {
        // slice sums of the row: lane i takes slice i
        unsigned long long mine = 0;
        if (lane < n_slices)
            mine = __hip_atomic_load(slice_sums + (size_t)row * n_slices + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned long long incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned long long o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        const unsigned long long Z = __shfl(incl, 63);
        if (Z != 0) {
            const unsigned long long m24 = (unsigned long long)(__fmul_rn(u[row], 16777216.0f));
            const unsigned long long t = (m24 * Z) >> 24;
            const unsigned long long hit = __ballot(incl > t);           // (t < Z: some lane passes)
            const int target = __ffsll((long long)hit) - 1;
            unsigned long long run = __shfl(incl, target) - __shfl(mine, target);
            // wavefront 0 walks the target slice in blocks of 2048 tokens, 32 consecutive tokens per lane (as in
            // draw_fixed; a slice of the draft shapes is one block)
            const int tb = target * per, te = min(V, tb + per);
            constexpr int kPerLane = 32;
            if (wave == 0) {
                for (int blk = tb; blk < te; blk += 64 * kPerLane) {
                    const int v0 = blk + lane * kPerLane;
                    unsigned long long k[kPerLane];
                    unsigned long long acc = 0;
#pragma unroll
                    for (int e = 0; e < kPerLane; ++e) {
                        const int v = v0 + e;
                        k[e] = v < te ? to_fixed(r.p(min(v, te - 1))) : 0ull;
                        acc += k[e];
                    }
                    unsigned long long inc2 = acc;
#pragma unroll
                    for (int off = 1; off < 64; off <<= 1) {
                        const unsigned long long o = __shfl_up(inc2, off);
                        if (lane >= off) inc2 += o;
                    }
                    const unsigned long long h2 = __ballot(run + inc2 > t);
                    if (h2) {
                        const int srcl = __ffsll((long long)h2) - 1;
                        if (lane == srcl) {
                            unsigned long long c = run + inc2 - acc;
                            int tk = v0;
#pragma unroll
                            for (int e = 0; e < kPerLane; ++e) {
                                c += k[e];
                                if (c > t) { tk = v0 + e; break; }
                            }
                            s_tok = tk;
                        }
                        break;
                    }
                    run += __shfl(inc2, 63);
                }
            }
        }
        __syncthreads();
        tok = s_tok;
    }
    if (threadIdx.x == 0) {
        tok_out[(size_t)row * tok_stride] = tok;
        if (private_len != nullptr) private_len[slot != nullptr ? min(max(slot[row], 0), n_slots - 1) : row] += 1;
    }
}

// ---------------------------------------------------------------------------------------------------------
// Candidate trees (Section 2.2 "Tree Attention"; Section 4.1: k_config; appendix "Details of Tree Attention").
// Nodes are numbered in level order, node 0 the root (the pending token); at position j every node of position
// j - 1 has k_j children, consecutive.  The target row of node r holds the distribution that follows the path to
// r; q row r is the draft distribution from which r's children were drawn, independently.
// The walk: at the current node the children are tested in order.  The first as in the single-candidate rule,
// fl32(u q(x)) < p(x).  After i rejections the target is the normalised i-th residual, kept in fixed point:
//   R_2[w] = trunc(max(0, fl32(p_w - q_w)) 2^38),  Z_i = sum_w R_i[w],
//   R_{i+1}[w] = max(0, R_i[w] - trunc(fl64(q_w) * fl64(Z_i)))                       (one float64 multiply)
//   candidate i is accepted iff fl64(fl32(u q(x))) * fl64(Z_i) < fl64(R_i[x])         (one float64 multiply)
// so every decision is reproducible bit for bit by a serial implementation (integer sums, IEEE products).  When all
// children are rejected a token is drawn from the last residual (from p itself if a residual sums to zero) and
// the walk ends.  This multi-round rule keeps the output law equal to the target's for candidates drawn with
// replacement; with k_j = 1 everywhere it is the chain rule.
struct TreeShape {
    int G;                    // positions (depth of the tree), 1..kMaxTreeDepth
    int k[kMaxTreeDepth];     // children per node at position j + 1
    int off[kMaxTreeDepth + 2];   // first node of level j (off[0] = 0, off[1] = 1, ..., off[G + 1] = number of nodes)
};
__device__ __forceinline__ int tree_k(const TreeShape &t, int j) {      // k of level j (1-based): static indexing only
    int v = 1;
#pragma unroll
    for (int i = 0; i < kMaxTreeDepth; ++i) v = (i == j - 1) ? t.k[i] : v;
    return v;
}
__device__ __forceinline__ int tree_off(const TreeShape &t, int j) {
    int v = 0;
#pragma unroll
    for (int i = 0; i < kMaxTreeDepth + 2; ++i) v = (i == j) ? t.off[i] : v;
    return v;
}
// level of node i >= 1 and its parent
__device__ __forceinline__ void tree_parent(const TreeShape &t, int node, int &level, int &parent) {
    level = 1;
#pragma unroll
    for (int j = 2; j <= kMaxTreeDepth; ++j)
        if (j <= t.G && node >= t.off[j]) level = j;
    parent = tree_off(t, level - 1) + (node - tree_off(t, level)) / tree_k(t, level);
}

struct TreeShared {
    float mx[kMaxTreeNodes], inv_sum[kMaxTreeNodes];
    int best[kMaxTreeNodes];
    int ok1[kMaxTreeNodes];
    unsigned long long Z[kMaxTreeNodes + 1];     // Z[i]: total of the residual after i rejections at the current node
    unsigned long long rx;
    int flag;
};

// R after `n_rej` rejections (n_rej >= 1) at a node, for token v
__device__ __forceinline__ unsigned long long tree_residual(const TargetRow &row, const float *q, int v, int n_rej,
                                                            const unsigned long long *Z) {
    const float qv = q[v];
    const float r = __fsub_rn(row.p(v), qv);
    unsigned long long R = r > 0.f ? to_fixed(r) : 0ull;
    for (int i = 1; i < n_rej; ++i) {
        const unsigned long long Qz = (unsigned long long)__dmul_rn((double)qv, (double)Z[i]);
        R = R > Qz ? R - Qz : 0ull;
    }
    return R;
}

__device__ unsigned long long block_sum_u64(unsigned long long v, Shared &sm) {
    v = wave_sum_u64(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm.tot[threadIdx.x >> 6] = v;
    __syncthreads();
    unsigned long long r = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) r += sm.tot[i];
    return r;
}

// Fixed-point inverse CDF over the residual after n_rej rejections (the scan of draw_fixed on those weights).
__device__ int draw_tree_residual(const TargetRow &row, const float *q, int n_rej, const unsigned long long *Zs,
                                  float u, int V, Shared &sm) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int per = (((V + kWaves - 1) / kWaves) + 63) & ~63;
    const int base = wave * per;
    const int end = min(V, base + per);
    unsigned long long local = 0;
    for (int v = base + lane; v < end; v += 64) local += tree_residual(row, q, v, n_rej, Zs);
    local = wave_sum_u64(local);
    __syncthreads();
    if (lane == 0) sm.tot[wave] = local;
    if (threadIdx.x == 0) sm.tok = -1;
    __syncthreads();
    unsigned long long Z = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) Z += sm.tot[i];
    if (Z == 0) return -1;
    const unsigned long long m24 = (unsigned long long)(__fmul_rn(u, 16777216.0f));
    const unsigned long long t = (m24 * Z) >> 24;
    unsigned long long run = 0;
    int target = 0;
    for (int i = 0; i < kWaves; ++i) {
        unsigned long long nx = run + sm.tot[i];
        if (t < nx) { target = i; break; }
        run = nx;
    }
    if (wave == target) {
        for (int blk = base; blk < end; blk += 64) {
            const int v = blk + lane;
            const unsigned long long mine = v < end ? tree_residual(row, q, v, n_rej, Zs) : 0ull;
            unsigned long long incl = mine;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                unsigned long long o = __shfl_up(incl, off);
                if (lane >= off) incl += o;
            }
            const unsigned long long hit = __ballot(run + incl > t);
            if (hit) {
                if (lane == __ffsll((long long)hit) - 1) sm.tok = v;
                break;
            }
            run += __shfl(incl, 63);
        }
    }
    __syncthreads();
    return sm.tok;
}

// One workgroup per branch.  Phase A: softmax statistics of every target row (from the slices of
// row_stats_kernel, or computed here).  Phase B: the first-round test of every node, one thread per node.
// Phase C: the walk, uniform over the workgroup; residual totals and the final draw use all 16 wavefronts.
__global__ __launch_bounds__(kBlock) void accept_tree_kernel(seed_accept_args a, TreeShape t, const SliceStats *stats,
                                                            int n_slices, const int32_t *slot, int n_slots,
                                                            int32_t *status, int32_t *commit_rows) {
    __shared__ Shared sm;
    __shared__ TreeShared ts;
    const int b = blockIdx.x;
    const int G = t.G, Tp = a.n_target_rows, V = a.vocab;
    const int n_nodes = tree_off(t, G + 1), n_par = tree_off(t, G);
    const int is_logits = a.probs_kind == SEED_KIND_LOGITS;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const float inv_temp = a.greedy ? 1.0f : 1.0f / a.temperature;
    const float *rows = a.p_or_logits + (size_t)b * Tp * V;
    // ---- phase A
    if (is_logits || a.greedy) {
        if (stats != nullptr) {
            for (int r = wave; r < Tp; r += kWaves) {
                const SliceStats *st = stats + ((size_t)b * Tp + r) * n_slices;
                float lm = -INFINITY, ls = 0.f;
                int li = 0x7fffffff;
                if (lane < n_slices) {
                    const SliceStats e = st[lane];
                    lm = e.mx; li = e.idx; ls = e.sum;
                }
                float mv = lm;
                int mi = li;
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    const float ov = __shfl_xor(mv, off);
                    const int oi = __shfl_xor(mi, off);
                    if (ov > mv || (ov == mv && oi < mi)) { mv = ov; mi = oi; }
                }
                ls = lane < n_slices ? ls * exp_scaled(lm, mv, inv_temp) : 0.f;
                float tot = 0.f;
                for (int i = 0; i < n_slices; ++i) tot += __shfl(ls, i);          // fixed order
                if (lane == 0) { ts.mx[r] = mv; ts.inv_sum[r] = 1.0f / tot; ts.best[r] = mi; }
            }
        } else {
            for (int r = 0; r < Tp; ++r) {
                const float *src = rows + (size_t)r * V;
                if (a.greedy) {
                    const int best = block_argmax(src, V, sm);
                    if (threadIdx.x == 0) { ts.mx[r] = 0.f; ts.inv_sum[r] = 1.f; ts.best[r] = best; }
                } else {
                    const TargetRow row = make_row(src, 1, a.temperature, V, sm);
                    if (threadIdx.x == 0) { ts.mx[r] = row.mx; ts.inv_sum[r] = row.inv_sum; ts.best[r] = -1; }
                }
                __syncthreads();
            }
        }
    } else {
        for (int r = threadIdx.x; r < Tp; r += kBlock) { ts.mx[r] = 0.f; ts.inv_sum[r] = 1.f; ts.best[r] = -1; }
    }
    __syncthreads();
    auto row_of = [&](int r) { return TargetRow{rows + (size_t)r * V, is_logits, ts.mx[r], ts.inv_sum[r], inv_temp}; };
    const int32_t *tok = a.draft_tok + (size_t)b * (n_nodes - 1);            // entry i - 1: node i
    // ---- phase B: node i against the distribution at its parent (a token id outside [0, V) reads as token 0,
    // counts as rejected in every round and raises bit 2 of the status word)
    for (int i = 1 + threadIdx.x; i < n_nodes; i += kBlock) {
        int level, par;
        tree_parent(t, i, level, par);
        const int x_raw = tok[i - 1];
        const bool x_ok = (unsigned)x_raw < (unsigned)V;
        const int x = x_ok ? x_raw : 0;
        if (!x_ok && status != nullptr) atomicOr(status, 4);
        int ok = 0;
        float pj = 0.f;
        if (a.greedy) {
            ok = x_ok && x == ts.best[par];
        } else {
            pj = x_ok ? row_of(par).p(x) : 0.f;
            ok = x_ok && __fmul_rn(a.u_acc[(size_t)b * (n_nodes - 1) + i - 1], a.q[((size_t)b * n_par + par) * V + x]) < pj;
        }
        ts.ok1[i] = ok;
        if (a.p_tok != nullptr) a.p_tok[(size_t)b * (n_nodes - 1) + i - 1] = pj;
    }
    __syncthreads();
    // ---- phase C
    int cur = 0, local = 0, acc = 0, new_tok = -1;      // current node, its index within its level, accepted depth
    for (int level = 1; level <= G; ++level) {
        const int kj = tree_k(t, level);
        const int c0 = tree_off(t, level) + local * kj;
        const float *q = a.greedy ? nullptr : a.q + ((size_t)b * n_par + cur) * V;
        const TargetRow row = row_of(cur);
        int chosen = -1, n_rej = 0;
        bool dead = false;                              // a residual summed to zero: stop testing, draw from p
        for (int i = 0; i < kj; ++i) {
            const int c = c0 + i;
            int ok;
            if (i == 0 || a.greedy) {
                ok = ts.ok1[c];
            } else {
                if (threadIdx.x == 0) {
                    const int x_raw = tok[c - 1];
                    const bool x_ok = (unsigned)x_raw < (unsigned)V;
                    const int x = x_ok ? x_raw : 0;
                    const float uq = __fmul_rn(a.u_acc[(size_t)b * (n_nodes - 1) + c - 1], q[x]);
                    const unsigned long long R = tree_residual(row, q, x, n_rej, ts.Z);
                    ts.flag = x_ok && __dmul_rn((double)uq, (double)ts.Z[n_rej]) < (double)R;
                }
                __syncthreads();
                ok = ts.flag;
            }
            if (ok) { chosen = c; break; }
            if (a.greedy) continue;
            // rejected: total of the next residual
            ++n_rej;
            unsigned long long part = 0;
            for (int v = threadIdx.x; v < V; v += kBlock) part += tree_residual(row, q, v, n_rej, ts.Z);
            const unsigned long long Z = block_sum_u64(part, sm);
            __syncthreads();
            if (threadIdx.x == 0) ts.Z[n_rej] = Z;
            __syncthreads();
            if (Z == 0) { dead = true; break; }
        }
        if (chosen < 0) {
            if (a.greedy) {
                new_tok = ts.best[cur];
            } else {
                new_tok = dead ? -1 : draw_tree_residual(row, q, n_rej, ts.Z, a.u_res[b], V, sm);
                if (new_tok < 0) new_tok = draw_fixed<0>(row, nullptr, a.u_res[b], V, sm);
            }
            break;
        }
        if (threadIdx.x == 0) {
            a.out_tok[(size_t)b * (G + 1) + acc] = tok[chosen - 1];
            if (a.path_node != nullptr) a.path_node[(size_t)b * G + acc] = chosen;
            if (commit_rows != nullptr) commit_rows[(size_t)b * (kMaxTreeDepth + 2) + 1 + acc] = chosen;
        }
        cur = chosen;
        local = chosen - tree_off(t, level);
        ++acc;
        __syncthreads();
    }
    if (acc == G && Tp == n_nodes && n_par < n_nodes) {                 // bonus rows: a token after a full path
        if (a.greedy) new_tok = ts.best[cur];
        else new_tok = draw_fixed<0>(row_of(cur), nullptr, a.u_res[b], V, sm);
    }
    for (int j = acc + threadIdx.x; j <= G; j += kBlock) a.out_tok[(size_t)b * (G + 1) + j] = (j == acc) ? new_tok : -1;
    if (a.path_node != nullptr)
        for (int j = acc + threadIdx.x; j < G; j += kBlock) a.path_node[(size_t)b * G + j] = -1;
    if (threadIdx.x == 0) {
        a.accept_len[b] = acc;
        a.n_out[b] = acc + (new_tok >= 0 ? 1 : 0);
        // rows that stay in the cache: the root and the accepted nodes that were fed (Algorithm 1's bookkeeping)
        const int n_commit = min(acc + 1, Tp == n_nodes ? G + 1 : G);
        if (commit_rows != nullptr) {
            commit_rows[(size_t)b * (kMaxTreeDepth + 2)] = n_commit;
            commit_rows[(size_t)b * (kMaxTreeDepth + 2) + 1 + acc] = -1;
        }
        if (a.private_len != nullptr) {
            const int sb = slot != nullptr ? min(max(slot[b], 0), n_slots - 1) : b;
            a.private_len[sb] += n_commit;
        }
    }
}

__global__ __launch_bounds__(kBlock) void sample_probs_kernel(const float *probs, int64_t row_stride,
                                                              const float *u, int32_t *tok_out, int V) {
    __shared__ Shared sm;
    const int b = blockIdx.x;
    TargetRow row{probs + (size_t)b * row_stride, 0, 0.f, 1.f, 1.f};
    int tok = draw_fixed<0>(row, nullptr, u[b], V, sm);
    if (threadIdx.x == 0) tok_out[b] = tok;
}

}  // namespace

// Number of vocabulary slices of the row statistics launch for a given number of rows, and a slice's length.
static int stats_slices(int rows, int vocab, int *per) {
    int n_slices = rows <= 32 ? 16 : (rows <= 64 ? 8 : 4);
    while (n_slices > 1 && vocab / n_slices < 256) n_slices /= 2;
    *per = (((vocab + n_slices - 1) / n_slices) + 63) & ~63;
    return (vocab + *per - 1) / *per;
}

// (slice statistics, then -- draft side -- the slices' 64-bit weight sums)
size_t accept_scratch_bytes(int max_rows) { return (size_t)max_rows * kMaxSlices * (sizeof(SliceStats) + 8); }

// The row statistics of the entry point that allocates nothing (seed_accept_resample_static): one copy of this
// array per GPU, held until the process ends.  1 MiB: kStaticAcceptRows rows x 16 slices x 16 bytes.
// Every slice entry a call reads is written by that call's row statistics launch first, so nothing here needs
// clearing between calls; calls that overlap on one GPU would share it and race.
static __device__ __align__(256) unsigned char scratch[(size_t)kStaticAcceptRows * kMaxSlices * sizeof(SliceStats)];

// Device address of this GPU's copy of the array (the array's name is only a host-side stand-in for it).
// Looked up once per device, with that device current; no allocation.
int accept_static_scratch(void **out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *ptrs[kMaxDevices] = {};
    int dev = -1;
    int rc = hip_fail(hipGetDevice(&dev), "hipGetDevice");
    if (rc) return rc;
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("accept: device ordinal %d is outside the table of %d", dev, kMaxDevices);
        return SEED_E_CAPACITY;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (ptrs[dev] == nullptr) {
        void *p = nullptr;
        rc = hip_fail(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (rc) return rc;
        if (p == nullptr) { set_error("accept: the static scratch array has no device address"); return SEED_E_HIP; }
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return SEED_OK;
}

// scratch (optional, accept_scratch_bytes(n_branches * n_target_rows) bytes): with it the softmax statistics
// of the rows are computed by a launch that fills the chip; without it inside the one workgroup per branch.
// status (optional): device status word; bit 2 is raised by a draft token id outside [0, vocab).
int launch_accept(const seed_accept_args &a, void *scratch, const int32_t *branch_slot, int n_slots,
                  int32_t *status, hipStream_t st) {
    if (a.n_branches == 0) return SEED_OK;
    const bool need_stats = a.probs_kind == SEED_KIND_LOGITS || a.greedy;
    SliceStats *stats = nullptr;
    int n_slices = 0;
    if (scratch != nullptr && need_stats) {
        const int rows = a.n_branches * a.n_target_rows;
        int per;
        n_slices = stats_slices(rows, a.vocab, &per);
        stats = (SliceStats *)scratch;
        hipLaunchKernelGGL(row_stats_kernel, dim3(rows, n_slices), dim3(256), 0, st, a.p_or_logits, a.vocab, per,
                           a.greedy ? 1.0f : 1.0f / a.temperature, stats);
    }
    hipLaunchKernelGGL(accept_resample_kernel, dim3(a.n_branches), dim3(kBlock), 0, st, a, stats, n_slices,
                       branch_slot, n_slots, status);
    return hip_fail(hipGetLastError(), "accept_resample launch");
}

int launch_accept_tree(const seed_accept_args &a, const TreeInfo &ti, void *scratch, const int32_t *branch_slot,
                       int n_slots, int32_t *status, int32_t *commit_rows, hipStream_t st) {
    if (a.n_branches == 0) return SEED_OK;
    TreeShape t{};
    t.G = ti.G;
    for (int i = 0; i < kMaxTreeDepth; ++i) t.k[i] = i < ti.G ? ti.k[i] : 1;
    for (int i = 0; i < kMaxTreeDepth + 2; ++i) t.off[i] = i <= ti.G + 1 ? ti.off[i] : ti.n_nodes;
    const bool need_stats = a.probs_kind == SEED_KIND_LOGITS || a.greedy;
    SliceStats *stats = nullptr;
    int n_slices = 0;
    if (scratch != nullptr && need_stats) {
        const int rows = a.n_branches * a.n_target_rows;
        int per;
        n_slices = stats_slices(rows, a.vocab, &per);
        stats = (SliceStats *)scratch;
        hipLaunchKernelGGL(row_stats_kernel, dim3(rows, n_slices), dim3(256), 0, st, a.p_or_logits, a.vocab, per,
                           a.greedy ? 1.0f : 1.0f / a.temperature, stats);
    }
    hipLaunchKernelGGL(accept_tree_kernel, dim3(a.n_branches), dim3(kBlock), 0, st, a, t, stats, n_slices, branch_slot,
                       n_slots, status, commit_rows);
    return hip_fail(hipGetLastError(), "accept_tree launch");
}

// scratch (optional, accept_scratch_bytes(n_rows) bytes, rows contiguous: logits_stride == vocab): as in
// launch_accept, followed by the rows' slice sums.  counters (optional, one int per row, zero on entry, left zero):
// with scratch and counters the draw runs over (rows, slices) workgroups, else one workgroup per row.
int launch_softmax_sample(const float *logits, int64_t logits_stride, float temperature, int greedy,
                          const float *u, float *q_out, int64_t q_stride, int32_t *tok_out,
                          int64_t tok_stride, int32_t *private_len, int n_rows, int vocab, void *scratch,
                          int *counters, const int32_t *branch_slot, int n_slots, hipStream_t st) {
    if (n_rows == 0) return SEED_OK;
    SliceStats *stats = nullptr;
    int n_slices = 0, per = 0;
    if (scratch != nullptr && logits_stride == vocab) {
        n_slices = stats_slices(n_rows, vocab, &per);
        stats = (SliceStats *)scratch;
        hipLaunchKernelGGL(row_stats_kernel, dim3(n_rows, n_slices), dim3(256), 0, st, logits, vocab, per,
                           1.0f / temperature, stats);
    }
    if (stats != nullptr && counters != nullptr) {
        unsigned long long *sums = (unsigned long long *)((char *)scratch + (size_t)n_rows * kMaxSlices * sizeof(SliceStats));
        hipLaunchKernelGGL(softmax_sample_slices_kernel, dim3(n_rows, n_slices), dim3(256), 0, st, logits, vocab, per,
                           temperature, greedy, u, q_out, q_stride, tok_out, tok_stride, private_len, stats, sums,
                           counters, branch_slot, n_slots);
        return hip_fail(hipGetLastError(), "softmax_sample launch");
    }
    hipLaunchKernelGGL(softmax_sample_kernel, dim3(n_rows), dim3(kBlock), 0, st, logits, logits_stride,
                       temperature, greedy, u, q_out, q_stride, tok_out, tok_stride, private_len, vocab, stats,
                       n_slices, branch_slot, n_slots);
    return hip_fail(hipGetLastError(), "softmax_sample launch");
}

int launch_sample_probs(const float *probs, int64_t row_stride, const float *u, int32_t *tok_out,
                        int n_rows, int vocab, hipStream_t st) {
    if (n_rows == 0) return SEED_OK;
    hipLaunchKernelGGL(sample_probs_kernel, dim3(n_rows), dim3(kBlock), 0, st, probs, row_stride, u,
                       tok_out, vocab);
    return hip_fail(hipGetLastError(), "sample_probs launch");
}

}  // namespace seedv
