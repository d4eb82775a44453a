// Rounds-scheduled speculative execution (paper Section 3.3, Algorithm 1) on one GPU: host-side scheduler
// over the two entry points of the hot path, seed_draft_step (draft context, its own stream) and
// seed_verify_step (target context, its own stream), both over subsets of cache slots.
//
// A scheduling unit is a group of branches that were ready together.  For every unit the host enqueues, in
// this order and without waiting: [draft stream] k draft steps; [target stream] wait for that unit's draft
// event, one verify + accept step, copy of the accept results to pinned host memory.  Units are verified in
// the order in which they were formed (first come, first served); the host only ever blocks on the oldest
// unit's "verified" event, folds its results into the branches' state, and forms new units from the
// branches that became ready.  While one unit is verified the next one drafts: the two streams overlap.
#include <chrono>
#include <deque>
#include <vector>

#include "seed_internal.h"
#include "../../include/seed_sched.h"

namespace seedv {
namespace {

constexpr int kMaxN = SEED_SCHED_MAX_BRANCHES;

struct UnitInit {          // passed by value: the host knows slots, positions and pending tokens
    int n;
    int slot[kMaxN], pos[kMaxN], pending[kMaxN];
};
struct SetLen {
    int n;
    int slot[kMaxN], val[kMaxN];
};

// Staging of one unit, rows r0 .. r0+n of the ring: cache slots, pending tokens, and the uniforms of this
// round gathered by position (u[b][L + j]).
__global__ void sched_unit_init_kernel(UnitInit u, const float *u_draft, const float *u_acc, const float *u_res,
                                       int stride, int gamma, int cap, int r0, int32_t *slots, int32_t *pend,
                                       int32_t *cur, float *ud, float *ua, float *ur) {
    const int i = threadIdx.x;
    if (i >= u.n) return;
    const int r = r0 + i;
    slots[r] = u.slot[i];
    pend[r] = u.pending[i];
    cur[r] = u.pending[i];
    const size_t base = (size_t)u.slot[i] * stride + u.pos[i];
    for (int j = 0; j < gamma; ++j) {
        ud[(size_t)j * cap + r] = u_draft[base + j];      // [gamma][cap]: step j reads a dense run of n values
        ua[(size_t)r * gamma + j] = u_acc[base + j];
    }
    ur[r] = u_res[base];
}

// cur[r] = draft token j of row r: the input of draft step j + 1
__global__ void sched_next_input_kernel(const int32_t *draft_tok, int gamma, int j, int r0, int n, int32_t *cur) {
    const int i = threadIdx.x;
    if (i < n) cur[r0 + i] = draft_tok[(size_t)(r0 + i) * gamma + j];
}

// verify rows of a unit: the pending token, then drafts 1 .. gamma-1 (the gamma-th draft is never fed)
__global__ void sched_build_rows_kernel(const int32_t *pend, const int32_t *draft_tok, int gamma, int r0, int n,
                                        int32_t *row_tok) {
    const int i = threadIdx.x / gamma, j = threadIdx.x % gamma;
    if (i >= n) return;
    const size_t r = (size_t)(r0 + i);
    row_tok[r * gamma + j] = j == 0 ? pend[r] : draft_tok[r * gamma + j - 1];
}

__global__ void sched_set_len_kernel(SetLen s, int32_t *len) {
    const int i = threadIdx.x;
    if (i < s.n) len[s.slot[i]] = s.val[i];
}

struct Layout {
    int cap;     // ring rows (3n: a unit's rows are contiguous, units are freed in the order they were taken)
    size_t q, draft_tok, row_tok, cur, pend, slots, ud, ua, ur, alen, otok, nout, total;
};
Layout make_layout(int n, int gamma, int vocab) {
    Layout L{};
    L.cap = 3 * n;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = (off + bytes + 255) & ~(size_t)255; return o; };
    L.q = take((size_t)L.cap * gamma * vocab * 4);
    L.draft_tok = take((size_t)L.cap * gamma * 4);
    L.row_tok = take((size_t)L.cap * gamma * 4);
    L.cur = take((size_t)L.cap * 4);
    L.pend = take((size_t)L.cap * 4);
    L.slots = take((size_t)L.cap * 4);
    L.ud = take((size_t)L.cap * gamma * 4);
    L.ua = take((size_t)L.cap * gamma * 4);
    L.ur = take((size_t)L.cap * 4);
    L.alen = take((size_t)L.cap * 4);
    L.otok = take((size_t)L.cap * (gamma + 1) * 4);
    L.nout = take((size_t)L.cap * 4);
    L.total = off;
    return L;
}

struct Unit {
    int n = 0, r0 = 0;
    int branch[kMaxN];
    hipEvent_t drafted = nullptr, verified = nullptr;
};

struct Branch {
    int emitted = 0;       // validated tokens so far (L_i of Algorithm 1, counted from 0)
    int pending = 0;       // validated token whose KV is not cached yet
    int draft_len = 0;     // committed rows of the draft context's private cache
    bool done = false;
};

}  // namespace
}  // namespace seedv

using namespace seedv;

extern "C" {

size_t seed_sched_workspace_bytes(int32_t n_branches, int32_t gamma, int32_t vocab) {
    if (n_branches < 1 || n_branches > kMaxN || gamma < 1 || vocab < 1) return 0;
    return make_layout(n_branches, gamma, vocab).total;
}

int seed_sched_run(seed_ctx *target, seed_ctx *draft, const seed_sched_args *a) {
    if (target == nullptr || draft == nullptr) { set_error("sched: a context is NULL"); return SEED_E_NOT_INIT; }
    if (a == nullptr) { set_error("sched: args is NULL"); return SEED_E_NULL_PTR; }
    const seed_model_cfg &gt = seed_ctx_cfg(target), &gd = seed_ctx_cfg(draft);
    const int n = a->n_branches, G = a->gamma, V = gt.vocab;
    if (n < 1 || n > kMaxN || G < 1 || a->max_new < 1) {
        set_error("sched: need 1 <= n_branches <= %d, gamma >= 1, max_new >= 1", kMaxN);
        return SEED_E_INVALID_ARG;
    }
    if (gt.dtype == SEED_DTYPE_F32 || gd.dtype == SEED_DTYPE_F32) {
        set_error("sched: both contexts must be bf16 contexts");
        return SEED_E_UNSUPPORTED_DTYPE;
    }
    if (gd.vocab != V) { set_error("sched: draft vocab %d != target vocab %d", gd.vocab, V); return SEED_E_SHAPE; }
    if (n > gt.max_branches || n > gd.max_branches || G > gt.max_rows_per_branch) {
        set_error("sched: n_branches / gamma exceed the contexts' capacity");
        return SEED_E_CAPACITY;
    }
    if (!(a->temperature > 0.f) || a->u_stride < a->max_new + G) {
        set_error("sched: need temperature > 0 and u_stride >= max_new + gamma");
        return SEED_E_INVALID_ARG;
    }
    if (!a->first_tok || !a->u_draft || !a->u_acc || !a->u_res || !a->target_private_len || !a->draft_private_len ||
        !a->workspace || !a->out_tok || !a->out_len) {
        set_error("sched: a required pointer is NULL");
        return SEED_E_NULL_PTR;
    }
    const Layout L = make_layout(n, G, V);
    if (((uintptr_t)a->workspace & 255) != 0 || a->workspace_bytes < L.total) {
        set_error("sched: workspace must be 256-byte aligned and hold %zu bytes", L.total);
        return SEED_E_CAPACITY;
    }
    char *ws = (char *)a->workspace;
    float *q = (float *)(ws + L.q), *ud = (float *)(ws + L.ud), *ua = (float *)(ws + L.ua), *ur = (float *)(ws + L.ur);
    int32_t *draft_tok = (int32_t *)(ws + L.draft_tok), *row_tok = (int32_t *)(ws + L.row_tok);
    int32_t *cur = (int32_t *)(ws + L.cur), *pend = (int32_t *)(ws + L.pend), *slots = (int32_t *)(ws + L.slots);
    int32_t *alen = (int32_t *)(ws + L.alen), *otok = (int32_t *)(ws + L.otok), *nout = (int32_t *)(ws + L.nout);
    hipStream_t sd = seed_ctx_stream(draft), st = seed_ctx_stream(target);
    const int U = (a->unit_branches <= 0 || a->unit_branches > n) ? n : a->unit_branches;

    // host state (the contexts' earlier work, e.g. their prefills, must be complete before lengths are read)
    std::vector<Branch> br(n);
    std::vector<int32_t> dlen0(n);
    int rc;
    if ((rc = hip_fail(hipStreamSynchronize(sd), "sched: draft stream")) ||
        (rc = hip_fail(hipStreamSynchronize(st), "sched: target stream")))
        return rc;
    rc = hip_fail(hipMemcpy(dlen0.data(), a->draft_private_len, sizeof(int32_t) * n, hipMemcpyDeviceToHost),
                      "sched: read draft lengths");
    if (rc) return rc;
    for (int b = 0; b < n; ++b) {
        br[b].pending = a->first_tok[b];
        br[b].draft_len = dlen0[b];
        a->out_len[b] = 0;
    }
    int32_t *hres = nullptr;                                  // pinned: [cap] alen, [cap] nout, [cap][G+1] otok
    rc = hip_fail(hipHostMalloc((void **)&hres, (size_t)L.cap * (G + 3) * sizeof(int32_t), hipHostMallocDefault),
                  "sched: pinned buffer");
    if (rc) return rc;
    int32_t *h_alen = hres, *h_nout = hres + L.cap, *h_otok = hres + 2 * L.cap;
    std::vector<hipEvent_t> events;
    auto new_event = [&](hipEvent_t *e) {
        int r = hip_fail(hipEventCreateWithFlags(e, hipEventDisableTiming), "sched: event");
        if (!r) events.push_back(*e);
        return r;
    };
    seed_sched_stats stats{};
    std::deque<int> ready;
    for (int b = 0; b < n; ++b) ready.push_back(b);
    std::deque<Unit> inflight;
    int ring_next = 0, n_done = 0;
    const auto t0 = std::chrono::steady_clock::now();

    // enqueue the drafting and the verification of one unit (nothing here waits for the GPU)
    auto launch_unit = [&](Unit &u) -> int {
        if (ring_next + u.n > L.cap) ring_next = 0;
        u.r0 = ring_next;
        ring_next += u.n;
        int r;
        if ((r = new_event(&u.drafted)) || (r = new_event(&u.verified))) return r;
        UnitInit ui{};
        ui.n = u.n;
        for (int i = 0; i < u.n; ++i) {
            const Branch &B = br[u.branch[i]];
            ui.slot[i] = u.branch[i];
            ui.pos[i] = B.emitted;
            ui.pending[i] = B.pending;
        }
        hipLaunchKernelGGL(sched_unit_init_kernel, dim3(1), dim3(64), 0, sd, ui, a->u_draft, a->u_acc, a->u_res,
                           a->u_stride, G, L.cap, u.r0, slots, pend, cur, ud, ua, ur);
        if ((r = hip_fail(hipGetLastError(), "sched: unit init launch"))) return r;
        for (int j = 0; j < G; ++j) {
            seed_draft_args da{};
            da.n_branches = u.n;
            da.shared_len = a->shared_len_draft;
            da.temperature = a->temperature;
            da.row_tok = cur + u.r0;
            da.private_len = a->draft_private_len;
            da.u = ud + (size_t)j * L.cap + u.r0;
            da.q_out = q + ((size_t)u.r0 * G + j) * V;
            da.q_stride = (int64_t)G * V;
            da.tok_out = draft_tok + (size_t)u.r0 * G + j;
            da.tok_stride = G;
            da.branch_slot = slots + u.r0;
            if ((r = seed_draft_step(draft, &da))) return r;
            ++stats.draft_steps;
            if (j + 1 < G) {
                hipLaunchKernelGGL(sched_next_input_kernel, dim3(1), dim3(64), 0, sd, draft_tok, G, j, u.r0, u.n, cur);
                if ((r = hip_fail(hipGetLastError(), "sched: next input launch"))) return r;
            }
        }
        if ((r = hip_fail(hipEventRecord(u.drafted, sd), "sched: record drafted"))) return r;
        // verification: first come, first served = the order of these calls on the target stream
        if ((r = hip_fail(hipStreamWaitEvent(st, u.drafted, 0), "sched: wait for drafts"))) return r;
        hipLaunchKernelGGL(sched_build_rows_kernel, dim3(1), dim3(u.n * G), 0, st, pend, draft_tok, G, u.r0, u.n,
                           row_tok);
        if ((r = hip_fail(hipGetLastError(), "sched: build rows launch"))) return r;
        seed_accept_args acc{};
        acc.gamma = G;
        acc.temperature = a->temperature;
        acc.q = q + (size_t)u.r0 * G * V;
        acc.draft_tok = draft_tok + (size_t)u.r0 * G;
        acc.u_acc = ua + (size_t)u.r0 * G;
        acc.u_res = ur + u.r0;
        acc.accept_len = alen + u.r0;
        acc.out_tok = otok + (size_t)u.r0 * (G + 1);
        acc.n_out = nout + u.r0;
        seed_step_args sa{};
        sa.n_branches = u.n;
        sa.rows_per_branch = G;
        sa.shared_len = a->shared_len_target;
        sa.row_tok = row_tok + (size_t)u.r0 * G;
        sa.private_len = a->target_private_len;
        sa.accept = &acc;
        sa.branch_slot = slots + u.r0;
        if ((r = seed_verify_step(target, &sa))) return r;
        if ((r = hip_fail(hipMemcpyAsync(h_alen + u.r0, alen + u.r0, sizeof(int32_t) * u.n, hipMemcpyDeviceToHost, st),
                          "sched: copy accept_len")) ||
            (r = hip_fail(hipMemcpyAsync(h_nout + u.r0, nout + u.r0, sizeof(int32_t) * u.n, hipMemcpyDeviceToHost, st),
                          "sched: copy n_out")) ||
            (r = hip_fail(hipMemcpyAsync(h_otok + (size_t)u.r0 * (G + 1), otok + (size_t)u.r0 * (G + 1),
                                         sizeof(int32_t) * u.n * (G + 1), hipMemcpyDeviceToHost, st),
                          "sched: copy out_tok")))
            return r;
        return hip_fail(hipEventRecord(u.verified, st), "sched: record verified");
    };

    // fold a verified unit into its branches (Algorithm 1, verification process: accepted drafts extend the
    // validated sequence, the first rejection adds the target's replacement token and ends the round)
    auto retire_unit = [&](const Unit &u) -> int {
        SetLen sl{};
        sl.n = u.n;
        for (int i = 0; i < u.n; ++i) {
            const int b = u.branch[i], r = u.r0 + i;
            Branch &B = br[b];
            const int acc_n = h_alen[r], n_o = h_nout[r];
            if (acc_n < 0 || acc_n > G || n_o < acc_n || n_o > G + 1 || n_o < 1) {
                set_error("sched: implausible accept result (%d accepted, %d emitted) for branch %d", acc_n, n_o, b);
                return SEED_E_HIP;
            }
            const int32_t *toks = h_otok + (size_t)r * (G + 1);
            for (int j = 0; j < n_o; ++j)
                if (B.emitted + j < a->max_new) a->out_tok[(size_t)b * a->max_new + B.emitted + j] = toks[j];
            B.emitted += n_o;
            B.pending = toks[n_o - 1];                        // replacement token, or the gamma-th accepted draft
            B.draft_len += (acc_n + 1 < G) ? acc_n + 1 : G;   // rows of this round the draft cache keeps
            sl.slot[i] = b;
            sl.val[i] = B.draft_len;
            stats.drafted += G;
            stats.accepted += acc_n;
            stats.emitted += n_o;
            if (B.emitted >= a->max_new) {
                B.done = true;
                a->out_len[b] = a->max_new;
                ++n_done;
            } else {
                a->out_len[b] = B.emitted;
                ready.push_back(b);
            }
        }
        ++stats.units;
        // the draft context appended gamma rows per branch while drafting: keep only the validated ones
        hipLaunchKernelGGL(sched_set_len_kernel, dim3(1), dim3(64), 0, sd, sl, a->draft_private_len);
        return hip_fail(hipGetLastError(), "sched: set draft lengths launch");
    };

    auto fail = [&](int code) {
        (void)hipStreamSynchronize(sd);
        (void)hipStreamSynchronize(st);
        for (hipEvent_t e : events) (void)hipEventDestroy(e);
        (void)hipHostFree(hres);
        return code;
    };

    while (n_done < n) {
        while (!ready.empty()) {                              // form units from whatever is ready, in order
            Unit u;
            while (u.n < U && !ready.empty()) {
                u.branch[u.n++] = ready.front();
                ready.pop_front();
            }
            if ((rc = launch_unit(u))) return fail(rc);
            inflight.push_back(u);
        }
        if (inflight.empty()) { set_error("sched: no unit in flight but %d branches unfinished", n - n_done); return fail(SEED_E_HIP); }
        const Unit u = inflight.front();
        inflight.pop_front();
        if ((rc = hip_fail(hipEventSynchronize(u.verified), "sched: wait for a verified unit"))) return fail(rc);
        if ((rc = retire_unit(u))) return fail(rc);
    }
    if ((rc = hip_fail(hipStreamSynchronize(sd), "sched: draft stream")) ||
        (rc = hip_fail(hipStreamSynchronize(st), "sched: target stream")))
        return fail(rc);
    stats.wall_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    if (a->stats) *a->stats = stats;
    return fail(SEED_OK);
}

}  // extern "C"
