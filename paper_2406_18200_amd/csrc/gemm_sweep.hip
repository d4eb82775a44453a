// Stand-alone timing of the projection kernels over workgroup shapes, n-tiles per wavefront, split-K factors and
// both kernel forms, on the projection shapes of the 7B / 13B decoders: the measurements gemm_bf16_pick's rules
// come from.  Not part of the library.
//
//   python -m paper_2406_18200_amd.build --sweep        (builds paper_2406_18200_amd/gemm_sweep)
//   gemm_sweep ROWS [MODE] [BIG]     ROWS 1..128; MODE 0 = every configuration, 1 = the picked one only,
//                                    2 = the picked one and every wide-form one; BIG 1 = 13B shapes
//
// Weights rotate through a 3 GiB pool so that no launch finds its weights in a cache; every launch is the
// library's own launcher (shape checks included); a line "[run] ..." is flushed before each configuration.
#include "gemm_bf16.hip"
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <utility>
#include <vector>

namespace seedv {
void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vprintf(fmt, ap);
    va_end(ap);
    printf("\n");
}
int hip_fail(hipError_t e, const char *what) {
    if (e == hipSuccess) return 0;
    printf("%s: %s\n", what, hipGetErrorString(e));
    return SEED_E_HIP;
}
}  // namespace seedv
using namespace seedv;

#define CK(x)                                                                     \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

int main(int argc, char **argv) {
    const int M = argc > 1 ? atoi(argv[1]) : 12;
    const int mode = argc > 2 ? atoi(argv[2]) : 0;
    const int big = argc > 3 ? atoi(argv[3]) : 0;
    if (M < 1 || M > 128) {
        printf("ROWS must be 1..128\n");
        return 2;
    }
    const int d = big ? 5120 : 4096, F = big ? 13824 : 11008, V = 32000;
    const int Mp = (M + 15) / 16 * 16, m_tiles = Mp / 16;
    const size_t pool_bytes = (size_t)3 << 30;
    const size_t part_floats = (size_t)M * 65536 * 2;          // split-K partials: up to 8 x M x 16384 outputs
    char *pool;
    void *X, *act_out, *gain;
    float *out, *part, *x, *ssq;
    int *counters;
    CK(hipMalloc(&pool, pool_bytes));
    CK(hipMemset(pool, 0x11, pool_bytes));
    CK(hipMalloc(&X, (size_t)Mp * F * 4));                     // packed hi/lo activations of the widest input
    CK(hipMemset(X, 0, (size_t)Mp * F * 4));
    CK(hipMalloc(&act_out, (size_t)Mp * F * 4));
    CK(hipMalloc(&out, (size_t)Mp * V * 4));
    CK(hipMalloc(&part, part_floats * 4));
    CK(hipMalloc(&x, (size_t)Mp * d * 4));
    CK(hipMemset(x, 0, (size_t)Mp * d * 4));
    CK(hipMalloc(&ssq, (size_t)Mp * 512 * 4));
    CK(hipMemset(ssq, 0, (size_t)Mp * 512 * 4));
    CK(hipMalloc(&counters, 4096 * 4));
    CK(hipMemset(counters, 0, 4096 * 4));
    CK(hipMalloc(&gain, (size_t)V * 2));
    CK(hipMemset(gain, 0, (size_t)V * 2));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));

    struct Proj { const char *name; int Nout, K, epi; };
    const Proj projs[] = {{"qkv", 3 * d, d, EPI_STORE}, {"o", d, d, EPI_RESID}, {"gu", 2 * F, d, EPI_SWIGLU},
                          {"down", d, F, EPI_RESID}, {"lm", V, d, EPI_STORE}};
    const int iters = 24;
    for (const Proj &s : projs) {
        GemmArgs a{};
        a.Xp = X; a.NT = s.Nout / 16; a.KT = s.K / 32; a.M = M;
        a.part = part; a.part_floats = part_floats; a.counters = counters; a.eps = 1e-5f;
        a.out = out; a.ld_out = s.Nout; a.ssq_in = ssq; a.NT_in = d / 16;
        a.x = x; a.gain = gain; a.act_out = (uint16_t *)act_out;
        a.KT_out = s.epi == EPI_SWIGLU ? F / 32 : d / 32; a.ssq = ssq;
        int pwn, pwk, ptn, psk, pwide;
        gemm_bf16_pick(a.NT, a.KT, s.epi, m_tiles, &pwn, &pwk, &ptn, &psk, &pwide);
        for (int wide : {0, 1})
            for (int tn : {1, 2, 4})
                for (int sk : {1, 2, 3, 4, 6})
                    for (auto sh : {std::pair<int, int>{8, 1}, {4, 2}, {2, 4}, {1, 8}, {4, 4}, {1, 16}, {3, 4}}) {
                        const int wn = sh.first, wk = sh.second;
                        const bool picked = wn == pwn && wk == pwk && tn == ptn && sk == psk && wide == pwide;
                        if (mode == 1 && !picked) continue;
                        if (mode == 2 && !wide && !picked) continue;
                        if (a.NT % tn || (s.epi == EPI_SWIGLU && tn < 2)) continue;
                        if ((size_t)sk * M * s.Nout > part_floats) continue;     // (the launcher would refuse it too)
                        // the combinations the launchers instantiate
                        const bool twelve = wn == 3 && wk == 4 && tn <= 2;
                        if (wide ? (m_tiles < 3 || (!twelve && (tn < 2 || wn * wk != 8 || wn > 4)))
                                 : (wn == 3 || (m_tiles <= 2 ? tn > 2 : (tn != 2 || wn * wk != 8 || wk > 4))))
                            continue;
                        a.SK = sk;
                        const size_t wbytes = (size_t)s.Nout * s.K * 2, nslots = pool_bytes / wbytes;
                        bool ok = true;
                        auto launch = [&](int i) {
                            a.Wp = pool + (i % nslots) * wbytes;
                            if (launch_gemm_bf16_cfg(a, s.epi, m_tiles, wn, wk, tn, wide, 0)) ok = false;
                        };
                        printf("[run] %s rows=%d %s %dx%d tn=%d sk=%d\n", s.name, M, wide ? "wide" : "base", wn, wk, tn, sk);
                        fflush(stdout);
                        launch(0);
                        if (!ok) continue;                                       // (shape not available: message printed)
                        for (int i = 1; i < 3; ++i) launch(i);
                        CK(hipDeviceSynchronize());
                        CK(hipEventRecord(e0));
                        for (int i = 0; i < iters; ++i) launch(i + 3);
                        CK(hipEventRecord(e1));
                        CK(hipEventSynchronize(e1));
                        float ms;
                        CK(hipEventElapsedTime(&ms, e0, e1));
                        printf("%-5s epi%d %s %2dx%-2d TN%d SK %d%s  %8.2f us  %7.1f GB/s\n", s.name, s.epi,
                               wide ? "wide" : "base", wn, wk, tn, sk, picked ? "*" : " ", ms * 1e3 / iters,
                               wbytes / (ms / iters * 1e-3) / 1e9);
                    }
    }
    return 0;
}
