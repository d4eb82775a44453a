// float32 plumbing path (dtype 0): straightforward kernels used for small fp32 models, where the
// point is exactness against the oracle rather than speed.  No MFMA: plain fp32 FMAs, wave reductions.
#include "seed_internal.h"
#include "device_utils.h"

namespace seedv {
namespace {

// Y[r][n] = sum_k X[r][k] * W[n][k];  one wavefront per output feature n, 8 rows at a time.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ W, const float *__restrict__ X,
                                                       float *__restrict__ Y, int M, int Nout, int K, int ldy) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (n >= Nout) return;
    const float *w = W + (size_t)n * K;
    for (int r0 = 0; r0 < M; r0 += 8) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        for (int k = lane; k < K; k += 64) {
            const float wv = w[k];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (r0 + i < M) acc[i] = fmaf(wv, X[(size_t)(r0 + i) * K + k], acc[i]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float v = wave_reduce_sum(acc[i]);
            if (lane == 0 && r0 + i < M) Y[(size_t)(r0 + i) * ldy + n] = v;
        }
    }
}

// One wavefront per (row, head): scores over the visible keys into LDS, softmax, weighted sum of V.
__global__ __launch_bounds__(64) void attn_f32_kernel(const float *__restrict__ q, const float *__restrict__ k_shared,
                                                      const float *__restrict__ v_shared,
                                                      const float *__restrict__ k_priv,
                                                      const float *__restrict__ v_priv,
                                                      const int32_t *private_len, float *__restrict__ out, int T,
                                                      int H, int dh, int S, int prefill_shared, int cap_s,
                                                      int cap_p, int max_private) {
    extern __shared__ float sc[];
    const int r = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int HD = H * dh;
    const int b = r / T, j = r - b * T;
    int n_shared, n_priv;
    if (prefill_shared) {
        n_shared = S + j + 1;
        n_priv = 0;
    } else {
        const int pl = min(max(private_len[b], 0), max_private);
        n_shared = S;
        n_priv = pl + j + 1;
    }
    const float *qv = q + (size_t)r * HD + h * dh;
    const float *ks = k_shared + (size_t)h * cap_s * dh;
    const float *vs = v_shared + (size_t)h * cap_s * dh;
    const float *kp = k_priv + ((size_t)b * H + h) * cap_p * dh;
    const float *vp = v_priv + ((size_t)b * H + h) * cap_p * dh;
    const int n = n_shared + n_priv;
    const float scale = 1.0f / sqrtf((float)dh);
    float mx = -INFINITY;
    for (int t = lane; t < n; t += 64) {
        const float *kr = t < n_shared ? ks + (size_t)t * dh : kp + (size_t)(t - n_shared) * dh;
        float s = 0.f;
        for (int i = 0; i < dh; ++i) s = fmaf(qv[i], kr[i], s);
        s *= scale;
        sc[t] = s;
        mx = fmaxf(mx, s);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float sum = 0.f;
    for (int t = lane; t < n; t += 64) {
        const float e = expf(sc[t] - mx);
        sc[t] = e;
        sum += e;
    }
    sum = wave_reduce_sum(sum);
    __syncthreads();
    const float inv = 1.0f / sum;
    for (int i = lane; i < dh; i += 64) {
        float acc = 0.f;
        for (int t = 0; t < n; ++t) {
            const float *vr = t < n_shared ? vs + (size_t)t * dh : vp + (size_t)(t - n_shared) * dh;
            acc = fmaf(sc[t], vr[i], acc);
        }
        out[(size_t)r * HD + h * dh + i] = acc * inv;
    }
}

}  // namespace

int launch_gemm_f32(const void *W, const void *X, float *Y, int M, int Nout, int K, int ldy, hipStream_t st) {
    hipLaunchKernelGGL(gemm_f32_kernel, dim3((Nout + 3) / 4), dim3(256), 0, st, (const float *)W, (const float *)X,
                       Y, M, Nout, K, ldy);
    return hip_fail(hipGetLastError(), "gemm_f32 launch");
}

int launch_attn_f32(const void *q, const void *k_shared, const void *v_shared, const void *k_priv,
                    const void *v_priv, const int32_t *private_len, float *out, int M, int T, int H, int dh, int S,
                    int prefill_shared, int cap_s, int cap_p, int max_private, hipStream_t st) {
    const size_t lds = (size_t)(cap_s + cap_p) * sizeof(float);
    hipLaunchKernelGGL(attn_f32_kernel, dim3(M, H), dim3(64), lds, st, (const float *)q, (const float *)k_shared,
                       (const float *)v_shared, (const float *)k_priv, (const float *)v_priv, private_len, out, T, H,
                       dh, S, prefill_shared, cap_s, cap_p, max_private);
    return hip_fail(hipGetLastError(), "attn_f32 launch");
}

}  // namespace seedv
