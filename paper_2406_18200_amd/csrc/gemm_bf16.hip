// Weight-streaming skinny GEMM for the verify step:  Y[M][Nout] = X[M][K] . W[Nout][K]^T  with M <= 128
// token rows (N branches x gamma drafts), bf16 operands, fp32 accumulation on the MFMA units.
//
// These projections (QKV, O, gate/up, down, LM head) carry 85-98 % of the bytes of a verify step and
// each weight is used by M <= 128 rows only, so the kernel is HBM-bound: the design goal is that every
// wavefront streams its share of W exactly once with 1 KiB fully-coalesced loads and no LDS staging.
//   * W is repacked once at init into MFMA A-fragment order: tile (nt, kt) = 16 output features x 32
//     inputs = 1 KiB contiguous, lane l holding W[nt*16 + l%16][kt*32 + 8*(l/16) .. +8].  All k-tiles of
//     an n-tile are contiguous, so a wavefront's stream is one contiguous run.
//   * X (activations, tiny, L2-resident) is kept in the matching B-fragment order by its producer, as a
//     hi/lo pair of bf16 values per element (two MFMAs per weight fragment): the weights stay bf16 but the
//     activations keep ~16 significant bits, so their rounding does not pile up over 32-40 layers.
//   * v_mfma_f32_16x16x32_bf16 computes Y^T tiles: D[i = feature][j = token row].
//   * Split-K partial sums go to a [SK][Mpad][Nout] fp32 buffer that the next row kernel reduces in a
//     fixed order (deterministic; no atomics).
#include "seed_internal.h"
#include "device_utils.h"

namespace seedv {
namespace {

constexpr int kUnroll = 4;   // k-tiles in flight per wavefront and n-tile

template <int TM, int TN>
__global__ __launch_bounds__(256) void gemm_ws_kernel(const bf16x8 *__restrict__ Wp,
                                                      const bf16x8 *__restrict__ Xp,
                                                      float *__restrict__ out, int n_groups, int KT,
                                                      int SK, int kt_per_split, int m_rows_out,
                                                      int64_t split_stride, int ld_out) {
    const int lane = threadIdx.x & 63;
    const int wid = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= n_groups * SK) return;
    const int ng = wid / SK, sk = wid - ng * SK;
    const int k0 = sk * kt_per_split;
    const int k1 = min(KT, k0 + kt_per_split);

    f32x4 acc[TN][TM];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const bf16x8 *wbase = Wp + ((size_t)ng * TN * KT) * 64 + lane;
    const bf16x8 *xbase = Xp + lane;

    int kt = k0;
    for (; kt + kUnroll <= k1; kt += kUnroll) {
        bf16x8 a[kUnroll][TN], b[kUnroll][TM][2];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                a[u][tn] = __builtin_nontemporal_load(wbase + ((size_t)tn * KT + kt + u) * 64);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                b[u][tm][0] = xbase[((size_t)tm * KT + kt + u) * 128];
                b[u][tm][1] = xbase[((size_t)tm * KT + kt + u) * 128 + 64];
            }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][tn], b[u][tm][1], acc[tn][tm], 0, 0, 0);
                    acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][tn], b[u][tm][0], acc[tn][tm], 0, 0, 0);
                }
    }
    for (; kt < k1; ++kt) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            bf16x8 a = __builtin_nontemporal_load(wbase + ((size_t)tn * KT + kt) * 64);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const bf16x8 bh = xbase[((size_t)tm * KT + kt) * 128];
                const bf16x8 bl = xbase[((size_t)tm * KT + kt) * 128 + 64];
                acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl, acc[tn][tm], 0, 0, 0);
                acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh, acc[tn][tm], 0, 0, 0);
            }
        }
    }
    // D[i][j]: lane holds features 4*(lane/16)+0..3 of token row lane%16
    float *obase = out + (size_t)sk * split_stride;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int row = tm * 16 + (lane & 15);
        if (row >= m_rows_out) continue;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int col = (ng * TN + tn) * 16 + 4 * (lane >> 4);
            *reinterpret_cast<f32x4 *>(obase + (size_t)row * ld_out + col) = acc[tn][tm];
        }
    }
}

// Repack row-major W[n_rows][K] (bf16) into fragment tiles.  Destination tile index of source n-tile
// t is dst_tile0 + t * dst_tile_step (step 2 interleaves the gate and up projections tile by tile).
__global__ void pack_weight_kernel(const uint16_t *__restrict__ W, u32x4 *__restrict__ dst, int n_tiles,
                                   int K, int KT, int dst_tile0, int dst_tile_step) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one 16-byte fragment each
    const size_t total = (size_t)n_tiles * KT * 64;
    if (idx >= total) return;
    const int lane = idx & 63;
    const size_t tile = idx >> 6;
    const int kt = tile % KT;
    const int nt = tile / KT;
    const uint16_t *src = W + (size_t)(nt * 16 + (lane & 15)) * K + kt * 32 + 8 * (lane >> 4);
    const u32x4 v = *reinterpret_cast<const u32x4 *>(src);
    dst[(((size_t)(dst_tile0 + nt * dst_tile_step)) * KT + kt) * 64 + lane] = v;
}

template <int TM, int TN>
void launch_one(const void *Wp, const void *Xp, float *out, int NT, int KT, int SK, int m_rows_out,
                int64_t split_stride, int ld_out, hipStream_t st) {
    const int n_groups = NT / TN;
    const int kt_per_split = (KT + SK - 1) / SK;
    const int waves = n_groups * SK;
    hipLaunchKernelGGL((gemm_ws_kernel<TM, TN>), dim3((waves + 3) / 4), dim3(256), 0, st,
                       (const bf16x8 *)Wp, (const bf16x8 *)Xp, out, n_groups, KT, SK, kt_per_split,
                       m_rows_out, split_stride, ld_out);
}

}  // namespace

int gemm_bf16_pick_tn(int NT, int m_tiles) {
    // two n-tiles per wavefront once there are several m-tiles to reuse the activation fragments
    return (m_tiles >= 3 && NT % 2 == 0) ? 2 : 1;
}

int launch_gemm_bf16(const void *Wp, const void *Xp, float *out, int Nout, int K, int m_tiles, int SK,
                     int m_rows_out, int64_t split_stride, int ld_out, hipStream_t st) {
    const int NT = Nout / 16, KT = K / 32;
    const int TN = gemm_bf16_pick_tn(NT, m_tiles);
#define SEEDV_CASE(TMv)                                                                              \
    case TMv:                                                                                        \
        if (TN == 2) launch_one<TMv, 2>(Wp, Xp, out, NT, KT, SK, m_rows_out, split_stride, ld_out, st); \
        else launch_one<TMv, 1>(Wp, Xp, out, NT, KT, SK, m_rows_out, split_stride, ld_out, st);       \
        break;
    switch (m_tiles) {
        SEEDV_CASE(1) SEEDV_CASE(2) SEEDV_CASE(3) SEEDV_CASE(4) SEEDV_CASE(5) SEEDV_CASE(6) SEEDV_CASE(7)
        SEEDV_CASE(8)
        default:
            set_error("gemm: unsupported m_tiles %d", m_tiles);
            return SEED_E_CAPACITY;
    }
#undef SEEDV_CASE
    return hip_fail(hipGetLastError(), "gemm launch");
}

int launch_pack_weight(const void *W, void *dst, int n_rows, int K, int dst_tile0, int dst_tile_step,
                       hipStream_t st) {
    const int n_tiles = n_rows / 16, KT = K / 32;
    const size_t total = (size_t)n_tiles * KT * 64;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const uint16_t *)W, (u32x4 *)dst, n_tiles, K, KT, dst_tile0, dst_tile_step);
    return hip_fail(hipGetLastError(), "pack launch");
}

}  // namespace seedv
