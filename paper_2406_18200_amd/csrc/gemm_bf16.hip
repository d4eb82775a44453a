// Weight-streaming skinny GEMM for the verify step:  Y[M][Nout] = X[M][K] . W[Nout][K]^T  with M <= 128
// token rows (N branches x gamma drafts), bf16 weights, fp32 accumulation on the MFMA units, with the
// row-wise work that follows each projection fused into its epilogue.
//
// These projections (QKV, O, gate/up, down, LM head) carry 85-98 % of the bytes of a verify step and each
// weight is used by M <= 128 rows only, so the kernel is HBM-bound.  Design:
//   * W is repacked once at init into MFMA A-fragment order: tile (nt, kt) = 16 output features x 32
//     inputs = 1 KiB contiguous, lane l holding W[nt*16 + l%16][kt*32 + 8*(l/16) .. +8]; all k-tiles of an
//     n-tile are contiguous.  Every wavefront streams its n-tile(s) with fully coalesced 1 KiB non-temporal
//     loads straight into registers, prefetched one group of k-tiles ahead; W never touches LDS.
//   * X (activations: tiny, L2-resident) is kept in the matching B-fragment order by its producer, as a
//     hi/lo pair of bf16 values per element (two MFMAs per weight fragment): the weights stay bf16 but the
//     activations keep ~16 significant bits, so their rounding does not pile up over 32-40 layers.
//     The 8 wavefronts of a workgroup own different n-tiles but the same k-range, and stage the X
//     fragments of that range through LDS in chunks, so each fragment crosses the L2->CU path once per
//     workgroup instead of once per wavefront (measured: that path, not HBM, was the limiter otherwise).
//   * v_mfma_f32_16x16x32_bf16 computes Y^T tiles: D[i = feature][j = token row].
//   * Split-K across workgroups (narrow outputs need it to fill 256 CUs): partial sums go to an fp32 buffer,
//     and the LAST workgroup to finish a column group (device-scope counter) re-reads all partials in a fixed
//     order (all its wavefronts, a share of the tiles each) and runs the epilogue, so results are deterministic
//     and no separate reduction kernel is needed.
//   * Epilogues: STORE (optional per-row scale = the RMSNorm factor of the input rows), RESID (residual add,
//     next RMSNorm's gain folded into the packed hi/lo activation, per-tile sums of squares of the new
//     residual rows), SWIGLU (gate and up tiles are interleaved in the packed weight so one wavefront holds
//     both; emits the packed activation of the down projection).  The RMSNorm factor 1/rms of the input rows
//     is applied AFTER the contraction: each consuming workgroup sums the producer's per-tile sums of squares
//     in a fixed order at its start, while its first weight loads are already in flight.
// Two kernel forms share the weight layout, the split-K exchange and the epilogues (finish_tiles):
// gemm_kernel (1..4 row tiles, and the narrow outputs at any row count) and gemm_wide_kernel (5..8 row tiles
// on outputs of 600 n-tiles and more; described where it is defined).  gemm_bf16_pick chooses form, workgroup
// shape and split from measurements on the 7B / 13B projection shapes.
#include <cstdlib>
#include <map>
#include <mutex>
#include <type_traits>
#include "seed_internal.h"
#include "device_utils.h"

namespace seedv {
namespace {

// Workgroup shapes: WN wavefronts side by side on different n-tile groups x WK wavefronts splitting every
// k-chunk of the same n-tiles (their partial tiles are summed through LDS at the end, in a fixed order).
//   wide outputs  (many n-tiles): WN large -> each activation fragment is shared by more wavefronts
//   narrow outputs (d_model wide): WK large -> enough wavefronts per n-tile to keep 256 CUs streaming
// U = k-tiles each wavefront prefetches per chunk; a chunk is WK * U k-tiles.
template <int TM, int TN, int WN, int WK>
struct Shape {
    static constexpr int kWaves = WN * WK;
    // k-tiles of staged activations (2 KiB per k-tile and row tile) that fit the LDS budget: 64 KiB for one or
    // two row tiles (and for three or four with WK <= 2, measured: two workgroups per CU pay there), 96 KiB above
    static constexpr int kBudget = (TM <= 2 || (WK <= 2 && TM <= 4)) ? 32 / TM : 48 / TM;
    static constexpr int kWant = TM <= 2 ? 4 : 2;                        // k-tiles per wavefront and group
    // largest U <= kWant that still lets two weight groups (prefetch depth 2) fit the staged chunk
    static constexpr int U = (2 * WK * kWant <= kBudget) ? kWant : ((2 * WK * 2 <= kBudget && kWant >= 2) ? 2 : 1);
    static constexpr int KC = WK * U;                                    // k-tiles per weight group
    static constexpr bool kValid = KC <= kBudget;
    // weight groups per staged activation chunk: fewer workgroup barriers per k-tile
    static constexpr int kFit = kBudget / KC;
    static constexpr int XG = kFit >= 8 ? 8 : (kFit >= 4 ? 4 : (kFit >= 2 ? 2 : 1));
    // weight groups (U k-tiles x TN tiles per wavefront) kept in flight: 2 (4 was measured no faster at 12 rows
    // and slower for the 4x2 shapes at 40 and 96).  When a chunk holds fewer groups than that, the k loop is
    // unrolled over OU chunks so that ring slots stay compile-time indices.
    static constexpr int D = 2;
    static constexpr int OU = D > XG ? D / XG : 1;
    // tiles summed per round of the cross-wavefront reduction (<= 64 KiB of LDS per round)
    static constexpr int kRedTiles = (64 / (WK * WN)) >= 1 ? (64 / (WK * WN)) : 1;
};

__device__ __forceinline__ void pin_args(const GemmArgs &a) {
    asm volatile("" ::"s"(a.Wp), "s"(a.Xp), "s"(a.NT), "s"(a.KT), "s"(a.kt_per_split), "s"(a.SK), "s"(a.M),
                 "s"(a.part), "s"(a.counters), "s"(a.out), "s"(a.ld_out), "s"(a.ssq_in), "s"(a.NT_in), "s"(a.x),
                 "s"(a.gain), "s"(a.act_out), "s"(a.KT_out), "s"(a.ssq), "s"(a.eps), "s"(a.MS), "s"(a.w_scale));
}

// 8-bit weights (context dtype SEED_DTYPE_BF16_W8): the same tiles with one byte per weight, an OCP e4m3 code
// (sign, 4 exponent bits of bias 7, 3 mantissa bits; no infinities), and one float scale per output feature:
// tile (nt, kt) is 512 bytes, lane l holding the 8 codes of W[nt*16 + l%16][kt*32 + 8*(l/16) .. +8].  Half the
// bytes cross HBM; on the way into the MFMA every code is widened to the bf16 of the same value (exact: three
// mantissa bits) with the hardware's packed fp8 -> float32 conversion, and the scale multiplies the fp32 sums once,
// after the k loop (before anything is exchanged or reduced: scaling is linear).
__device__ __forceinline__ bf16x8 widen_e4m3(u32x2 c) {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t src = (i < 2) ? c[0] : c[1];
        const auto f = (i & 1) ? __builtin_amdgcn_cvt_pk_f32_fp8(src, true) : __builtin_amdgcn_cvt_pk_f32_fp8(src, false);
        // the bf16 of a float32 that has at most four significant bits is its upper half
        r[i] = (__float_as_uint(f[0]) >> 16) | (__float_as_uint(f[1]) & 0xffff0000u);
    }
    return __builtin_bit_cast(bf16x8, r);
}

// 4-bit weights (context dtype SEED_DTYPE_BF16_W4): the OCP microscaling format MXFP4 -- elements are E2M1 codes
// (sign, two exponent bits, one mantissa bit: 0, 0.5, 1, 1.5, 2, 3, 4, 6), every 32 consecutive inputs of an output
// feature share a power-of-two scale stored as an E8M0 byte (2^(e - 127)).  A k-tile is exactly one such block per
// row: tile (nt, kt) is 256 bytes of codes, lane l holding the 8 codes of W[nt*16 + l%16][kt*32 + 8*(l/16) .. +8]
// (input k in the low nibble of byte k/2 for even k), plus 16 scale bytes in a separate array [nt][kt][16].
// On the way into the MFMA a code pair becomes a bf16 pair with the hardware's scaled conversion (exact: one
// mantissa bit times a power of two), so the kernel computes with exactly the values the codes stand for.
__device__ __forceinline__ bf16x8 widen_mxfp4(uint32_t c, uint32_t e8m0) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const float scale = __uint_as_float(e8m0 << 23);
    u32x4 r;
    const bf16x2_t p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(c, scale, 0);
    const bf16x2_t p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(c, scale, 1);
    const bf16x2_t p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(c, scale, 2);
    const bf16x2_t p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(c, scale, 3);
    r[0] = __builtin_bit_cast(uint32_t, p0);
    r[1] = __builtin_bit_cast(uint32_t, p1);
    r[2] = __builtin_bit_cast(uint32_t, p2);
    r[3] = __builtin_bit_cast(uint32_t, p3);
    return __builtin_bit_cast(bf16x8, r);
}

// Which column group and which share of the rows this workgroup works on.  With MS > 1 the rows of a step are
// split over MS workgroups per column group (TM row tiles each): every workgroup then stages and re-reads only
// its own rows' activations through LDS -- the saturated resource at 65..128 rows -- and takes MS times the columns
// instead.  The MS workgroups of a column group read the same weights; they are laid out so that they run on the
// SAME XCD at the same time (workgroups go to the eight XCDs round robin in launch order, so ids L and L + 8 are
// neighbours in time on one XCD): the second request finds the line in that XCD's L2 and HBM is still read once.
// The grid is rounded up to whole rounds of eight column groups; padding workgroups return at once.
__device__ __forceinline__ bool wg_coords(const GemmArgs &a, int tiles_per_wg, int &cg, int &mh) {
    cg = blockIdx.x;
    mh = 0;
    if (a.MS > 1) {
        const int L = blockIdx.x;
        mh = (L >> 3) % a.MS;
        cg = (L / (8 * a.MS)) * 8 + (L & 7);
    }
    return cg * tiles_per_wg < a.NT;
}

__device__ __forceinline__ void store_act4(uint16_t *act, int row, int col0, int KT, const float *v) {
    uint16_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) split_bf16(v[i], hi[i], lo[i]);
    uint16_t *dst = act + packed_offset(row, col0, KT);
    uint2 wh = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
    uint2 wl = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
    *reinterpret_cast<uint2 *>(dst) = wh;
    *reinterpret_cast<uint2 *>(dst + kActLoOffset) = wl;
}

// 1/rms of the input rows from the producer's per-tile sums of squares, summed in a fixed order: wavefront w
// takes rows w, w + kWaves, ...; a row of up to 512 sums is two 16-byte loads per lane, and the loads of eight
// rows are in flight together (row after row would pay a memory latency each: twelve of them at 96 rows).
template <int kWaves>
__device__ __forceinline__ void rows_rinv(const GemmArgs &a, float *s_rinv, int w, int lane, int r_lo, int r_hi) {
    // rows r_lo .. r_hi - 1 (this workgroup's share); s_rinv is indexed from r_lo
    constexpr int kRowsAtOnce = 8;
    const int nt_in = a.NT_in;
    if (nt_in <= 512 && (nt_in & 3) == 0) {
        for (int row0 = r_lo + w; row0 < r_hi; row0 += kRowsAtOnce * kWaves) {
            f32x4 v[kRowsAtOnce][2];
#pragma unroll
            for (int r = 0; r < kRowsAtOnce; ++r)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int row = min(row0 + r * kWaves, r_hi - 1), t = 4 * lane + 256 * i;
                    // (the load itself is unconditional, its value masked: a select on the value lets the compiler
                    // put the load under a branch, and a branch around a load drains the load queue at the join)
                    const u32x4 x = *reinterpret_cast<const u32x4 *>(a.ssq_in + (size_t)row * nt_in + (t < nt_in ? t : 0));
                    const uint32_t keep = t < nt_in ? 0xffffffffu : 0u;
                    v[r][i] = __builtin_bit_cast(f32x4, x & keep);
                }
#pragma unroll
            for (int r = 0; r < kRowsAtOnce; ++r) {
                const f32x4 q = v[r][0] + v[r][1];
                const float ssum = wave_reduce_sum_dpp((q[0] + q[1]) + (q[2] + q[3]));
                // (no branch: every lane writes the one value; a row past the end repeats the last row's)
                s_rinv[min(row0 + r * kWaves, r_hi - 1) - r_lo] = 1.0f / sqrtf(ssum / (float)(nt_in * 16) + a.eps);
            }
        }
    } else {
        for (int row = r_lo + w; row < r_hi; row += kWaves) {
            float ssum = 0.f;
            for (int t = lane; t < nt_in; t += 64) ssum += a.ssq_in[(size_t)row * nt_in + t];
            ssum = wave_reduce_sum(ssum);
            if (lane == 0) s_rinv[row - r_lo] = 1.0f / sqrtf(ssum / (float)(nt_in * 16) + a.eps);
        }
    }
}

// Everything after the k loop, shared by both kernel forms: 1/rms of the input rows (unless the prologue had
// it already), the cross-wavefront reduction of a workgroup's WK partial tiles, the split-K exchange between
// workgroups, and the epilogue.  `smem` is the k loop's staging memory, reused for the reduction.
template <int TM, int TN, int WN, int WK, int EPI, bool kPre>
__device__ __forceinline__ void finish_tiles(const GemmArgs &a, f32x4 (&acc)[TN][TM], char *smem, int *s_last_p,
                                             float *s_rinv, const f32x4 (&x_pre)[TN][TM], const uint2 (&gain_pre)[TN],
                                             bool ssq_early, int nt0, bool active, int cg, int mh) {
    using S = Shape<TM, TN, WN, WK>;
    constexpr int kWaves = S::kWaves;
    constexpr int RT = S::kRedTiles < TN * TM ? S::kRedTiles : TN * TM;   // tiles per reduction round
    f32x4(*red)[WN][RT][64] = reinterpret_cast<f32x4(*)[WN][RT][64]>(smem);                 // [WK][WN][RT][64]
    int &s_last = *s_last_p;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wn = w % WN, wk = w / WN;
    const int g = lane >> 4, rlow = lane & 15;
    const int nt_last = a.NT - 1;
    if (EPI != EPI_RESID && a.ssq_in != nullptr && !ssq_early) {
        // (after the k loop: a wait for these loads inside it would also wait for the weight prefetch)
        rows_rinv<kWaves>(a, s_rinv, w, lane, mh * TM * 16, min(a.M, (mh + 1) * TM * 16));
    }
    __syncthreads();                                      // s_rinv visible; xs no longer read

    if (WK > 1) {
        // sum the WK partial tiles of each n-tile group through LDS (fixed order), RT tiles per round;
        // wavefronts with wk == 0 end up holding the finished tiles
#pragma unroll
        for (int t0 = 0; t0 < TN * TM; t0 += RT) {
            __syncthreads();                              // xs / the previous round is no longer read
#pragma unroll
            for (int t = 0; t < RT; ++t)
                if (t0 + t < TN * TM) red[wk][wn][t][lane] = acc[(t0 + t) / TM][(t0 + t) % TM];
            __syncthreads();
            if (wk == 0) {
#pragma unroll
                for (int t = 0; t < RT; ++t)
                    if (t0 + t < TN * TM) {
                        f32x4 s = red[0][wn][t][lane];
#pragma unroll
                        for (int i = 1; i < WK; ++i) s += red[i][wn][t][lane];
                        acc[(t0 + t) / TM][(t0 + t) % TM] = s;
                    }
            }
        }
    }
    const bool owner = active && wk == 0;                 // this wavefront holds finished tiles
    const int bx_ = cg;
    const int rbase = mh * TM * 16;                       // first row of this workgroup's share

    // D[i][j]: lane holds features 4*(lane/16)+0..3 (columns) of token row lane%16
    const int ld_part = a.NT * 16;
    if (a.SK > 1) {
        // split-K across workgroups: publish the partial, then the last workgroup of this column group sums
        // all partials in a fixed order
        if (owner) {
            float *pb = a.part + (size_t)blockIdx.y * a.M * ld_part;   // (partials are indexed by global row)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int row = rbase + tm * 16 + rlow;
                if (row >= a.M) continue;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    if (nt0 + tn <= nt_last)
                        store4_agent(pb + (size_t)row * ld_part + (nt0 + tn) * 16 + 4 * g, acc[tn][tm]);
            }
        }
        if (!arrive_last(&a.counters[cg * a.MS + mh], a.SK, &s_last)) return;
        if constexpr (EPI != EPI_SWIGLU) {
            // Every wavefront of the last workgroup finishes a share of the workgroup's tiles: the partials lie
            // in global memory, so the wavefront that computed a tile need not be the one that sums it.  (With
            // only the wk == 0 wavefronts at it, two of eight, this tail of a 4-way split at 96 rows took 13 us
            // next to an 11 us k loop.)  Same order of summation as below: partial 0, 1, 2, ...
            constexpr int kTilesN = WN * TN;
            const size_t ps = (size_t)a.M * ld_part;
            const int wu = __builtin_amdgcn_readfirstlane(w);
            if (wu >= kWaves) return;
            // one tile's share of the epilogue, given the sum s of its partials (and, RESID, its residual rows
            // and the next norm's gains)
            auto finish_one = [&](int nt, int row, int col, bool valid, const f32x4 &s, const f32x4 &x_in, const uint2 &gw) {
                if (EPI == EPI_STORE) {
                    const float sc = (valid && a.ssq_in != nullptr) ? s_rinv[max(row - rbase, 0)] : 1.f;
                    if (valid) *reinterpret_cast<f32x4 *>(a.out + (size_t)row * a.ld_out + col) = s * sc;
                } else {
                    float ss = 0.f;
                    if (valid) {
                        const f32x4 xv = x_in + s;
                        *reinterpret_cast<f32x4 *>(a.x + (size_t)row * ld_part + col) = xv;
                        const float gv[4] = {bf2f((uint16_t)(gw.x & 0xffff)), bf2f((uint16_t)(gw.x >> 16)),
                                             bf2f((uint16_t)(gw.y & 0xffff)), bf2f((uint16_t)(gw.y >> 16))};
                        float v[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            ss += xv[i] * xv[i];
                            v[i] = xv[i] * gv[i];
                        }
                        store_act4(a.act_out, row, col, a.KT_out, v);
                    }
                    ss += __shfl_xor(ss, 16);
                    ss += __shfl_xor(ss, 32);
                    if (valid && g == 0) a.ssq[(size_t)row * a.NT + nt] = ss;
                }
            };
            constexpr int kTilesWG = kTilesN * TM;
            constexpr int kPerWave = (kTilesWG + kWaves - 1) / kWaves;
            constexpr int kBatchSK = 4;
            if (a.SK <= kBatchSK && kPerWave <= 4) {
                // Up to four partials of ALL of this wavefront's tiles are requested before the first is used: the
                // loads go around the L2 (a trip to memory each), and tile after tile would pay that latency
                // kPerWave times (three at 96 rows: most of a 9 us tail).  Straight-line code with clamped
                // addresses; what lies past the tile list or past SK is loaded again and dropped.
                f32x4 pv[kPerWave][kBatchSK], xin[kPerWave];
                uint2 gws[kPerWave];
                int nts[kPerWave], rows[kPerWave];
                bool oks[kPerWave];
#pragma unroll
                for (int q = 0; q < kPerWave; ++q) {
                    const int t = min(wu + q * kWaves, kTilesWG - 1);
                    const int tg = t / TM, tm = t - tg * TM;
                    const int nt = min(bx_ * kTilesN + tg, nt_last);
                    const int row = min(rbase + tm * 16 + rlow, a.M - 1), col = nt * 16 + 4 * g;
                    nts[q] = nt;
                    rows[q] = row;
                    oks[q] = wu + q * kWaves < kTilesWG && bx_ * kTilesN + tg <= nt_last && rbase + tm * 16 + rlow < a.M;
                    const float *pp = a.part + (size_t)row * ld_part + col;
#pragma unroll
                    for (int sk = 0; sk < kBatchSK; ++sk) pv[q][sk] = load4_agent(pp + (size_t)min(sk, a.SK - 1) * ps);
                    if (EPI == EPI_RESID) {
                        xin[q] = *reinterpret_cast<const f32x4 *>(a.x + (size_t)row * ld_part + col);
                        gws[q] = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(a.gain) + col);
                    }
                }
#pragma unroll
                for (int q = 0; q < kPerWave; ++q) {
                    f32x4 s = pv[q][0];                       // same order of summation as everywhere: 0, 1, 2, ...
#pragma unroll
                    for (int sk = 1; sk < kBatchSK; ++sk)
                        if (sk < a.SK) s += pv[q][sk];
                    if (wu + q * kWaves < kTilesWG && nts[q] == bx_ * kTilesN + min(wu + q * kWaves, kTilesWG - 1) / TM)
                        finish_one(nts[q], rows[q], nts[q] * 16 + 4 * g, oks[q], s, xin[q], gws[q]);
                }
                return;
            }
            for (int t = wu; t < kTilesN * TM; t += kWaves) {
                const int tg = t / TM, tm = t - tg * TM;
                const int nt = bx_ * kTilesN + tg;
                if (nt > nt_last) continue;                  // (uniform) ragged last column group
                const int row = rbase + tm * 16 + rlow, col = nt * 16 + 4 * g;
                const bool valid = row < a.M;
                f32x4 s = (f32x4){0.f, 0.f, 0.f, 0.f};
                f32x4 x_in = s;
                uint2 gw = {0u, 0u};
                if (valid) {
                    const float *pp = a.part + (size_t)row * ld_part + col;
                    int sk = 0;
                    for (; sk + 4 <= a.SK; sk += 4) {
                        const f32x4 p0 = load4_agent(pp + (sk + 0) * ps), p1 = load4_agent(pp + (sk + 1) * ps);
                        const f32x4 p2 = load4_agent(pp + (sk + 2) * ps), p3 = load4_agent(pp + (sk + 3) * ps);
                        s += p0;
                        s += p1;
                        s += p2;
                        s += p3;
                    }
                    for (; sk < a.SK; ++sk) s += load4_agent(pp + sk * ps);
                    if (EPI == EPI_RESID) {
                        x_in = *reinterpret_cast<const f32x4 *>(a.x + (size_t)row * ld_part + col);
                        gw = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(a.gain) + col);
                    }
                }
                finish_one(nt, row, col, valid, s, x_in, gw);
            }
            return;
        }
        if (owner) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int row = rbase + tm * 16 + rlow;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    f32x4 s = (f32x4){0.f, 0.f, 0.f, 0.f};
                    if (row < a.M && nt0 + tn <= nt_last) {
                        const float *pp = a.part + (size_t)row * ld_part + (nt0 + tn) * 16 + 4 * g;
                        const size_t ps = (size_t)a.M * ld_part;
                        int sk = 0;
                        for (; sk + 4 <= a.SK; sk += 4) {        // four loads in flight; summed in fixed order
                            const f32x4 p0 = load4_agent(pp + (sk + 0) * ps), p1 = load4_agent(pp + (sk + 1) * ps);
                            const f32x4 p2 = load4_agent(pp + (sk + 2) * ps), p3 = load4_agent(pp + (sk + 3) * ps);
                            s += p0;
                            s += p1;
                            s += p2;
                            s += p3;
                        }
                        for (; sk < a.SK; ++sk) s += load4_agent(pp + sk * ps);
                    }
                    acc[tn][tm] = s;
                }
            }
        }
    }

    if (!owner) return;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int row = rbase + tm * 16 + rlow;
        const bool valid = row < a.M;
        if (EPI == EPI_STORE) {
            const float sc = (valid && a.ssq_in != nullptr) ? s_rinv[row - rbase] : 1.f;
            if (valid) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    if (nt0 + tn <= nt_last)
                        *reinterpret_cast<f32x4 *>(a.out + (size_t)row * a.ld_out + (nt0 + tn) * 16 + 4 * g) = acc[tn][tm] * sc;
            }
        } else if (EPI == EPI_RESID) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int col = (nt0 + tn) * 16 + 4 * g;
                float ss = 0.f;
                const bool tile_ok = nt0 + tn <= nt_last;
                if (valid && tile_ok) {
                    float *xp2 = a.x + (size_t)row * ld_part + col;
                    f32x4 xv = (kPre ? x_pre[tn][tm] : *reinterpret_cast<f32x4 *>(xp2)) + acc[tn][tm];
                    *reinterpret_cast<f32x4 *>(xp2) = xv;
                    const uint2 gw = kPre ? gain_pre[tn]
                                          : *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(a.gain) + col);
                    const float gv[4] = {bf2f((uint16_t)(gw.x & 0xffff)), bf2f((uint16_t)(gw.x >> 16)),
                                         bf2f((uint16_t)(gw.y & 0xffff)), bf2f((uint16_t)(gw.y >> 16))};
                    float v[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        ss += xv[i] * xv[i];
                        v[i] = xv[i] * gv[i];
                    }
                    store_act4(a.act_out, row, col, a.KT_out, v);
                }
                ss += __shfl_xor(ss, 16);
                ss += __shfl_xor(ss, 32);
                if (valid && tile_ok && g == 0) a.ssq[(size_t)row * a.NT + nt0 + tn] = ss;
            }
        } else {   // EPI_SWIGLU: tiles (nt0 + 2p, nt0 + 2p + 1) = (gate, up) of feature block nt0 / 2 + p
            if (valid) {
                const float sc = s_rinv[row - rbase];
#pragma unroll
                for (int p = 0; p < TN / 2; ++p) {
                    if (nt0 + 2 * p + 1 > nt_last) continue;          // ragged last group: no such feature block
                    float h[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float gt = acc[2 * p][tm][i] * sc, up = acc[(2 * p + 1) % TN][tm][i] * sc;
                        h[i] = gt / (1.0f + expf(-gt)) * up;
                    }
                    store_act4(a.act_out, row, ((nt0 >> 1) + p) * 16 + 4 * g, a.KT_out, h);
                }
            }
        }
    }
}

template <int TM, int TN, int WN, int WK, int EPI, int WB>   // WB: bits per weight (16, 8 or 4)
__global__ __launch_bounds__(WN * WK * 64) void gemm_kernel(GemmArgs a) {
    using S = Shape<TM, TN, WN, WK>;
    constexpr int U = S::U, KC = S::KC, D = S::D, XG = S::XG, kWaves = S::kWaves;
    constexpr int XKT = XG * KC;                          // k-tiles per staged activation chunk
    constexpr int FR = XKT * TM * 2;                      // 1 KiB activation fragments per chunk
    constexpr int PER = (FR + kWaves - 1) / kWaves;       // fragments each wavefront copies
    constexpr int XS_BYTES = FR * 1024;
    constexpr int RT = S::kRedTiles < TN * TM ? S::kRedTiles : TN * TM;   // tiles per reduction round
    constexpr int RED_BYTES = (WK > 1) ? WK * WN * RT * 1024 : 16;
    __shared__ __attribute__((aligned(16))) char smem[XS_BYTES > RED_BYTES ? XS_BYTES : RED_BYTES];
    __shared__ int s_last;
    __shared__ float s_rinv[128];
    bf16x8(*xs)[TM][2][64] = reinterpret_cast<bf16x8(*)[TM][2][64]>(smem);                 // [XKT][TM][2][64]
    // All kernel arguments are fetched in ONE batch of scalar loads at the top: left alone, the compiler loads
    // each field just before its first use, and every such load is a round trip to memory (the argument
    // block is not in any cache when a launch starts) in front of the first weight request.
    pin_args(a);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wn = w % WN, wk = w / WN;
    int cg, mh;
    if (!wg_coords(a, WN * TN, cg, mh)) return;          // (uniform: a padding workgroup of a row-split launch)
    const int mt0 = mh * TM, mt_last = (a.M + 15) / 16 - 1;   // first row tile of this workgroup; last one there is
    const int nt0 = (cg * WN + wn) * TN;
    const bool active = nt0 < a.NT;
    const int KT = a.KT;
    const int k0 = blockIdx.y * a.kt_per_split, k1 = min(KT, k0 + a.kt_per_split);
    // every column group walks its k range from its own starting chunk (see gemm_wide_kernel): virtual k-tile
    // position v in [k0, k1) -> the k-tile actually read; only where the range is whole chunks
    const int krange = k1 - k0;
    const bool rot_ok = a.rot != 0 && krange > 0 && krange % (S::OU * XKT) == 0;
    const int rotk = rot_ok ? ((cg * a.rot) % (krange / XKT)) * XKT : 0;
    auto kmap = [&](int v) { return v < k1 ? (v + rotk >= k1 ? v + rotk - krange : v + rotk) : v; };

    f32x4 acc[TN][TM];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int nt_last = a.NT - 1;                        // a ragged last group re-reads the last tile (never stored)
    const bf16x8 *xp = reinterpret_cast<const bf16x8 *>(a.Xp);
    // The k loop is straight-line code (no data-dependent branches, clamped addresses), so that the compiler
    // keeps the prefetched registers live across iterations without copies and never has to wait for the
    // youngest loads: a ragged tail is handled by feeding ZERO activation fragments for k-tiles >= k1.
    bf16x8 xr[PER];
    auto load_x = [&](int kc0) {                          // chunk at k-tile kc0 -> registers
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int f = min(w + i * kWaves, FR - 1);    // fragment (k, tm, hi|lo) of the chunk
            const int k = f / (TM * 2), r = f - k * (TM * 2);
            xr[i] = xp[(((size_t)min(mt0 + (r >> 1), mt_last) * KT + min(kc0 + k, KT - 1)) * 2 + (r & 1)) * 64 + lane];
        }
    };
    auto store_x = [&](int kc0) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int f = w + i * kWaves;
            if (f < FR) {                                  // compile-time for all but the last i
                const int k = f / (TM * 2), r = f - k * (TM * 2);
                bf16x8 v = xr[i];
                if (kc0 + k >= k1) v = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
                xs[k][r >> 1][r & 1][lane] = v;
            }
        }
    };
    constexpr bool W8 = WB == 8, W4 = WB == 4;
    // a lane's piece of a weight tile: 8 bf16, 8 one-byte codes or 8 four-bit codes (with their block's scale)
    struct Frag4 { uint32_t c, e; };
    using WFrag = std::conditional_t<W4, Frag4, std::conditional_t<W8, u32x2, bf16x8>>;
    using WLoad = std::conditional_t<W4, uint32_t, std::conditional_t<W8, u32x2, bf16x8>>;
    const WLoad *wbase_f = reinterpret_cast<const WLoad *>(a.Wp) + lane;
    WFrag ring[D][U][TN];                                 // weight fragments in flight: D chunks ahead
    auto load_a = [&](WFrag (&dst)[U][TN], int k) {       // this wavefront's U k-tiles of the chunk at k
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const size_t tile = (size_t)min(nt0 + tn, nt_last) * KT + min(k + wk * U + u, KT - 1);
                if constexpr (W4) {
                    dst[u][tn].c = __builtin_nontemporal_load(wbase_f + tile * 64);
                    dst[u][tn].e = a.w_mx[tile * 16 + (lane & 15)];
                } else {
                    dst[u][tn] = __builtin_nontemporal_load(wbase_f + tile * 64);
                }
            }
    };
    // Prologue order: the first weight groups and the first activation chunk are requested at once; the
    // epilogue operands that do not depend on this launch follow (vector loads complete in order, so they are
    // back long before they are used and the tail of the kernel has no global load left to wait for): the
    // residual rows and the next norm's gain (RESID, small M), the input rows' sums of squares.  All of it is
    // straight-line code with clamped addresses: a branch around a load makes the compiler drain the whole
    // load queue where the paths join, which would hold back everything issued after it by a memory latency.
    load_x(kmap(k0));
#pragma unroll
    for (int dd = 0; dd < D; ++dd) load_a(ring[dd], kmap(k0 + dd * KC));
    constexpr bool kPre = EPI == EPI_RESID && TM <= 2;
    const int g = lane >> 4, rlow = lane & 15;
    f32x4 x_pre[TN][TM];
    uint2 gain_pre[TN];
    if (kPre) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int col = min(nt0 + tn, nt_last) * 16 + 4 * g;
            gain_pre[tn] = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(a.gain) + col);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int row = min(mt0 * 16 + tm * 16 + rlow, a.M - 1);
                x_pre[tn][tm] = *reinterpret_cast<const f32x4 *>(a.x + (size_t)row * (a.NT * 16) + col);
            }
        }
    }
    constexpr int kSsqRows = 2;                            // rows per wavefront handled by the early path
    constexpr int kSsqPer = 8;                             // and 64-wide slices of their sums of squares
    const bool ssq_early = EPI != EPI_RESID && a.ssq_in != nullptr && a.M <= kSsqRows * kWaves &&
                           a.NT_in <= 64 * kSsqPer;
    if (EPI != EPI_RESID) {
        // (without the early path the loads read the start of the activation buffer and are dropped)
        const float *sp = ssq_early ? a.ssq_in : reinterpret_cast<const float *>(a.Xp);
        const int nt_in = ssq_early ? a.NT_in : 1;
        float ssq_pre[kSsqRows][kSsqPer];
#pragma unroll
        for (int r = 0; r < kSsqRows; ++r)
#pragma unroll
            for (int i = 0; i < kSsqPer; ++i) {
                const int row = min(w + r * kWaves, a.M - 1), t = lane + 64 * i;
                const float v = sp[(size_t)row * nt_in + (t < nt_in ? t : 0)];
                ssq_pre[r][i] = t < nt_in ? v : 0.f;
            }
#pragma unroll
        for (int r = 0; r < kSsqRows; ++r) {
            float ssum = 0.f;
#pragma unroll
            for (int i = 0; i < kSsqPer; ++i) ssum += ssq_pre[r][i];       // same order as the late path
            ssum = wave_reduce_sum_dpp(ssum);
            const int row = w + r * kWaves;
            if (ssq_early && lane == 0 && row < a.M) s_rinv[row] = 1.0f / sqrtf(ssum / (float)(nt_in * 16) + a.eps);
        }
    }
    constexpr int OU = S::OU;
    const int n_outer = (k1 - k0 + OU * XKT - 1) / (OU * XKT);
    // one staged chunk: XG weight groups against the activations in LDS.  LAST (the final chunk of this
    // workgroup's k range, peeled below) requests nothing that would never be used: the loads would only be
    // waited for at the barrier after the loop.
    auto chunk = [&](int kx, int oc, auto last_tag) {
        constexpr bool LAST = decltype(last_tag)::value;
        lds_barrier();                                    // the previous chunk is no longer read
        store_x(kx);
        lds_barrier();
        if (!LAST) load_x(kmap(kx + XKT));
#pragma unroll
        for (int gq = 0; gq < XG; ++gq) {
            const int dd = (oc * XG + gq) % D;            // OU * XG is a multiple of D: the slot is static
            const int kc = kx + gq * KC;
            if (LAST && kc >= k1) break;                  // (uniform) the k range ends inside this chunk
#pragma unroll
            for (int u = 0; u < U; ++u) {
                bf16x8 bh[TM], bl[TM];
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    bh[tm] = xs[gq * KC + wk * U + u][tm][0][lane];
                    bl[tm] = xs[gq * KC + wk * U + u][tm][1][lane];
                }
                bf16x8 wa[TN];
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    if constexpr (W4) wa[tn] = widen_mxfp4(ring[dd][u][tn].c, ring[dd][u][tn].e);
                    else if constexpr (W8) wa[tn] = widen_e4m3(ring[dd][u][tn]);
                    else wa[tn] = ring[dd][u][tn];
                }
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[tn], bl[tm], acc[tn][tm], 0, 0, 0);
                        acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[tn], bh[tm], acc[tn][tm], 0, 0, 0);
                    }
            }
            if (!LAST || gq + D < XG) load_a(ring[dd], kmap(kc + D * KC));   // refill this slot D groups ahead (clamped)
        }
    };
    if constexpr (OU == 1) {
        for (int it = 0; it < n_outer - 1; ++it) chunk(k0 + it * XKT, 0, std::false_type{});
        if (n_outer > 0) chunk(k0 + (n_outer - 1) * XKT, 0, std::true_type{});
    } else {
        for (int it = 0; it < n_outer; ++it) {
#pragma unroll
            for (int oc = 0; oc < OU; ++oc) chunk(k0 + (it * OU + oc) * XKT, oc, std::false_type{});
        }
    }
    if constexpr (W8) {
        // one scale per output feature: lane (., g) holds features 4g .. 4g + 3 of each of its n-tiles
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const f32x4 sc = *reinterpret_cast<const f32x4 *>(a.w_scale + (size_t)min(nt0 + tn, nt_last) * 16 + 4 * g);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) acc[tn][tm] *= sc;
        }
    }
    finish_tiles<TM, TN, WN, WK, EPI, kPre>(a, acc, smem, &s_last, s_rinv, x_pre, gain_pre, ssq_early, nt0, active, cg, mh);
}

// ---------------------------------------------------------------------------------------------------------
// Form for three to eight row tiles (33..128 rows).  With that many rows a k-tile of activations is 6-16 KiB
// and every wavefront reads all of it for each of its n-tiles: what limits the kernel is no longer HBM alone
// but how many activation fragments a wavefront can have on their way from LDS while its MFMAs run, and how
// many registers are left for weights in flight.  Differences from the form above:
//   * the activation stages are filled by global -> LDS loads that bypass the registers (each lane's 16 bytes
//     land at the stage base + 16 * lane, which is the fragment order the MFMAs read); NS stages of one weight
//     group each, filled NS - 1 groups ahead, ONE workgroup barrier per group;
//   * one, two or four n-tiles per wavefront and workgroups of eight or twelve wavefronts (3 x 4: three per
//     SIMD, at most 168 registers), chosen so that a launch is one round of workgroups over most of the CUs;
//   * weights are addressed as a wavefront-uniform base in scalar registers plus one 32-bit lane offset per
//     n-tile: with 64-bit per-lane addresses the kernel spilled at six row tiles;
//   * the LDS reads are issued as one batch per k-tile and waited for fragment by fragment (inline assembly:
//     the compiler, which cannot see that a read does not touch the stage being filled, would otherwise wait
//     for the youngest global -> LDS load, and with it for every weight load issued before, ahead of each read).
// Counting rule the waits rely on: per group every wavefront issues exactly P stage loads, then U * TN weight
// loads, all unconditional with clamped addresses (the last round of groups issues no weight loads and counts
// accordingly); loads complete in issue order.  tests/test_isa_inflight.py replays the compiled ISA against
// these counts.
struct WideParams {
    int U, GK, stage_bytes, NS, F, P, D, wait_stage, wait_weights;
    bool valid;
};
constexpr WideParams wide_params(int TM, int TN, int WN, int WK) {
    WideParams p{};
    const int waves = WN * WK, budget = 144 * 1024;
    // k-tiles per wavefront and group: two where a k-tile is only a few MFMAs, if three stages still fit
    p.U = (TM * TN < 24 && 3 * (WK * 2 * TM * 2048) <= budget) ? 2 : 1;
    p.GK = WK * p.U;                                      // k-tiles per group = per LDS stage
    p.stage_bytes = p.GK * TM * 2048;
    const int fit = budget / p.stage_bytes;
    p.NS = fit > 4 ? 4 : fit;                             // stages
    p.F = p.GK * TM * 2;                                  // 1 KiB fragments per stage
    p.P = p.F / waves;                                    // stage loads per wavefront and group
    // weight groups in flight per wavefront: about 16 KiB, and no more than the stages are filled ahead (a
    // stage load completes only after the weight loads issued before it, so deeper rings gain nothing)
    const int want = 16 / (p.U * TN) < 2 ? 2 : 16 / (p.U * TN);
    p.D = want > p.NS - 1 ? p.NS - 1 : want;
    // loads a wavefront may still have in flight at the end of group g with the stage of group g + 1 complete
    p.wait_stage = (p.NS - 1) * p.U * TN + (p.NS - 2) * p.P;
    // ... and when group g starts its MFMAs, with the weights requested D groups ago complete: the stage loads
    // and weight loads of the D - 1 groups between, and this group's stage loads
    p.wait_weights = (p.D - 1) * (p.P + p.U * TN) + p.P;
    p.valid = p.NS >= 3 && p.F % waves == 0 && p.wait_stage < 64 && p.wait_weights < 64;   // (6-bit vmcnt)
    return p;
}
template <int TM, int TN, int WN, int WK>
struct WideShape {
    static constexpr WideParams p = wide_params(TM, TN, WN, WK);
    static constexpr int kWaves = WN * WK;
    static constexpr int U = p.U, GK = p.GK, kStageBytes = p.stage_bytes, NS = p.NS, F = p.F, P = p.P, D = p.D;
    static constexpr int kWaitStage = p.wait_stage, kWaitWeights = p.wait_weights;
    static constexpr bool kValid = p.valid;
};

// The loads of the k loop are issued and waited for by hand (inline assembly): with a global -> LDS load
// among the pending ones the compiler's own counting falls back to "wait for everything" ahead of every use.
// A register filled by such a load must not be touched before the matching wait; the waits take the
// registers as in/out operands, so that nothing that uses them can be scheduled ahead of the wait.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
template <int N, int TN>
__device__ __forceinline__ void wait_weights(bf16x8 (&wf)[TN]) {
    static_assert(N >= 0 && N < 64 && (TN == 1 || TN == 2 || TN == 4), "vmcnt is a 6-bit field");
    if constexpr (TN == 1) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(wf[0]) : "n"(N));
    else if constexpr (TN == 2) asm volatile("s_waitcnt vmcnt(%2)" : "+v"(wf[0]), "+v"(wf[1]) : "n"(N));
    else asm volatile("s_waitcnt vmcnt(%4)" : "+v"(wf[0]), "+v"(wf[1]), "+v"(wf[2]), "+v"(wf[3]) : "n"(N));
}
// (wavefront-uniform 64-bit base in scalar registers + a 32-bit byte offset per lane: one address register
// per load instead of two)
__device__ __forceinline__ void load_weight_nt(bf16x8 &dst, const void *base, unsigned offset) {
    asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(dst) : "v"(offset), "s"(base));
}

// All 2 * TM fragments of one k-tile (hi and lo of every row tile; 1 KiB apart) in one batch.
template <int TM>
__device__ __forceinline__ void lds_read_ktile(bf16x8 (&f)[2 * TM], unsigned addr) {
#pragma unroll
    for (int i = 0; i < 2 * TM; ++i)
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f[i]) : "v"(addr), "n"(i * 1024));
}
// Wait until at most N of the batch's reads are outstanding; the fragments named become usable.
template <int N>
__device__ __forceinline__ void lds_wait(bf16x8 &a, bf16x8 &b) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}

// The MFMAs of one k-tile, row tile by row tile: fragments 2 tm (hi) and 2 tm + 1 (lo) are waited for while the
// 2 TM - 2 tm - 2 reads issued after them may still be on their way.
template <int TM, int TN, int tm = 0>
struct KtileMfma {
    static __device__ __forceinline__ void run(bf16x8 (&f)[2 * TM], const bf16x8 (&wf)[TN], f32x4 (&acc)[TN][TM]) {
        lds_wait<2 * TM - 2 * tm - 2>(f[2 * tm], f[2 * tm + 1]);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[tn], f[2 * tm + 1], acc[tn][tm], 0, 0, 0);
            acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[tn], f[2 * tm], acc[tn][tm], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);                // keep wait -> MFMAs -> next wait in this order
        if constexpr (tm + 1 < TM) KtileMfma<TM, TN, tm + 1>::run(f, wf, acc);
    }
};

template <int TM, int TN, int WN, int WK, int EPI>
__global__ __launch_bounds__(WN * WK * 64) void gemm_wide_kernel(GemmArgs a) {
    using S = WideShape<TM, TN, WN, WK>;
    using S0 = Shape<TM, TN, WN, WK>;
    constexpr int U = S::U, GK = S::GK, NS = S::NS, D = S::D, P = S::P, kWaves = S::kWaves;
    constexpr int kStage = S::kStageBytes;
    constexpr int RT = S0::kRedTiles < TN * TM ? S0::kRedTiles : TN * TM;
    constexpr int RED_BYTES = (WK > 1) ? WK * WN * RT * 1024 : 16;
    constexpr int XS_BYTES = NS * kStage;
    static_assert(2 * TM * 1024 <= 65536, "ds_read offsets are 16-bit");
    __shared__ __attribute__((aligned(1024))) char smem[XS_BYTES > RED_BYTES ? XS_BYTES : RED_BYTES];
    __shared__ int s_last;
    __shared__ float s_rinv[128];
    pin_args(a);
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (scalar: addresses below stay in SGPRs)
    const int wn = w % WN, wk = w / WN;
    int cg, mh;
    if (!wg_coords(a, WN * TN, cg, mh)) return;          // (uniform: a padding workgroup of a row-split launch)
    const int mt0 = mh * TM, mt_last = (a.M + 15) / 16 - 1;   // first row tile of this workgroup; last one there is
    const int nt0 = (cg * WN + wn) * TN;
    const bool active = nt0 < a.NT;
    const int KT = a.KT;
    const int k0 = blockIdx.y * a.kt_per_split, k1 = min(KT, k0 + a.kt_per_split);
    const int n_groups = (k1 - k0 + GK - 1) / GK;
    // Every column group walks the k range from its own starting group: the workgroups of a launch start together
    // and run in step (a barrier per group), so without this all of them read the same k position at the same
    // time -- and the weights of different n-tiles at one k position lie KT KiB apart, i.e. on few memory
    // channels.  Measured at 96 rows on the 7B shapes: QKV 34.4 -> 32.5 us, gate/up 52.6 -> 50.8, LM head 71 -> 66
    // (any odd multiplier does the same).  The sums come out in another order per column group, still a fixed
    // one.  Only where the range is whole groups (no ragged tail to meet in mid-walk).
    const bool rot_ok = a.rot != 0 && (k1 - k0) % GK == 0 && n_groups > 1;
    const int rot = rot_ok ? (cg * a.rot) % n_groups : 0;
    auto kgroup = [&](int g) { return g < n_groups ? (g + rot >= n_groups ? g + rot - n_groups : g + rot) : g; };

    f32x4 acc[TN][TM];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int nt_last = a.NT - 1;
    unsigned woff[TN];                                   // byte offset of this lane's piece of k-tile 0 of each n-tile
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) woff[tn] = ((unsigned)min(nt0 + tn, nt_last) * (unsigned)KT * 64u + lane) * 16u;
    const bf16x8 *xp = reinterpret_cast<const bf16x8 *>(a.Xp) + lane;
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char *)smem;   // LDS byte address

    // stage load of group g: fragment f = w + i * kWaves of the stage, f = (kk * TM + tm) * 2 + hl; k-tiles past
    // the end of the matrix are clamped (their MFMAs are skipped)
    auto stage_load = [&](int g) {
        const unsigned base = (unsigned)((g % NS) * kStage);
#pragma unroll
        for (int i = 0; i < P; ++i) {
            const int f = w + i * kWaves;
            const int kk = f / (2 * TM), r = f - kk * (2 * TM);
            const int kt = min(k0 + kgroup(g) * GK + kk, KT - 1);
            const bf16x8 *src = xp + (((size_t)min(mt0 + (r >> 1), mt_last) * KT + kt) * 2 + (r & 1)) * 64;
            __builtin_amdgcn_global_load_lds(src, (__attribute__((address_space(3))) void *)(smem + base + f * 1024), 16,
                                             0, 0);
        }
    };
    bf16x8 ring[D][U][TN];
    auto load_a = [&](bf16x8 (&dst)[U][TN], int g) {     // this wavefront's k-tiles of group g (clamped)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const char *base = reinterpret_cast<const char *>(a.Wp) + (size_t)min(k0 + kgroup(g) * GK + wk * U + u, k1 - 1) * 1024;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) load_weight_nt(dst[u][tn], base, woff[tn]);
        }
    };
    // prologue: the first NS - 1 stages and D weight groups, everything waited for once
#pragma unroll
    for (int g = 0; g < NS - 1; ++g) stage_load(g);
#pragma unroll
    for (int dd = 0; dd < D; ++dd) load_a(ring[dd], dd);
    // the input rows' 1/rms while the first weights are on their way (its loads come back after them, so the
    // wait inside is the prologue's wait)
    if (EPI != EPI_RESID && a.ssq_in != nullptr) rows_rinv<kWaves>(a, s_rinv, w, lane, mt0 * 16, min(a.M, (mt0 + TM) * 16));
#pragma unroll
    for (int dd = 0; dd < D; ++dd)
#pragma unroll
        for (int u = 0; u < U; ++u) wait_weights<0, TN>(ring[dd][u]);
    wait_vmcnt<0>();
    lds_barrier();

    // One group.  DD = its ring slot.  TAIL = it belongs to the last round, which requests no further weights
    // (a register that a load is still going to write must stay reserved until a wait covers that load: the
    // result of a load nobody uses would be handed to other values at once) and where the k range may end
    // inside the group; its waits count the loads that the groups before it really issued.
    auto group = [&](int g, auto dd_tag, auto tail_tag) {
        constexpr int DD = decltype(dd_tag)::value;
        constexpr bool TAIL = decltype(tail_tag)::value;
        // loads issued after the weights of this group, which were requested at the end of group g - D
        constexpr int kWaitW = TAIL ? (D - 1 - DD) * (P + U * TN) + (DD + 1) * P : S::kWaitWeights;
        // loads issued after the stage loads of group g + 1 (start of group g + 2 - NS): the weight loads of
        // those of the groups g + 2 - NS .. g that are not in the last round, the stage loads of the later ones
        constexpr int kTailWeightGroups = NS - 2 - DD > 0 ? NS - 2 - DD : 0;
        constexpr int kWaitS = TAIL ? kTailWeightGroups * U * TN + (NS - 2) * P : S::kWaitStage;
        stage_load(g + NS - 1);                           // into the stage group g - 1 was read from
        __builtin_amdgcn_sched_barrier(0);
        const unsigned sbase = lds0 + (unsigned)((g % NS) * kStage) + lane * 16;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kk = wk * U + u;
            wait_weights<kWaitW, TN>(ring[DD][u]);        // (also in a skipped k-tile: the registers stay reserved)
            if (TAIL && k0 + g * GK + kk >= k1) continue; // (uniform)
            bf16x8 f[2 * TM];
            lds_read_ktile<TM>(f, sbase + (unsigned)(kk * TM * 2048));
            KtileMfma<TM, TN>::run(f, ring[DD][u], acc);
        }
        if constexpr (!TAIL) load_a(ring[DD], g + D);     // refill this slot D groups ahead
        wait_vmcnt<kWaitS>();                             // the stage of group g + 1 is complete (this wavefront's part)
        lds_barrier();                                    // ... everybody's part; stage g % NS is free again
    };
    // groups in rounds of D (ring slots are compile-time indices); the last round is peeled
    const int n_rounds = (n_groups + D - 1) / D;
    auto round = [&](int r, auto tail_tag) {
        const int g0 = r * D;
        constexpr bool TAIL = decltype(tail_tag)::value;  // only the last round can be incomplete
        group(g0, std::integral_constant<int, 0>{}, tail_tag);
        if constexpr (D > 1) {
            if (!TAIL || g0 + 1 < n_groups) {
                group(g0 + 1, std::integral_constant<int, 1>{}, tail_tag);
                if constexpr (D > 2) {
                    if (!TAIL || g0 + 2 < n_groups) {
                        group(g0 + 2, std::integral_constant<int, 2>{}, tail_tag);
                        if constexpr (D > 3) {
                            if (!TAIL || g0 + 3 < n_groups) group(g0 + 3, std::integral_constant<int, 3>{}, tail_tag);
                        }
                    }
                }
            }
        }
        static_assert(D <= 4, "rounds are written out for up to four ring slots");
    };
    for (int r = 0; r < n_rounds - 1; ++r) round(r, std::false_type{});
    if (n_rounds > 0) round(n_rounds - 1, std::true_type{});
    // Everything still in flight lands before the registers and the staging memory get other uses: weights
    // requested for groups past the end of the k range (the ring is named, so it stays reserved up to here)
    // and stage loads past the last group.
#pragma unroll
    for (int dd = 0; dd < D; ++dd)
#pragma unroll
        for (int u = 0; u < U; ++u) wait_weights<0, TN>(ring[dd][u]);
    wait_vmcnt<0>();
    f32x4 x_pre[TN][TM];
    uint2 gain_pre[TN];
    finish_tiles<TM, TN, WN, WK, EPI, false>(a, acc, smem, &s_last, s_rinv, x_pre, gain_pre, /*ssq_early=*/true, nt0, active, cg, mh);
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

// The same repacking for one-byte weights: row-major codes [n_rows][K] into 512-byte tiles, and the per-row
// scales into the order of the packed tiles.
__global__ void pack_weight8_kernel(const uint8_t *__restrict__ W, uint2 *__restrict__ dst, int n_tiles, int K, int KT,
                                    int dst_tile0, int dst_tile_step) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one 8-byte fragment each
    const size_t total = (size_t)n_tiles * KT * 64;
    if (idx >= total) return;
    const int lane = idx & 63;
    const size_t tile = idx >> 6;
    const int kt = tile % KT;
    const int nt = tile / KT;
    const uint8_t *src = W + (size_t)(nt * 16 + (lane & 15)) * K + kt * 32 + 8 * (lane >> 4);
    dst[(((size_t)(dst_tile0 + nt * dst_tile_step)) * KT + kt) * 64 + lane] = *reinterpret_cast<const uint2 *>(src);
}
__global__ void pack_scale_kernel(const float *__restrict__ src, float *__restrict__ dst, int n_rows, int dst_tile0,
                                  int dst_tile_step) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < n_rows) dst[(size_t)(dst_tile0 + (r >> 4) * dst_tile_step) * 16 + (r & 15)] = src[r];
}

// ... and for four-bit weights: row-major codes [n_rows][K/2] into 256-byte tiles, the E8M0 block scales
// [n_rows][K/32] into [n-tile][k-tile][16].
__global__ void pack_weight4_kernel(const uint8_t *__restrict__ W, uint32_t *__restrict__ dst, int n_tiles, int K, int KT,
                                    int dst_tile0, int dst_tile_step) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one 4-byte fragment each
    const size_t total = (size_t)n_tiles * KT * 64;
    if (idx >= total) return;
    const int lane = idx & 63;
    const size_t tile = idx >> 6;
    const int kt = tile % KT;
    const int nt = tile / KT;
    const uint8_t *src = W + ((size_t)(nt * 16 + (lane & 15)) * K + kt * 32 + 8 * (lane >> 4)) / 2;
    dst[(((size_t)(dst_tile0 + nt * dst_tile_step)) * KT + kt) * 64 + lane] = *reinterpret_cast<const uint32_t *>(src);
}
__global__ void pack_mx_scale_kernel(const uint8_t *__restrict__ src, uint8_t *__restrict__ dst, int n_rows, int KT,
                                     int dst_tile0, int dst_tile_step) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one (row, k-tile) each
    if (idx >= (size_t)n_rows * KT) return;
    const int r = idx / KT, kt = idx % KT;
    dst[((size_t)(dst_tile0 + (r >> 4) * dst_tile_step) * KT + kt) * 16 + (r & 15)] = src[idx];
}

template <int TM, int TN, int WN, int WK>
int launch_shape(const GemmArgs &a, int epi, hipStream_t st) {
    using S = Shape<TM, TN, WN, WK>;
    if constexpr (!S::kValid) {
        set_error("gemm: workgroup shape %dx%d does not fit %d row tiles", WN, WK, TM);
        return SEED_E_CAPACITY;
    } else {
        // splits are as even as k-tiles allow (a ragged last chunk stops at the first group past its range);
        // only the unrolled-rounds form (a chunk smaller than the weight ring) needs whole rounds
        constexpr int KC = S::OU > 1 ? S::OU * S::XG * S::KC : 1;
        GemmArgs b = a;
        b.kt_per_split = ((a.KT + a.SK - 1) / a.SK + KC - 1) / KC * KC;
        b.SK = (a.KT + b.kt_per_split - 1) / b.kt_per_split;
        if (b.SK > 1 && (size_t)b.SK * a.M * a.NT * 16 > a.part_floats) {
            set_error("gemm: %d-way split of %d x %d outputs exceeds the partial buffer (%zu floats)", b.SK, a.M,
                      a.NT * 16, a.part_floats);
            return SEED_E_CAPACITY;
        }
        const int groups = (a.NT + WN * TN - 1) / (WN * TN);
        if (b.MS < 1) b.MS = 1;
        dim3 grid(b.MS > 1 ? (groups + 7) / 8 * 8 * b.MS : groups, b.SK), block(WN * WK * 64);
        const int wb = b.w_mx != nullptr ? 4 : (b.w_scale != nullptr ? 8 : 16);
#define SEEDV_LAUNCH(EPIv)                                                                                  \
        do {                                                                                                \
            if (wb == 4) hipLaunchKernelGGL((gemm_kernel<TM, TN, WN, WK, EPIv, 4>), grid, block, 0, st, b);      \
            else if (wb == 8) hipLaunchKernelGGL((gemm_kernel<TM, TN, WN, WK, EPIv, 8>), grid, block, 0, st, b); \
            else hipLaunchKernelGGL((gemm_kernel<TM, TN, WN, WK, EPIv, 16>), grid, block, 0, st, b);             \
        } while (0)
        if (epi == EPI_SWIGLU) {
            if constexpr (TN >= 2) {
                SEEDV_LAUNCH(EPI_SWIGLU);
            } else { set_error("gemm: SwiGLU epilogue needs paired tiles"); return SEED_E_INVALID_ARG; }
        } else if (epi == EPI_RESID) {
            SEEDV_LAUNCH(EPI_RESID);
        } else {
            SEEDV_LAUNCH(EPI_STORE);
        }
#undef SEEDV_LAUNCH
        return hip_fail(hipGetLastError(), "gemm launch");
    }
}

// The wide form counts its own loads; a kernel that the compiler gave spill code (scratch loads and stores
// are loads in that count too) must not run.  Checked once per kernel.
int wide_kernel_usable(const void *kernel) {
    static std::mutex mu;
    static std::map<const void *, int> seen;
    std::lock_guard<std::mutex> lock(mu);
    auto it = seen.find(kernel);
    if (it == seen.end()) {
        hipFuncAttributes fa{};
        const int rc = hip_fail(hipFuncGetAttributes(&fa, kernel), "hipFuncGetAttributes");
        if (rc) return rc;
        it = seen.emplace(kernel, (int)fa.localSizeBytes).first;
    }
    if (it->second != 0) {
        set_error("gemm: this wide kernel was compiled with %d bytes of scratch per lane and is not used", it->second);
        return SEED_E_UNSUPPORTED_DTYPE;
    }
    return SEED_OK;
}

template <int TM, int TN, int WN, int WK>
int launch_wide_shape(const GemmArgs &a, int epi, hipStream_t st) {
    using S = WideShape<TM, TN, WN, WK>;
    if constexpr (!S::kValid) {
        set_error("gemm: the wide form has no %dx%d workgroup with %d n-tiles for %d row tiles", WN, WK, TN, TM);
        return SEED_E_CAPACITY;
    } else {
        GemmArgs b = a;
        b.kt_per_split = (a.KT + a.SK - 1) / a.SK;
        b.SK = (a.KT + b.kt_per_split - 1) / b.kt_per_split;
        if (b.SK > 1 && (size_t)b.SK * a.M * a.NT * 16 > a.part_floats) {
            set_error("gemm: %d-way split of %d x %d outputs exceeds the partial buffer (%zu floats)", b.SK, a.M,
                      a.NT * 16, a.part_floats);
            return SEED_E_CAPACITY;
        }
        if (a.w_scale != nullptr || a.w_mx != nullptr) { set_error("gemm: the wide form streams bf16 weights only"); return SEED_E_UNSUPPORTED_DTYPE; }
        if ((size_t)a.NT * a.KT * 1024 >= ((size_t)1 << 32)) {
            set_error("gemm: the wide form addresses weights with 32-bit offsets (matrix of %d x %d tiles)", a.NT, a.KT);
            return SEED_E_CAPACITY;
        }
        const int groups = (a.NT + WN * TN - 1) / (WN * TN);
        if (b.MS < 1) b.MS = 1;
        dim3 grid(b.MS > 1 ? (groups + 7) / 8 * 8 * b.MS : groups, b.SK), block(WN * WK * 64);
        int rc;
        if (epi == EPI_SWIGLU) {
            if constexpr (TN >= 2) {
                if ((rc = wide_kernel_usable((const void *)gemm_wide_kernel<TM, TN, WN, WK, EPI_SWIGLU>))) return rc;
                hipLaunchKernelGGL((gemm_wide_kernel<TM, TN, WN, WK, EPI_SWIGLU>), grid, block, 0, st, b);
            } else {
                set_error("gemm: the SwiGLU epilogue needs paired tiles");
                return SEED_E_INVALID_ARG;
            }
        } else if (epi == EPI_RESID) {
            if ((rc = wide_kernel_usable((const void *)gemm_wide_kernel<TM, TN, WN, WK, EPI_RESID>))) return rc;
            hipLaunchKernelGGL((gemm_wide_kernel<TM, TN, WN, WK, EPI_RESID>), grid, block, 0, st, b);
        } else {
            if ((rc = wide_kernel_usable((const void *)gemm_wide_kernel<TM, TN, WN, WK, EPI_STORE>))) return rc;
            hipLaunchKernelGGL((gemm_wide_kernel<TM, TN, WN, WK, EPI_STORE>), grid, block, 0, st, b);
        }
        return hip_fail(hipGetLastError(), "gemm launch");
    }
}

// Three to eight row tiles in the wide form: two or four n-tiles per wavefront.
template <int TM>
int launch_wide(const GemmArgs &a, int epi, int wn, int wk, int tn, hipStream_t st) {
#define SEEDV_SHAPE(WNv, WKv)                                                             \
    if (wn == WNv && wk == WKv)                                                           \
        return tn == 4 ? launch_wide_shape<TM, 4, WNv, WKv>(a, epi, st) : launch_wide_shape<TM, 2, WNv, WKv>(a, epi, st);
    if (tn == 2 || tn == 4) {
        SEEDV_SHAPE(4, 2) SEEDV_SHAPE(2, 4) SEEDV_SHAPE(1, 8)
    }
#undef SEEDV_SHAPE
    // twelve wavefronts, six n-tiles per workgroup: 1376 n-tiles (7B gate/up) become 230 workgroups instead of 172
    if (tn == 2 && wn == 3 && wk == 4) return launch_wide_shape<TM, 2, 3, 4>(a, epi, st);
    // ... twelve n-tiles per workgroup: the shape of the row-split launches (half the rows, twice the columns)
    if constexpr (TM <= 4) {
        if (tn == 4 && wn == 3 && wk == 4) return launch_wide_shape<TM, 4, 3, 4>(a, epi, st);
    }
    // ... and three n-tiles per workgroup, one per wavefront: 768 n-tiles (7B QKV) become 256 workgroups
    if (tn == 1 && wn == 3 && wk == 4 && epi != EPI_SWIGLU) return launch_wide_shape<TM, 1, 3, 4>(a, epi, st);
    set_error("gemm: unsupported wide workgroup shape %dx%d with %d n-tiles", wn, wk, tn);
    return SEED_E_INVALID_ARG;
}

// One or two row tiles (<= 32 rows): one or two n-tiles per wavefront, all workgroup shapes.
template <int TM>
int launch_small(const GemmArgs &a, int epi, int wn, int wk, int tn, hipStream_t st) {
#define SEEDV_SHAPE(WNv, WKv)                                                             \
    if (wn == WNv && wk == WKv)                                                           \
        return tn == 2 ? launch_shape<TM, 2, WNv, WKv>(a, epi, st) : launch_shape<TM, 1, WNv, WKv>(a, epi, st);
    SEEDV_SHAPE(8, 1) SEEDV_SHAPE(4, 2) SEEDV_SHAPE(2, 4) SEEDV_SHAPE(1, 8) SEEDV_SHAPE(4, 4) SEEDV_SHAPE(1, 16)
#undef SEEDV_SHAPE
    set_error("gemm: unsupported workgroup shape %dx%d", wn, wk);
    return SEED_E_INVALID_ARG;
}

// Three to eight row tiles: two n-tiles per wavefront (every activation fragment read from LDS feeds two
// MFMAs), fewer shapes.  (Four tiles per wavefront were measured slower at 40 and 96 rows.)
template <int TM>
int launch_large(const GemmArgs &a, int epi, int wn, int wk, int tn, hipStream_t st) {
    if (tn != 2) {
        set_error("gemm: %d row tiles run with two n-tiles per wavefront", TM);
        return SEED_E_INVALID_ARG;
    }
#define SEEDV_SHAPE(WNv, WKv)                                                             \
    if (wn == WNv && wk == WKv) return launch_shape<TM, 2, WNv, WKv>(a, epi, st);
    SEEDV_SHAPE(8, 1) SEEDV_SHAPE(4, 2) SEEDV_SHAPE(2, 4)
#undef SEEDV_SHAPE
    set_error("gemm: unsupported workgroup shape %dx%d for %d row tiles", wn, wk, TM);
    return SEED_E_INVALID_ARG;
}

}  // namespace

// Launch with an explicit workgroup shape (wn x wk wavefronts, tn n-tiles per wavefront) and a.SK
// workgroups along K.
int launch_gemm_bf16_cfg(const GemmArgs &a, int epi, int m_tiles, int wn, int wk, int tn, int wide, hipStream_t st) {
    if (a.MS > 1) m_tiles = (m_tiles + a.MS - 1) / a.MS;          // row tiles per workgroup of a row-split launch
    if (epi == EPI_SWIGLU && (tn < 2 || a.NT % 2 != 0)) {
        set_error("gemm: the SwiGLU epilogue needs paired tiles (tn=%d, NT=%d)", tn, a.NT);
        return SEED_E_INVALID_ARG;
    }
    if (wide) {
        switch (m_tiles) {
            case 3: return launch_wide<3>(a, epi, wn, wk, tn, st);
            case 4: return launch_wide<4>(a, epi, wn, wk, tn, st);
            case 5: return launch_wide<5>(a, epi, wn, wk, tn, st);
            case 6: return launch_wide<6>(a, epi, wn, wk, tn, st);
            case 7: return launch_wide<7>(a, epi, wn, wk, tn, st);
            case 8: return launch_wide<8>(a, epi, wn, wk, tn, st);
            default:
                set_error("gemm: the wide form runs three to eight row tiles, not %d", m_tiles);
                return SEED_E_INVALID_ARG;
        }
    }
    switch (m_tiles) {
        case 1: return launch_small<1>(a, epi, wn, wk, tn, st);
        case 2: return launch_small<2>(a, epi, wn, wk, tn, st);
        case 3: return launch_large<3>(a, epi, wn, wk, tn, st);
        case 4: return launch_large<4>(a, epi, wn, wk, tn, st);
        case 5: return launch_large<5>(a, epi, wn, wk, tn, st);
        case 6: return launch_large<6>(a, epi, wn, wk, tn, st);
        case 7: return launch_large<7>(a, epi, wn, wk, tn, st);
        case 8: return launch_large<8>(a, epi, wn, wk, tn, st);
        default:
            set_error("gemm: unsupported m_tiles %d", m_tiles);
            return SEED_E_CAPACITY;
    }
}

// Workgroup shape and split from sweeps on MI355X over the 7B / 13B projection shapes at 12, 24, 40 and 96
// rows: wide outputs share activation fragments across wavefronts (WN); narrow outputs split K inside the
// workgroup (WK), over all eight wavefronts when that gives one workgroup per CU without a split across
// workgroups (no partials to exchange), else over four with two workgroups along K.
// Multiplier of the per-column-group rotation of the k walk (see gemm_wide_kernel); 0 switches it off.
constexpr int kRotation = 3;
// Row-split launches (65..128 rows): can be switched off for A/B measurements with SEED_GEMM_ROW_SPLIT=0.
void gemm_bf16_pick_share(int NT, int KT, int epi, int m_tiles, int *wn, int *wk, int *tn, int *sk, int *wide, int *ms,
                          int w8);
static bool row_split_enabled() {
    static const bool on = [] {
        const char *e = getenv("SEED_GEMM_ROW_SPLIT");
        return e == nullptr || e[0] != '0';
    }();
    return on;
}

void gemm_bf16_pick(int NT, int KT, int epi, int m_tiles, int *wn, int *wk, int *tn, int *sk, int *wide, int *ms,
                    int w8) {
    *sk = 1;
    *wide = 0;
    *ms = 1;
    if (m_tiles > 8) {
        // More than 128 rows: blocks of at most six row tiles, each run in the shape (and with the row shares)
        // picked for a step of that many rows; no split of K (the shares alone are several workgroups per CU).
        // All shares of a column group run on one XCD at about the same time (see wg_coords), so the weights
        // still come from memory once.
        if (NT % 4 == 0 && KT >= 64 && !w8) {
            // Past 128 rows the launch is bound by MFMA issue and LDS reads, not by memory, so the big register
            // tiles of the wide form: up to eight row tiles x four n-tiles per wavefront (a weight fragment feeds
            // up to 16 MFMAs, an activation fragment read from LDS four); 4 x 2 wavefronts for wide outputs, 2 x 4
            // (eight n-tiles per workgroup, K split four ways inside it) for narrow ones.  One such workgroup
            // fills a CU, so the launch runs in whole rounds of 256: the row tiles per workgroup are chosen for
            // the least rounds x (tiles + 2) (the 2: what a workgroup costs besides its MFMAs, in tiles).
            // Measured at the 7B shapes, 384 rows: gate/up 166 us (three-tile shares of the 96-row shape) -> 147,
            // QKV 109 -> 76.
            const int swn = NT >= 600 ? 4 : 2, swk = 8 / swn;
            const int groups = ((NT + 4 * swn - 1) / (4 * swn) + 7) / 8 * 8;
            int best_tm = 0, best_cost = 1 << 30;
            for (int t : {8, 6, 5, 4, 3}) {
                const int shares = (m_tiles + t - 1) / t, tm = (m_tiles + shares - 1) / shares;   // tm <= t
                if (tm < 3 || !wide_params(tm, 4, swn, swk).valid) continue;
                const int cost = ((groups * shares + 255) / 256) * (tm + 2);
                if (cost < best_cost) { best_cost = cost; best_tm = tm; }
            }
            if (best_tm > 0) {
                *wn = swn; *wk = swk; *tn = 4; *wide = 1; *ms = (m_tiles + best_tm - 1) / best_tm;
                return;
            }
        }
        const int blocks = (m_tiles + 5) / 6;
        int sk1, ms1;
        gemm_bf16_pick_share(NT, KT, epi, (m_tiles + blocks - 1) / blocks, wn, wk, tn, &sk1, wide, &ms1, w8);
        *ms = blocks * ms1;
        return;
    }
    gemm_bf16_pick_share(NT, KT, epi, m_tiles, wn, wk, tn, sk, wide, ms, w8);
}

// (at most eight row tiles; splits them into two shares itself where that was measured faster)
void gemm_bf16_pick_share(int NT, int KT, int epi, int m_tiles, int *wn, int *wk, int *tn, int *sk, int *wide, int *ms,
                          int w8) {
    *sk = 1;
    *wide = 0;
    *ms = 1;
    if (w8) {
        // one-byte weights run in the first form only (with row shares from five row tiles on)
        *tn = (m_tiles > 2 || epi == EPI_SWIGLU || (NT >= 1300 && NT % 2 == 0)) ? 2 : 1;
        if (m_tiles >= 5) *ms = 2;
        const int units = NT / *tn;
        if (m_tiles <= 2 && units >= 600) { *wn = 4; *wk = 2; }
        else if (m_tiles == 1 && NT <= 256) { *wn = 1; *wk = 8; }
        else if (m_tiles > 2 && NT >= 1300) { *wn = 4; *wk = 2; }
        else {
            *wn = 2; *wk = 4;
            if (NT < 600) {
                const int groups = (NT + *tn * 2 - 1) / (*tn * 2) * *ms;
                const int fill = (256 + groups / 2) / groups;
                *sk = fill < 1 ? 1 : (fill > 4 ? 4 : fill);
                if (m_tiles <= 2) *sk = NT <= 256 ? 2 : 1;
            }
        }
        if (KT < 64) *sk = 1;
        return;
    }
    if (m_tiles >= 5 && row_split_enabled()) {
        // Two workgroups per column group, three or four row tiles each (see wg_coords).
        const int tm = (m_tiles + 1) / 2;
        if (NT >= 600) {
            // wide outputs: twelve wavefronts (3 x 4); as few n-tiles per wavefront as keep the launch within one
            // round of workgroups (7B QKV: 2 -> 128 column groups x 2; 7B gate/up: 4 -> 115 x 2)
            for (int t : {2, 4}) {
                const int groups = ((NT + 3 * t - 1) / (3 * t) + 7) / 8 * 8;
                if (groups * 2 <= 256 && wide_params(tm, t, 3, 4).valid && NT % t == 0) {
                    *wn = 3; *wk = 4; *tn = t; *wide = 1; *ms = 2;
                    return;
                }
            }
        } else if (KT >= 64) {
            // narrow outputs: 2 x 4 wavefronts, four n-tiles per workgroup, and a split of K that brings the
            // launch to about one workgroup per CU (7B O / down: 64 column groups x 2 row shares x 2)
            const int groups = ((NT + 3) / 4 + 7) / 8 * 8;
            int fill = (256 + groups) / (2 * groups);
            fill = fill < 1 ? 1 : (fill > 4 ? 4 : fill);
            *wn = 2; *wk = 4; *tn = 2; *sk = fill; *ms = 2;
            return;
        }
    }
    if (m_tiles <= 2) {
        *tn = (epi == EPI_SWIGLU || (NT >= 1300 && NT % 2 == 0)) ? 2 : 1;
        const int units = NT / *tn;                        // n-tile groups a wavefront owns one of
        if (units >= 600) { *wn = 4; *wk = 2; }
        else if (m_tiles == 1 && NT <= 256) { *wn = 1; *wk = 8; }
        else { *wn = 2; *wk = 4; *sk = NT <= 256 ? 2 : 1; }
    } else {
        *tn = 2;
        if (NT >= 1300) { *wn = 4; *wk = 2; }
        else if (NT >= 600) { *wn = 2; *wk = 4; }
        else {
            // narrow outputs: as many workgroups along k as bring the launch closest to one per CU
            *wn = 2; *wk = 4;
            const int groups = (NT + 3) / 4;
            const int fill = (256 + groups / 2) / groups;
            *sk = fill < 1 ? 1 : (fill > 4 ? 4 : fill);
        }
        // The wide outputs run in the form that stages activations with global -> LDS loads: from five row tiles
        // on always; from three on where a twelve-wavefront shape fits the output (measured at 40 rows on the 7B
        // shapes: gate/up 42 -> 38 us, QKV 32 -> 29.5 us; elsewhere the first form is as fast or faster there).
        if (NT >= 600) {
            const bool five = m_tiles >= 5;
            if (five && !wide_params(m_tiles, *tn, *wn, *wk).valid) { *wn = 4; *wk = 2; }   // (seven, eight row tiles)
            if (*wn == 4 && (NT + 5) / 6 <= 256 && (NT + 7) / 8 < 200 && wide_params(m_tiles, 2, 3, 4).valid) {
                // six n-tiles per workgroup where that still is one round of workgroups and eight would leave a
                // quarter of the CUs idle: 7B gate/up, 1376 n-tiles, 230 workgroups instead of 172
                *wn = 3; *wk = 4; *wide = 1;
            } else if (*wn == 2 && epi != EPI_SWIGLU && (NT + 2) / 3 <= 256 && (NT + 3) / 4 < 200 &&
                       wide_params(m_tiles, 1, 3, 4).valid) {
                // three (one per wavefront) for the mid-width outputs: 7B QKV, 768 n-tiles, 256 workgroups
                // instead of 192
                *wn = 3; *wk = 4; *tn = 1; *wide = 1;
            } else if (five) {
                *wide = wide_params(m_tiles, *tn, *wn, *wk).valid;
            }
        }
    }
    if (KT < 64) *sk = 1;
}

int launch_gemm_bf16(GemmArgs a, int epi, int m_tiles, hipStream_t st) {
    int wn, wk, tn, sk, wide, ms;
    gemm_bf16_pick(a.NT, a.KT, epi, m_tiles, &wn, &wk, &tn, &sk, &wide, &ms, a.w_scale != nullptr || a.w_mx != nullptr);
    a.MS = ms;
    // (only while the whole activation matrix -- hi and lo halves of every row -- stays in an XCD's 4 MiB L2 next to
    // the weight stream: workgroups at different k positions read different parts of it; at 384 rows and more
    // the rotation cost the narrow outputs 25-45 %)
    a.rot = (size_t)m_tiles * 16 * a.KT * 32 * 4 <= ((size_t)2 << 20) ? kRotation : 0;
    if (a.SK < 1) a.SK = sk;
    return launch_gemm_bf16_cfg(a, epi, m_tiles, wn, wk, tn, wide, st);
}

int launch_pack_weight8(const void *codes, const float *scale, void *dst, float *scale_dst, int n_rows, int K,
                        int dst_tile0, int dst_tile_step, hipStream_t st) {
    const int n_tiles = n_rows / 16, KT = K / 32;
    const size_t total = (size_t)n_tiles * KT * 64;
    hipLaunchKernelGGL(pack_weight8_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const uint8_t *)codes, (uint2 *)dst, n_tiles, K, KT, dst_tile0, dst_tile_step);
    hipLaunchKernelGGL(pack_scale_kernel, dim3((n_rows + 255) / 256), dim3(256), 0, st, scale, scale_dst, n_rows,
                       dst_tile0, dst_tile_step);
    return hip_fail(hipGetLastError(), "pack launch");
}

int launch_pack_weight4(const void *codes, const void *mx_scale, void *dst, void *scale_dst, int n_rows, int K,
                        int dst_tile0, int dst_tile_step, hipStream_t st) {
    const int n_tiles = n_rows / 16, KT = K / 32;
    const size_t total = (size_t)n_tiles * KT * 64;
    hipLaunchKernelGGL(pack_weight4_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const uint8_t *)codes, (uint32_t *)dst, n_tiles, K, KT, dst_tile0, dst_tile_step);
    hipLaunchKernelGGL(pack_mx_scale_kernel, dim3((unsigned)(((size_t)n_rows * KT + 255) / 256)), dim3(256), 0, st,
                       (const uint8_t *)mx_scale, (uint8_t *)scale_dst, n_rows, KT, dst_tile0, dst_tile_step);
    return hip_fail(hipGetLastError(), "pack launch");
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
