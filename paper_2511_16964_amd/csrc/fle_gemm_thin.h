// The thin GEMM: at most 32 rows of x (a batch of one to a few tokens), bound by reading W once.
#pragma once
#include "fle_device_common.h"
#include "fle_gemm_general.h"

namespace fle {

// ------------------------------------------------------------------ thin GEMM (M <= 32, every dtype)
// The regime of a multi-layer perceptron at batch 1 .. 32: each layer reads its whole weight matrix for a
// handful of output rows, so the kernel is a stream over W and everything else is latency.  The skinny
// kernel's 128-row W tiles give such a layer too few workgroups (32 for N = 4096) and force a split of K
// with a second launch; here a workgroup owns only 16 rows of W and all of K, so N = 4096 already gives
// one workgroup per CU in a single launch, and larger N several.
//
// The 4 waves split K in steps of 64 bytes per row: wave w takes steps w, w + 4, ..., so together they read
// 256 contiguous bytes of each row at a time.  In a step a lane loads 16 bytes of its W row (row lane & 15,
// chunk lane >> 4) straight into the operand layout of the 16x16 MFMA (16x16x32 on bf16 / fp16: 8 k per
// lane; fp32: four 16x16x4 steps, step e taking element e of every lane's vector, the same k permutation
// for both operands) and the matching 16 bytes of x (rows beyond M and chunks beyond K come back as zeros
// from the buffer load).  No LDS staging: the bytes in flight are register batches of U steps, two batches
// deep (one being multiplied while the next is on its way).  W loads carry the non-temporal hint (read
// once); x is a few KB and stays in L2.  The partial tiles of the 4 waves are summed through LDS in a
// fixed order, then the 16 x 16 tile is finished exactly like a sub-tile of the general kernel.
template <int DT, int TM>
__global__ __launch_bounds__(256) void gemm_thin(const GemmArgs a) {
    constexpr bool F32 = DT == FLE_F32;
    constexpr int ES = F32 ? 4 : 2;
    constexpr int U = 8;  // steps per register batch
    __shared__ float red[4][TM][64][4];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r16 = lane & 15, q4 = lane >> 4;
    const int64_t M = a.M, N = a.N, K = a.K;
    const int64_t n0 = int64_t(blockIdx.x) * 16;
    const int dtype = DT;

    // epilogue coordinates (wave t < TM finishes the 16 rows 16 t ..); the bias is fetched now, behind the K loop
    f32x4 bias_v = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (a.epi.bias && wave < TM) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (n0 + 4 * q4 + e < N) bias_v[e] = ld_elem(a.epi.bias, n0 + 4 * q4 + e, dtype);
    }

    const int64_t wrows = (N - n0) < 16 ? (N - n0) : 16;
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char *>(reinterpret_cast<const char *>(a.w) + n0 * a.ldw * ES), 0, uint32_t(((wrows - 1) * a.ldw + K) * ES), 0x00020000);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.x), 0, uint32_t(((M - 1) * a.ldx + K) * ES), 0x00020000);
    const uint32_t kc = uint32_t(K * ES / 16);  // 16-byte chunks per row
    const uint32_t w_off = uint32_t(r16) * uint32_t(a.ldw) * ES + uint32_t(q4) * 16;
    uint32_t x_off[TM];
#pragma unroll
    for (int t = 0; t < TM; ++t) x_off[t] = uint32_t(16 * t + r16) * uint32_t(a.ldx) * ES + uint32_t(q4) * 16;

    using frag_t = typename std::conditional<F32, f32x4, typename std::conditional<DT == FLE_F16, f16x8, bf16x8>::type>::type;
    struct Batch {
        u32x4 w[U], x[TM][U];
    };
    // batch j of this wave: steps wave + 4 (j U + u), u = 0 .. U-1; a step past the end of the row loads zeros
    auto load = [&](Batch &b, uint32_t j) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t step = uint32_t(wave) + 4 * (j * U + u);
            const bool valid = 4 * step + uint32_t(q4) < kc;
            const uint32_t col = valid ? step * 64 : 0x80000000u;
            b.w[u] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, w_off + col, 0, 2));
#pragma unroll
            for (int t = 0; t < TM; ++t) b.x[t][u] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, x_off[t] + col, 0, 0));
        }
    };
    f32x4 acc[TM];
#pragma unroll
    for (int t = 0; t < TM; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    auto multiply = [&](const Batch &b) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const frag_t fw = __builtin_bit_cast(frag_t, b.w[u]);
#pragma unroll
            for (int t = 0; t < TM; ++t) {
                const frag_t fx = __builtin_bit_cast(frag_t, b.x[t][u]);
                if constexpr (F32) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(fw[e], fx[e], acc[t], 0, 0, 0);
                } else if constexpr (DT == FLE_F16) {
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw, fx, acc[t], 0, 0, 0);
                } else {
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw, fx, acc[t], 0, 0, 0);
                }
            }
        }
    };
    const uint32_t steps = (kc + 3) / 4;
    const uint32_t mine = steps > uint32_t(wave) ? (steps - uint32_t(wave) + 3) / 4 : 0;  // steps of this wave
    const uint32_t batches = (mine + U - 1) / U;
    Batch b0, b1;
    if (batches > 0) load(b0, 0);
    for (uint32_t j = 0; j < batches; j += 2) {
        load(b1, j + 1);  // past the last batch: zeros, no memory traffic
        multiply(b0);
        load(b0, j + 2);
        multiply(b1);
    }

#pragma unroll
    for (int t = 0; t < TM; ++t) *reinterpret_cast<f32x4 *>(&red[wave][t][lane][0]) = acc[t];
    __syncthreads();
    if (wave >= TM) return;
    f32x4 v = *reinterpret_cast<const f32x4 *>(&red[0][wave][lane][0]);
#pragma unroll
    for (int ww = 1; ww < 4; ++ww) v += *reinterpret_cast<const f32x4 *>(&red[ww][wave][lane][0]);
    finish_tile16(a, v, bias_v, int64_t(16 * wave + r16), n0, q4, dtype);
}

// ------------------------------------------------------------------ GEMV form (M <= 4; fp32: M <= 8)
// A batch of one to eight rows: the matrix pipe has nothing to gain (15 of 16 tile rows would be zeros) and
// its operand layout costs the stream its coalescing (consecutive lanes sit on consecutive W rows, so every
// lane's 16 bytes are a request of their own).  Here a W row is read the way it lies in memory: one load
// instruction of a wave covers 1024 contiguous bytes of one row (lane l takes bytes 16 l ..), and the lane
// multiplies its 16 bytes with the same 16 bytes of each x row (converted to fp32, then plain FMAs: 8 + 8 M
// vector instructions per 16 bytes of a 2-byte dtype, which keeps up with HBM to M = 4; fp32 operands need
// 4 M and go to M = 8), accumulating per (W row, x row) in fp32.  A wave owns R (4, 2 or 1) W rows and all of K and keeps D blocks of
// 1 KB per row in flight in registers (two register batches, one multiplied while the next arrives); the x
// block of a lane is loaded once per K block and reused by the wave's rows.  At the end each (W row, x row) sum
// is reduced over the 64 lanes by a butterfly (fixed order), the 16 x MR results of the workgroup meet in
// LDS, and wave 0 finishes them as one 16 x 16 tile like the general kernel.
// 16 bytes of a row as fp32 values (8 of a 2-byte dtype, else 4).
template <int DT>
struct Unpacked {
    float v[DT == FLE_F32 ? 4 : 8];
};
template <int DT>
__device__ __forceinline__ Unpacked<DT> unpack16(u32x4 r) {
    Unpacked<DT> o;
    if constexpr (DT == FLE_F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) o.v[e] = __uint_as_float(r[e]);
    } else if constexpr (DT == FLE_F16) {
        const f16x8 h = __builtin_bit_cast(f16x8, r);
#pragma unroll
        for (int e = 0; e < 8; ++e) o.v[e] = float(h[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o.v[2 * e] = __uint_as_float(r[e] << 16);
            o.v[2 * e + 1] = __uint_as_float(r[e] & 0xffff0000u);
        }
    }
    return o;
}

// MR: x rows held per lane (M <= MR).
// R: W rows per wave; the workgroup always owns 16 rows, so it has 16 / R waves.  R = 4 and 4 waves is the
// default; R = 1 and 16 waves (used for a single x row) keeps more loads in flight per CU.
// LNP: LayerNorm of the x rows over K in front of the multiplication, in the same sweep.  With
// xn_k = (x_k - mean) rstd gamma_k + beta_k the dot product is
//     sum_k w_k xn_k = rstd (S1 - mean S2) + S3,   S1 = sum_k (w_k gamma_k) x_k,  S2 = sum_k w_k gamma_k,  S3 = sum_k w_k beta_k,
// so every lane accumulates S1 per (W row, x row) as it does the plain products, S2 and S3 per W row, and the sum and
// sum of squares of its x values; mean and rstd come out of the same lane reduction as the dot products (every wave
// sees all of x).  One kernel and one pass over W where the unfused form launches a normalisation first: at one row
// of x, where the launch is a large part of the time, that is the point (the paper's perceptron tasks at batch 1,
// Appendix C).  The variance is E[x^2] - mean^2 in fp32, exact enough while |mean| is within a few hundred
// deviations; rows far off centre belong to the two-pass form in front of the other kernels.
template <int DT, int MR, int R, bool LNP = false>
__global__ __launch_bounds__(1024 / R) void gemm_gemv(const GemmArgs a) {
    constexpr int ES = DT == FLE_F32 ? 4 : 2;
    constexpr int NW = 16 / R;           // waves per workgroup
    constexpr int D = 2;                 // K blocks (1 KB of every row) per register batch (deeper batches gain nothing and cost occupancy)
    __shared__ float red[16][16];        // [W row of the workgroup][x row]
    __shared__ float part[NW][R * MR][65];  // per wave: [value][lane] (+1: the readers of different values hit different banks)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r16 = lane & 15, q4 = lane >> 4;
    const int64_t M = a.M, N = a.N, K = a.K;
    const int64_t n0 = int64_t(blockIdx.x) * 16, nw = n0 + R * wave;  // first W row of the workgroup / of this wave
    const int dtype = DT;

    f32x4 bias_v = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (a.epi.bias && wave == 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (n0 + 4 * q4 + e < N) bias_v[e] = ld_elem(a.epi.bias, n0 + 4 * q4 + e, dtype);
    }
    if (lane < 16) {  // x rows beyond MR (none are used) and W rows beyond N read as zero in the epilogue
#pragma unroll
        for (int r = 0; r < R; ++r) red[R * wave + r][lane] = 0.0f;
    }

    const int64_t wrows = N - nw < R ? N - nw : R;  // <= 0: this wave has no rows and loads nothing
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char *>(reinterpret_cast<const char *>(a.w) + (wrows > 0 ? nw : 0) * a.ldw * ES), 0,
        wrows > 0 ? uint32_t(((wrows - 1) * a.ldw + K) * ES) : 0u, 0x00020000);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.x), 0, uint32_t(((M - 1) * a.ldx + K) * ES), 0x00020000);
    const uint32_t kbytes = uint32_t(K * ES), ldwb = uint32_t(a.ldw) * ES, ldxb = uint32_t(a.ldx) * ES;

    struct Batch {
        u32x4 w[D][R], x[D][MR], g[LNP ? D : 1], be[LNP ? D : 1];
    };
    [[maybe_unused]] const __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.ln_gamma), 0, LNP && a.ln_gamma ? uint32_t(K * ES) : 0u, 0x00020000);
    [[maybe_unused]] const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.ln_beta), 0, LNP && a.ln_beta ? uint32_t(K * ES) : 0u, 0x00020000);
    // K blocks j D .. j D + D - 1; bytes past the end of the row, rows past N or M: zeros, no memory traffic
    auto load = [&](Batch &b, uint32_t j) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const uint32_t col = (j * D + d) * 1024 + uint32_t(lane) * 16;
            const uint32_t off = col < kbytes ? col : 0x80000000u;
#pragma unroll
            for (int m = 0; m < MR; ++m) b.x[d][m] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, uint32_t(m) * ldxb + off, 0, 0));
#pragma unroll
            for (int r = 0; r < R; ++r) b.w[d][r] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, uint32_t(r) * ldwb + off, 0, 2));
            if constexpr (LNP) {  // (a missing gamma / beta has an empty descriptor: its loads return zeros and cost nothing)
                b.g[d] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rg, off, 0, 0));
                b.be[d] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, off, 0, 0));
            }
        }
    };
    [[maybe_unused]] float s2[R], s3[R], xs[MR], xq[MR];  // LNP: S2, S3 per W row; sum and sum of squares per x row
    if constexpr (LNP) {
#pragma unroll
        for (int r = 0; r < R; ++r) s2[r] = s3[r] = 0.0f;
#pragma unroll
        for (int m = 0; m < MR; ++m) xs[m] = xq[m] = 0.0f;
    }
    [[maybe_unused]] const bool has_gamma = LNP && a.ln_gamma != nullptr;
    float acc[R][MR];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < MR; ++m) acc[r][m] = 0.0f;
    auto multiply = [&](const Batch &b) {
        constexpr int E = DT == FLE_F32 ? 4 : 8;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if constexpr (LNP) {
                const Unpacked<DT> g = unpack16<DT>(b.g[d]), be = unpack16<DT>(b.be[d]);
#pragma unroll
                for (int m = 0; m < MR; ++m) {
                    const Unpacked<DT> x = unpack16<DT>(b.x[d][m]);
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        xs[m] += x.v[e];
                        xq[m] = fmaf(x.v[e], x.v[e], xq[m]);
                    }
                }
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const Unpacked<DT> w = unpack16<DT>(b.w[d][r]);
                    float wg[E];
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        wg[e] = has_gamma ? w.v[e] * g.v[e] : w.v[e];
                        s2[r] += wg[e];
                        s3[r] = fmaf(w.v[e], be.v[e], s3[r]);
                    }
#pragma unroll
                    for (int m = 0; m < MR; ++m) {
                        const Unpacked<DT> x = unpack16<DT>(b.x[d][m]);
#pragma unroll
                        for (int e = 0; e < E; ++e) acc[r][m] = fmaf(wg[e], x.v[e], acc[r][m]);
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int m = 0; m < MR; ++m) {
                        // (the compiler hoists the conversions: x once per block, W once per row)
                        const Unpacked<DT> w = unpack16<DT>(b.w[d][r]), x = unpack16<DT>(b.x[d][m]);
#pragma unroll
                        for (int e = 0; e < E; ++e) acc[r][m] = fmaf(w.v[e], x.v[e], acc[r][m]);
                    }
            }
        }
    };
    const uint32_t blocks = (kbytes + 1023) / 1024, batches = (blocks + D - 1) / D;
    // The scheduling barriers keep the compiler from sinking a batch's loads down to their first use, which
    // would leave only one batch in flight.
    Batch b0, b1;
    load(b0, 0);
    for (uint32_t j = 0; j < batches; j += 2) {
        load(b1, j + 1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(b0);
        __builtin_amdgcn_sched_barrier(0);
        load(b0, j + 2);
        __builtin_amdgcn_sched_barrier(0);
        multiply(b1);
        __builtin_amdgcn_sched_barrier(0);
    }
    // Sum every (W row, x row) accumulator over the 64 lanes.  A butterfly per value would cost 6 cross-lane
    // exchanges each (up to 192 in all, several microseconds: more than a small layer takes), so the lanes'
    // partial sums are transposed through LDS instead: value v is summed by 64 / V lanes, each adding V of
    // the 64 partials in index order, and a short butterfly over those lanes finishes it.
    constexpr int V = R * MR, LPV = 64 / V;  // values per wave; lanes per value
    if constexpr (LNP) {
        // the statistics first, by butterflies (few values: 2 per x row and 2 per W row), then the dot products turn
        // into those of the normalised rows before they take the usual way
        float mean[MR], rstd[MR];
#pragma unroll
        for (int m = 0; m < MR; ++m) {
            float sx = xs[m], sq = xq[m];
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                sx += __shfl_xor(sx, d);
                sq += __shfl_xor(sq, d);
            }
            mean[m] = sx / float(K);
            const float var = sq / float(K) - mean[m] * mean[m];
            rstd[m] = rsqrtf((var > 0.0f ? var : 0.0f) + a.ln_eps);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float t2 = s2[r], t3 = s3[r];
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                t2 += __shfl_xor(t2, d);
                t3 += __shfl_xor(t3, d);
            }
            // per lane: rstd (S1_lane - mean S2 / 64) + S3 / 64 sums over the lanes to rstd (S1 - mean S2) + S3
#pragma unroll
            for (int m = 0; m < MR; ++m) acc[r][m] = rstd[m] * (acc[r][m] - mean[m] * t2 * (1.0f / 64.0f)) + t3 * (1.0f / 64.0f);
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < MR; ++m) part[wave][r * MR + m][lane] = acc[r][m];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // the wave's LDS writes are ordered before its reads below
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    {
        const int v = lane / LPV, sub = lane % LPV;
        float sum = 0.0f;
#pragma unroll
        for (int j = 0; j < V; ++j) sum += part[wave][v][sub + LPV * j];
#pragma unroll
        for (int d = 1; d < LPV; d <<= 1) sum += __shfl_xor(sum, d);
        if (sub == 0) red[R * wave + v / MR][v % MR] = sum;
    }
    __syncthreads();
    if (wave != 0) return;
    const f32x4 v = f32x4{red[4 * q4][r16], red[4 * q4 + 1][r16], red[4 * q4 + 2][r16], red[4 * q4 + 3][r16]};
    finish_tile16(a, v, bias_v, int64_t(r16), n0, q4, dtype);
}

}  // namespace fle
