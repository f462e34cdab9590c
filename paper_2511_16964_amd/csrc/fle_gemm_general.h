// The general GEMM: any shape and alignment, small tiles, in-block split of K.
#pragma once
#include "fle_device_common.h"

namespace fle {

// ------------------------------------------------------------------ general GEMM
// Block tile 32 x 32 (or 16 x 16) outputs; the 4 waves split K (wave w takes 16-wide k blocks w,
// w+4, ...), each computing the whole tile, then the partial tiles are summed through LDS in a
// fixed order.  A lane loads 4 consecutive k of its row.  fp32: four v_mfma_f32_16x16x4_f32 per k
// block, MFMA number e consuming element e of every lane's vector, i.e. the k order inside a block
// is permuted identically for both operands, which leaves the sum unchanged.  bf16: one
// v_mfma_f32_16x16x16_bf16 per k block on the raw values (its operand layout is exactly 4
// consecutive k per lane).
typedef __attribute__((ext_vector_type(4))) short s16x4;

// 4 consecutive k of one row: fp32 values, or the raw bit patterns of a 2-byte dtype (zeros outside the matrix).
template <bool BF16, bool VEC>
__device__ __forceinline__ auto load_k4(const void *base, int64_t ld, int64_t row, int64_t rows, int64_t k, int64_t K) {
    if constexpr (BF16) {
        s16x4 v = {0, 0, 0, 0};
        if (row >= rows) return v;
        const uint16_t *src = reinterpret_cast<const uint16_t *>(base) + row * ld + k;
        if (VEC) {
            if (k < K) v = *reinterpret_cast<const s16x4 *>(src);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k + e < K) v[e] = short(src[e]);
        }
        return v;
    } else {
        f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        if (row >= rows) return v;
        const float *src = reinterpret_cast<const float *>(base) + row * ld + k;
        if (VEC) {
            if (k < K) v = *reinterpret_cast<const f32x4 *>(src);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k + e < K) v[e] = src[e];
        }
        return v;
    }
}

// Finishes one 16 x 16 sub-tile held in the 16x16 MFMA result layout (a lane owns row m and columns
// nb + 4 q4 .. + 3 of the 16-column segment that starts at nb): the elementwise ops, the segment's
// row-reduction partial, the store.  Shared by the general and the thin kernel.
__device__ __forceinline__ void finish_tile16(const GemmArgs &a, f32x4 v, f32x4 bias_v, int64_t m, int64_t nb, int q4, int dtype) {
    const int64_t M = a.M, N = a.N;
    const int64_t n = nb + 4 * q4;
    for (int o = 0; o < a.epi.n_pre; ++o) {
        const DevOp op = a.epi.pre[o];
        if (op.kind == FLE_BIAS) {
            v += bias_v;
            continue;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (m < M && n + e < N) v[e] = apply_op(op, v[e], m, n + e, a.epi.bias, dtype);
    }
    if (a.epi.row_kind >= 0) {
        const int64_t left = N - nb;
        const float cnt = float(left < 16 ? (left > 0 ? left : 0) : 16);
        float s0, s1;
        if (a.epi.row_kind == FLE_LAYERNORM) {
            float sum = 0.0f;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (n + e < N) sum += v[e];
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            const float mean = cnt > 0.0f ? sum / cnt : 0.0f;
            float m2 = 0.0f;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (n + e < N) m2 += (v[e] - mean) * (v[e] - mean);
            m2 += __shfl_xor(m2, 16);
            m2 += __shfl_xor(m2, 32);
            s0 = mean;
            s1 = m2;
        } else {
            float mx = -INFINITY;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (n + e < N) mx = fmaxf(mx, v[e]);
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            float se = 0.0f;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (n + e < N) se += __expf(v[e] - mx);
            se += __shfl_xor(se, 16);
            se += __shfl_xor(se, 32);
            s0 = mx;
            s1 = se;
        }
        if (q4 == 0 && m < M && left > 0) {
            float *dstp = a.partials + (m * a.np + nb / 16) * 2;
            dstp[0] = s0;
            dstp[1] = s1;
        }
        if (a.dst_rel) v -= s0;
    }
    if (a.dst && m < M) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (n + e < N) st_elem(a.dst, m * a.ldd + n + e, a.dst_f32 ? FLE_F32 : dtype, v[e]);
    }
}

// T: 16 x 16 sub-tiles per side of the block tile (2: 32 x 32 outputs; 1: 16 x 16, for problems so small
// that 32 x 32 tiles would leave most CUs without a workgroup).
template <int DT, bool VEC, int T>
__global__ __launch_bounds__(256) void gemm_general(const GemmArgs a) {
    constexpr bool BF16 = DT != FLE_F32;  // 2-byte operands (bf16 or fp16): raw fragments, one 16x16x16 MFMA per k block
    constexpr int TS = 16 * T;
    __shared__ float red[4][T * T][64][4];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r16 = lane & 15, q4 = lane >> 4;
    const int64_t M = a.M, N = a.N, K = a.K;
    const int64_t tile_n = blockIdx.x % a.tiles_n, tile_m = blockIdx.x / a.tiles_n;
    const int64_t m0 = tile_m * TS, n0 = tile_n * TS;
    const int dtype = DT;
    // epilogue coordinates of this lane (wave t finishes sub-tile t = 2 i + j: row m, columns n .. n+3);
    // the bias is fetched now so that its latency hides behind the K loop (tiny problems are all latency)
    const int ti = T == 2 ? wave >> 1 : 0, tj = T == 2 ? wave & 1 : 0;  // waves beyond T * T leave after the sum
    const int64_t m = m0 + 16 * ti + r16;
    const int64_t nb = n0 + 16 * tj;        // first column of this wave's 16-column segment
    const int64_t n = nb + 4 * q4;
    f32x4 bias_v = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (a.epi.bias) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (n + e < N) bias_v[e] = ld_elem(a.epi.bias, n + e, dtype);
    }

    f32x4 acc[T][T];
#pragma unroll
    for (int i = 0; i < T; ++i)
#pragma unroll
        for (int j = 0; j < T; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // This wave's k blocks are wave, wave+4, ...; four of them are loaded at once (16 independent
    // vector loads in flight) before their MFMAs run, so small problems pay one memory latency, not four.
    const int64_t KB = (K + 15) / 16;
    constexpr int U = 4;
    for (int64_t kb0 = wave; kb0 < KB; kb0 += 4 * U) {
        using frag_t = typename std::conditional<BF16, s16x4, f32x4>::type;
        frag_t fw[U][T], fx[U][T];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t k = (kb0 + 4 * u) * 16 + 4 * q4;  // blocks past KB have k >= K and load zeros
#pragma unroll
            for (int t = 0; t < T; ++t) {
                fw[u][t] = load_k4<BF16, VEC>(a.w, a.ldw, n0 + 16 * t + r16, N, k, K);
                fx[u][t] = load_k4<BF16, VEC>(a.x, a.ldx, m0 + 16 * t + r16, M, k, K);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if constexpr (BF16) {  // one 16x16x16 bf16 step per k block: products of bf16 values are exact in fp32
#pragma unroll
                for (int i = 0; i < T; ++i)
#pragma unroll
                    for (int j = 0; j < T; ++j) {
                        if constexpr (DT == FLE_F16)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, fw[u][j]), __builtin_bit_cast(f16x4, fx[u][i]), acc[i][j], 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(fw[u][j], fx[u][i], acc[i][j], 0, 0, 0);
                    }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int i = 0; i < T; ++i)
#pragma unroll
                        for (int j = 0; j < T; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fw[u][j][e], fx[u][i][e], acc[i][j], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < T; ++i)
#pragma unroll
        for (int j = 0; j < T; ++j) *reinterpret_cast<f32x4 *>(&red[wave][i * T + j][lane][0]) = acc[i][j];
    __syncthreads();
    if (wave >= T * T) return;
    f32x4 v = *reinterpret_cast<const f32x4 *>(&red[0][wave][lane][0]);
#pragma unroll
    for (int ww = 1; ww < 4; ++ww) v += *reinterpret_cast<const f32x4 *>(&red[ww][wave][lane][0]);

    finish_tile16(a, v, bias_v, m, nb, q4, dtype);
}

}  // namespace fle
