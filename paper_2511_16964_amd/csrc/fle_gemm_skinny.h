// The HBM-bound skinny GEMM (row blocks of 32 rows; 2-byte operands also 64 .. 256).
#pragma once
#include "fle_device_common.h"

namespace fle {

// ------------------------------------------------------------------ skinny GEMM (row blocks of 32; bf16 / fp16 up to 256 rows)
// HBM-bound: W streams through once and the matrix pipe is nearly idle, so the design goal is
// bytes in flight.  One workgroup owns 128 rows of W (columns of out) and all of K; each of its
// 4 waves copies and consumes its own 32 W rows, the small x tile is shared.  The LDS ring is
// NST stages of (128 + 32 TMB) x BK elements, NST-1 of them in flight; measured, the length of
// the contiguous run per W row (2 BK bytes) matters more than the ring depth, and the W loads
// carry the non-temporal hint (W is read once and must not displace anything in L2 or the
// Infinity Cache).  Same swizzle and orientation as the tiled kernel; the wave tile is
// 32 TMB x 32, so the epilogue stays in the MFMA register layout.  BK is the K step in elements; a
// staged row is BK x (2 or 4) bytes.  fp32 operands run four v_mfma_f32_32x32x2_f32 per 16-byte chunk
// pair, which keeps the matrix pipe about as busy as the memory system, so they take row blocks of 32 only.
//
// SEQ (TMB = 2, 4 or 8 row blocks of 32, K step 256): a stage of W with all its x blocks does not fit
// LDS twice, so the blocks take turns on the same W stage, each through one of two 16 KB x buffers:
// two W stages of 64 KB and the two x buffers are exactly the 160 KB.  While block j is multiplied,
// x block j+1 (of the next K step after the last block) is on its way, and the next W stage all
// through the current one.  The copies of a wave return in order, so a wave that waited for a
// young x block would also wait for the W stage issued before it; therefore the copy duties are
// split by wave: waves 0 and 1 copy W (and wait once per stage), waves 2 and 3 copy x (and wait
// every block); all four multiply.
template <int TMB, int BK, int DT, bool SEQ = false>
__device__ __forceinline__ void gemm_bf16_skinny_body(const GemmArgs &a) {
    constexpr bool F32 = DT == FLE_F32;
    constexpr int ES = F32 ? 4 : 2;            // bytes per operand element
    static_assert(!SEQ || ((TMB == 2 || TMB == 4 || TMB == 8) && BK == 256 && !F32), "the sequential variant is 2, 4 or 8 row blocks on a 256-wide K step of a 2-byte dtype");
    static_assert(!F32 || TMB == 1, "fp32 operands: row blocks of 32 only (the matrix pipe is as busy as the memory system already)");
    using frag_t = typename std::conditional<F32, f32x4, typename std::conditional<DT == FLE_F16, f16x8, bf16x8>::type>::type;
    constexpr int BM = 32 * TMB, BN = 128;
    constexpr int RB = BK * ES;                // bytes per staged row
    constexpr int CPR = RB / 16, RPI = 64 / CPR;  // 16-byte chunks per row, rows per copy instruction
    constexpr int KPS = RB / 32;               // k slices (two 16-byte chunks of every row) per stage
    constexpr int SW = BN * RB, SX = BM * RB, STAGE = SW + SX;
    constexpr int NST = SEQ ? 2 : (160 * 1024) / STAGE < 8 ? (160 * 1024) / STAGE : 8;
    constexpr int NIW = 32 / RPI, NIX = (8 * TMB) / RPI, LPS = NIW + NIX;  // copy instructions per wave per stage
    static_assert(SEQ || (NST >= 2 && NIX >= 1 && (NST - 2) * LPS < 64), "ring does not fit the counters");
    constexpr int SXB = 32 * RB;  // one x block of 32 rows (SEQ)
    __shared__ __attribute__((aligned(1024))) char smem[SEQ ? 2 * SW + 2 * SXB : NST * STAGE];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t M = a.M, N = a.N;
    // Workgroup -> (W tile, block of BM rows of x).  The row blocks of one W tile get ids that differ
    // by multiples of 8, next to each other in dispatch order: they land on the same XCD at about the
    // same time, so W comes from HBM once and from that XCD's L2 for the other row blocks.
    int64_t n0, m0;
    {
        const uint32_t bid = blockIdx.x, xcd = bid % 8, rest = bid / 8, tm = uint32_t(a.tiles_m);
        const uint32_t tile_n = (rest / tm) * 8 + xcd;
        if (tile_n >= uint32_t(a.tiles_n)) return;  // grid rounded up to a multiple of 8 tiles; the whole workgroup leaves
        n0 = int64_t(tile_n) * BN;
        m0 = int64_t(rest % tm) * BM;
    }

    // Chunk c of a row is stored at position c ^ sw(row): every 16-lane group of a fragment read
    // (16 consecutive rows, one logical chunk) then covers 16 different 16-byte bank groups.
    auto sw = [](int row) { return CPR == 8 ? ((row & 7) ^ ((row >> 3) & 1)) : (row & 15); };
    const int lr = lane / CPR, lp = lane % CPR;
    __amdgpu_buffer_rsrc_t rw, rx;
    {
        const int64_t wrows = (N - n0) < BN ? (N - n0) : BN, xrows = (M - m0) < BM ? (M - m0) : BM;
        rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(reinterpret_cast<const char *>(a.w) + n0 * a.ldw * ES), 0,
                                               uint32_t(((wrows - 1) * a.ldw + a.K) * ES), 0x00020000);
        rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(reinterpret_cast<const char *>(a.x) + m0 * a.ldx * ES), 0,
                                               uint32_t(((xrows - 1) * a.ldx + a.K) * ES), 0x00020000);
    }
    const uint32_t ldwb = uint32_t(a.ldw) * ES, ldxb = uint32_t(a.ldx) * ES;
    auto issue = [&](int kt) {
        char *base = smem + (kt % NST) * STAGE;
        const uint32_t kb = uint32_t(kt) * RB;
#pragma unroll
        for (int j = 0; j < NIW; ++j) {  // this wave's own 32 rows of W
            const int row = j * RPI + lr;
            const uint32_t voff = uint32_t(wave * 32 + row) * ldwb + uint32_t((lp ^ sw(row)) & (CPR - 1)) * 16 + kb;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_void *)(base + (wave * 32 + j * RPI) * RB), 16, voff, 0, 0, 2);
        }
#pragma unroll
        for (int j = 0; j < NIX; ++j) {  // a quarter of the shared x tile
            const int row = wave * (8 * TMB) + j * RPI + lr;
            const uint32_t voff = uint32_t(row) * ldxb + uint32_t((lp ^ sw(row)) & (CPR - 1)) * 16 + kb;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_void *)(base + SW + (wave * (8 * TMB) + j * RPI) * RB), 16, voff, 0, 0, 0);
        }
    };
    const int fr = lane & 31, fh = lane >> 5, fs = sw(fr);
    f32x16 acc[TMB];
#pragma unroll
    for (int t = 0; t < TMB; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    auto compute = [&](int kt) {
        const char *sW = smem + (kt % NST) * STAGE + wave * 32 * RB + fr * RB, *sX = smem + (kt % NST) * STAGE + SW + fr * RB;
#pragma unroll
        for (int kk = 0; kk < KPS; ++kk) {
            const int off = (((2 * kk + fh) ^ fs) & (CPR - 1)) * 16;
            const frag_t fw = *reinterpret_cast<const frag_t *>(sW + off);
#pragma unroll
            for (int t = 0; t < TMB; ++t) {
                const frag_t fx = *reinterpret_cast<const frag_t *>(sX + t * 32 * RB + off);
                if constexpr (F32) {
                    // four 32x32x2 steps: step e pairs element e of the two 16-byte chunks of every row (the same k
                    // permutation for both operands)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(fw[e], fx[e], acc[t], 0, 0, 0);
                } else if constexpr (DT == FLE_F16) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw, fx, acc[t], 0, 0, 0);
                else acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, fx, acc[t], 0, 0, 0);
            }
        }
    };
    // K stages kt .. KT-1 of this workgroup (all of them unless K is split over gridDim.y)
    const int KA = int(a.K / BK);
    int kt = int(int64_t(blockIdx.y) * KA / gridDim.y);
    const int KT = int(int64_t(blockIdx.y + 1) * KA / gridDim.y);
    if constexpr (SEQ) {
        const bool w_wave = wave < 2;  // copy duty of this wave: W (waves 0, 1) or x (waves 2, 3)
        auto issue_w = [&](int k) {    // 64 rows of W stage k
            char *base = smem + (k & 1) * SW;
            const uint32_t kb = uint32_t(k) * RB;
#pragma unroll
            for (int j = 0; j < 64 / RPI; ++j) {
                const int row = wave * 64 + j * RPI + lr;
                const uint32_t voff = uint32_t(row) * ldwb + uint32_t((lp ^ sw(row)) & (CPR - 1)) * 16 + kb;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_void *)(base + (wave * 64 + j * RPI) * RB), 16, voff, 0, 0, 2);
            }
        };
        auto issue_x = [&](int k, int blk) {  // 16 rows of x block blk at K step k, into x buffer blk & 1
            char *base = smem + 2 * SW + (blk & 1) * SXB;
            const uint32_t kb = uint32_t(k) * RB;
#pragma unroll
            for (int j = 0; j < 16 / RPI; ++j) {
                const int row = (wave - 2) * 16 + j * RPI + lr;  // row within the block; rows beyond M read zeros (out of range)
                const uint32_t voff = uint32_t(blk * 32 + row) * ldxb + uint32_t((lp ^ sw(row)) & (CPR - 1)) * 16 + kb;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_void *)(base + ((wave - 2) * 16 + j * RPI) * RB), 16, voff, 0, 0, 0);
            }
        };
        auto compute_blk = [&](int k, auto blk_c) {
            constexpr int BLK = decltype(blk_c)::value;
            const char *sW = smem + (k & 1) * SW + wave * 32 * RB + fr * RB, *sX = smem + 2 * SW + (BLK & 1) * SXB + fr * RB;
#pragma unroll
            for (int kk = 0; kk < KPS; ++kk) {
                const int off = (((2 * kk + fh) ^ fs) & (CPR - 1)) * 16;
                const frag_t fw = *reinterpret_cast<const frag_t *>(sW + off);
                const frag_t fx = *reinterpret_cast<const frag_t *>(sX + off);
                if constexpr (F32) {  // (never instantiated: the sequential variant is for 2-byte dtypes)
                } else if constexpr (DT == FLE_F16) acc[BLK] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw, fx, acc[BLK], 0, 0, 0);
                else acc[BLK] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, fx, acc[BLK], 0, 0, 0);
            }
        };
        // one block step: wait for what this wave copied for it, let everyone catch up, send the next copies, multiply
        auto block_step = [&](int k, auto blk_c, bool more) {
            constexpr int BLK = decltype(blk_c)::value;
            if (!w_wave || BLK == 0) wait_vmcnt<0>();   // x wave: x block BLK has landed; W wave, block 0: W stage k has
            __builtin_amdgcn_s_barrier();                // everyone's have; the buffers of the previous block step are free
            if (w_wave) {
                if (BLK == 0 && more) issue_w(k + 1);
            } else {
                if (BLK + 1 < TMB) issue_x(k, BLK + 1);
                else if (more) issue_x(k + 1, 0);
            }
            compute_blk(k, blk_c);
        };
        if (kt < KT) {
            if (w_wave) issue_w(kt);
            else issue_x(kt, 0);
        }
        for (; kt < KT; ++kt) {
            const bool more = kt + 1 < KT;
            block_step(kt, std::integral_constant<int, 0>{}, more);
            block_step(kt, std::integral_constant<int, 1>{}, more);
            if constexpr (TMB >= 4) {
                block_step(kt, std::integral_constant<int, 2>{}, more);
                block_step(kt, std::integral_constant<int, 3>{}, more);
            }
            if constexpr (TMB >= 8) {
                block_step(kt, std::integral_constant<int, 4>{}, more);
                block_step(kt, std::integral_constant<int, 5>{}, more);
                block_step(kt, std::integral_constant<int, 6>{}, more);
                block_step(kt, std::integral_constant<int, 7>{}, more);
            }
        }
    } else {
#pragma unroll
        for (int s = 0; s < NST - 1; ++s)
            if (kt + s < KT) issue(kt + s);
        for (; kt + NST - 1 < KT; ++kt) {
            wait_vmcnt<(NST - 2) * LPS>();  // the newest NST-2 stages may still be in flight
            __builtin_amdgcn_s_barrier();    // stage kt is complete; stage kt-1 is no longer read
            issue(kt + NST - 1);
            compute(kt);
        }
        for (; kt < KT; ++kt) {
            wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            compute(kt);
        }
    }

    // ---- epilogue in the MFMA layout: acc[t][4q+e] = out[32 t + (lane & 31)][n_lane + 8 q + e]
    char *const dst = a.dst ? reinterpret_cast<char *>(a.dst) + int64_t(blockIdx.y) * a.split_stride : nullptr;
    const int h = lane >> 5;
    const int64_t n_lane = n0 + wave * 32 + 4 * h;
    if (n0 + wave * 32 >= N) return;
    int64_t n_c[4];  // clamped column of each group of four (loads stay in bounds; stores are masked)
#pragma unroll
    for (int q = 0; q < 4; ++q) n_c[q] = n_lane + 8 * q < N ? n_lane + 8 * q : N - 4;
    for (int o = 0; o < a.epi.n_pre; ++o) {
        const DevOp op = a.epi.pre[o];
        switch (op.kind) {
        case FLE_BIAS:
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 bv = ld4<DT>(a.epi.bias, n_c[q]);
#pragma unroll
                for (int t = 0; t < TMB; ++t)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[t][4 * q + e] += bv[e];
            }
            break;
        case FLE_SCALE:
#pragma unroll
            for (int t = 0; t < TMB; ++t) acc[t] *= op.alpha;
            break;
        case FLE_RELU:
#pragma unroll
            for (int t = 0; t < TMB; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][r] = relu_f(acc[t][r]);
            break;
        case FLE_GELU_ERF:
#pragma unroll
            for (int t = 0; t < TMB; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][r] = gelu_erf_f(acc[t][r]);
            break;
        case FLE_GELU_TANH:
#pragma unroll
            for (int t = 0; t < TMB; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][r] = gelu_tanh_f(acc[t][r]);
            break;
        case FLE_RESIDUAL:
#pragma unroll
            for (int t = 0; t < TMB; ++t) {
                const int64_t m = m0 + 32 * t + (lane & 31), mc = m < M ? m : M - 1;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 rv = ld4<DT>(op.p0, mc * op.ld + n_c[q]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[t][4 * q + e] += rv[e];
                }
            }
            break;
        case FLE_STORE:  // a copy of the values as they stand, rounded to the dtype
#pragma unroll
            for (int t = 0; t < TMB; ++t) {
                const int64_t m = m0 + 32 * t + (lane & 31);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t n = n_lane + 8 * q;
                    if (m < M && n < N) {
                        const f32x4 v = f32x4{acc[t][4 * q], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]};
                        if constexpr (F32) {
                            *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(const_cast<void *>(op.p0)) + m * op.ld + n) = v;
                        } else {
                            constexpr int DT2 = F32 ? FLE_BF16 : DT;
                            *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(const_cast<void *>(op.p0)) + m * op.ld + n) = pack4<DT2>(v);
                        }
                    }
                }
            }
            break;
        default: break;
        }
    }
    if (a.epi.row_kind >= 0) {  // one partial per (row, 32-column wave tile)
        const int64_t left = N - (n0 + wave * 32);
        const float cnt = float(left < 32 ? left : 32);
        const bool ln = a.epi.row_kind == FLE_LAYERNORM;
#pragma unroll
        for (int t = 0; t < TMB; ++t) {
            const int64_t m = m0 + 32 * t + (lane & 31);
            float s0, s1;
            if (ln) {
                float sum = 0.0f;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (n_lane + 8 * q < N)
#pragma unroll
                        for (int e = 0; e < 4; ++e) sum += acc[t][4 * q + e];
                sum += __shfl_xor(sum, 32);
                const float mean = sum / cnt;
                float m2 = 0.0f;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (n_lane + 8 * q < N)
#pragma unroll
                        for (int e = 0; e < 4; ++e) m2 += (acc[t][4 * q + e] - mean) * (acc[t][4 * q + e] - mean);
                m2 += __shfl_xor(m2, 32);
                s0 = mean;
                s1 = m2;
            } else {
                float mx = -INFINITY;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (n_lane + 8 * q < N)
#pragma unroll
                        for (int e = 0; e < 4; ++e) mx = fmaxf(mx, acc[t][4 * q + e]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                float se = 0.0f;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (n_lane + 8 * q < N)
#pragma unroll
                        for (int e = 0; e < 4; ++e) se += __expf(acc[t][4 * q + e] - mx);
                se += __shfl_xor(se, 32);
                s0 = mx;
                s1 = se;
            }
            if (h == 0 && m < M) *reinterpret_cast<float2 *>(a.partials + (m * a.np + (n0 + wave * 32) / 32) * 2) = make_float2(s0, s1);
            if (a.dst_rel) acc[t] -= s0;
        }
    }
    if (a.dst) {
#pragma unroll
        for (int t = 0; t < TMB; ++t) {
            const int64_t m = m0 + 32 * t + (lane & 31);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t n = n_lane + 8 * q;
                if (m < M && n < N) {
                    const f32x4 v = f32x4{acc[t][4 * q], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]};
                    if (F32 || a.dst_f32) {
                        *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(dst) + m * a.ldd + n) = v;
                    } else {
                        constexpr int DT2 = F32 ? FLE_BF16 : DT;  // (this branch is never taken for fp32 problems)
                        *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(dst) + m * a.ldd + n) = pack4<DT2>(v);
                    }
                }
            }
        }
    }
}
template <int TMB, int BK, int DT, bool SEQ = false>
__global__ __launch_bounds__(256) void gemm_bf16_skinny(const GemmArgs a) { gemm_bf16_skinny_body<TMB, BK, DT, SEQ>(a); }

}  // namespace fle
