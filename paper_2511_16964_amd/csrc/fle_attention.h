// Scaled dot-product attention (forward), one pass over the keys with a running softmax.
#pragma once
#include "fle_device_common.h"

namespace fle {

typedef __attribute__((ext_vector_type(4))) short i16x4;

struct AttnArgs {
    const void *q, *k, *v;
    void *o;
    int64_t ldq, ldk, ldv, ldo;  // elements between consecutive tokens
    int32_t T, H;
    int32_t causal;
    float scale_log2e;  // softmax scale times log2(e): the exponentials are taken in base 2
};

// Everything is computed transposed, so that a lane owns one query:
//
//     S^T[key, query] = K[key, :] . Q[query, :]          v_mfma_f32_32x32x16 (A = K rows, B = Q rows)
//     O^T[d,   query] += V^T[d, key] * P^T[key, query]   v_mfma_f32_32x32x16 (A = V^T,    B = P^T)
//
// In the 32x32 result layout a lane holds column (lane & 31) -- its query -- and 16 rows, so the
// running maximum, the running sum and the rescaling factor of a query are per-lane scalars (one
// exchange with lane ^ 32 completes a reduction over keys), and the exponentiated S^T registers,
// rounded to the storage dtype, are already laid out as the B operand of the second product: result
// register r of the lane half h = lane >> 5 is key 8 (r / 4) + 4 h + r % 4, so registers 8 c .. 8 c + 7
// are K-slots (h, 0 .. 7) of the 16-key step c, i.e. keys 16 c + 4 h + {0..3} and 16 c + 8 + 4 h + {0..3}.
// The A operand V^T is gathered in the same key order straight from the row-major V block in LDS with
// ds_read_b64_tr_b16: within 16 lanes, source lane j points at 4 consecutive d of key j / 4, and lane i
// receives d = i of those four keys.  A sum over keys does not care about their order, only that both
// operands agree on it.
//
// A workgroup is 4 waves; a wave owns QT tiles of 32 queries (QT = 2 halves the LDS reads per MFMA, which
// is what bounds QT = 1) and walks the key blocks of 64 that all four waves share through LDS, double
// buffered: the next block travels global -> registers while the current one is used, and is written to
// the other stage before the one barrier of the iteration.  Rows of K / V are stored with their 16-byte
// chunks XOR-ed by (row & 7), which spreads both the row-wise reads of K and the transposing reads of V
// over all banks.  With the causal mask a wave stops computing at its last visible block and only keeps
// the barriers; the mask itself is applied on the diagonal and tail blocks only.
template <int DT, int D, int QT>
__global__ __launch_bounds__(256) void flash_attention(const AttnArgs a) {
    static_assert(DT == FLE_BF16 || DT == FLE_F16, "2-byte dtypes only");
    static_assert(D == 64 || D == 128, "head dimension 64 or 128");
    using frag_t = typename std::conditional<DT == FLE_F16, f16x8, bf16x8>::type;
    constexpr int BKV = 64, WQ = 32 * QT, BQ = 4 * WQ;
    constexpr int NC = D / 16, ND = D / 32, RB = D * 2, CPR = D / 8;
    constexpr int NLD = BKV * CPR / 256;  // 16-byte chunks per thread and operand per block
    constexpr int STAGE = 2 * BKV * RB;
    __shared__ __attribute__((aligned(16))) char smem[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, h2 = lane >> 5;
    const int T = a.T;
    const int n_qb = (T + BQ - 1) / BQ;
    const int qb = a.causal ? n_qb - 1 - int(blockIdx.x) : int(blockIdx.x);  // longest rows first
    const int q0 = qb * BQ, wq0 = q0 + wave * WQ;
    const int64_t tok0 = int64_t(blockIdx.z) * T;
    const int64_t col0 = int64_t(blockIdx.y) * D;
    const char *qp = reinterpret_cast<const char *>(a.q) + (tok0 * a.ldq + col0) * 2;
    const char *kp = reinterpret_cast<const char *>(a.k) + (tok0 * a.ldk + col0) * 2;
    const char *vp = reinterpret_cast<const char *>(a.v) + (tok0 * a.ldv + col0) * 2;
    char *op = reinterpret_cast<char *>(a.o) + (tok0 * a.ldo + col0) * 2;

    const int n_blocks_all = (T + BKV - 1) / BKV;
    int n_blocks = n_blocks_all, wave_last = n_blocks_all - 1;
    if (a.causal) {
        const int need = (q0 + BQ - 1) / BKV + 1;
        n_blocks = need < n_blocks_all ? need : n_blocks_all;
        wave_last = (wq0 + WQ - 1) / BKV;
    }
    if (wq0 >= T) wave_last = -1;  // a wave of padding rows only keeps the barriers

    // Q fragments stay in registers: B operand, lane = query, 8 consecutive d per 16-wide step
    frag_t qf[QT][NC];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int row = wq0 + 32 * qt + l31;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (row < T) raw = *reinterpret_cast<const u32x4 *>(qp + int64_t(row) * a.ldq * 2 + (16 * c + 8 * h2) * 2);
            qf[qt][c] = __builtin_bit_cast(frag_t, raw);
        }
    }

    f32x16 oacc[ND][QT];
    float m_run[QT], l_run[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        m_run[qt] = -INFINITY;
        l_run[qt] = 0.0f;
#pragma unroll
        for (int dt = 0; dt < ND; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][qt][r] = 0.0f;
    }

    // global -> registers -> LDS copies of one K / V block
    u32x4 kreg[NLD], vreg[NLD];
    auto fetch = [&](int kb0) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int idx = i * 256 + tid, row = idx / CPR, ch = idx % CPR;
            kreg[i] = u32x4{0u, 0u, 0u, 0u};
            vreg[i] = u32x4{0u, 0u, 0u, 0u};
            if (kb0 + row < T) {
                kreg[i] = *reinterpret_cast<const u32x4 *>(kp + int64_t(kb0 + row) * a.ldk * 2 + ch * 16);
                vreg[i] = *reinterpret_cast<const u32x4 *>(vp + int64_t(kb0 + row) * a.ldv * 2 + ch * 16);
            }
        }
    };
    auto stash = [&](char *stage) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int idx = i * 256 + tid, row = idx / CPR, ch = idx % CPR;
            const int off = row * RB + ((ch ^ (row & 7)) * 16);
            *reinterpret_cast<u32x4 *>(stage + off) = kreg[i];
            *reinterpret_cast<u32x4 *>(stage + BKV * RB + off) = vreg[i];
        }
    };

    // per-lane LDS offsets that do not change over the loop
    // K fragment (A operand): row = 32 kt + l31, 16-byte chunk 2 c + h2
    // V^T fragment: source lane j of a 16-lane group points at key (j >> 2) + 4 h2 (+ 16 c2 + 8 e + 32 kt), d = 16 (group & 1) + 4 (j & 3) (+ 32 dt)
    const int vj = lane & 15, vg = lane >> 4;
    const int v_key = (vj >> 2) + 4 * (vg >> 1), v_d = 16 * (vg & 1) + 4 * (vj & 3);

    auto compute = [&](const char *stage, int kb0, auto mask_c) {
        constexpr bool MASK = decltype(mask_c)::value;
        const char *sK = stage, *sV = stage + BKV * RB;
        f32x16 s[2][QT];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kt][qt][r] = 0.0f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const int row = 32 * kt + l31;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const frag_t kf = *reinterpret_cast<const frag_t *>(sK + row * RB + (((2 * c + h2) ^ (row & 7)) * 16));
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    if constexpr (DT == FLE_F16) s[kt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[qt][c], s[kt][qt], 0, 0, 0);
                    else s[kt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qt][c], s[kt][qt], 0, 0, 0);
                }
            }
        }
        frag_t pf[QT][2][2];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            if constexpr (MASK) {
                const int query = wq0 + 32 * qt + l31;
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = kb0 + 32 * kt + 8 * (r / 4) + 4 * h2 + (r % 4);
                        if (key >= T || (a.causal && key > query)) s[kt][qt][r] = -INFINITY;
                    }
            }
            float mx = s[0][qt][0];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][qt][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[qt], mx * a.scale_log2e);
            const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_new);
            m_run[qt] = m_new;
            float ps = 0.0f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][qt][r], a.scale_log2e, -m_new));
                    s[kt][qt][r] = p;
                    ps += p;
                }
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) {
                    const u32x2 lo = pack4<DT>(f32x4{s[kt][qt][8 * c2 + 0], s[kt][qt][8 * c2 + 1], s[kt][qt][8 * c2 + 2], s[kt][qt][8 * c2 + 3]});
                    const u32x2 hi = pack4<DT>(f32x4{s[kt][qt][8 * c2 + 4], s[kt][qt][8 * c2 + 5], s[kt][qt][8 * c2 + 6], s[kt][qt][8 * c2 + 7]});
                    pf[qt][kt][c2] = __builtin_bit_cast(frag_t, u32x4{lo[0], lo[1], hi[0], hi[1]});
                }
            }
            ps += __shfl_xor(ps, 32);
            l_run[qt] = l_run[qt] * alpha + ps;
#pragma unroll
            for (int dt = 0; dt < ND; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[dt][qt][r] *= alpha;
        }
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int dt = 0; dt < ND; ++dt) {
                    struct { i16x4 e[2]; } part;
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int key = 32 * kt + 16 * c2 + 8 * e + v_key, d = 32 * dt + v_d;
                        const int off = key * RB + (((d >> 3) ^ (key & 7)) * 16) + (d & 7) * 2;
                        part.e[e] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(sV + off));
                    }
                    const frag_t vf = __builtin_bit_cast(frag_t, part);
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt) {
                        if constexpr (DT == FLE_F16) oacc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[qt][kt][c2], oacc[dt][qt], 0, 0, 0);
                        else oacc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qt][kt][c2], oacc[dt][qt], 0, 0, 0);
                    }
                }
    };

    fetch(0);
    stash(smem);
    __syncthreads();
    for (int j = 0; j < n_blocks; ++j) {
        const int kb0 = j * BKV;
        const bool more = j + 1 < n_blocks;
        if (more) fetch(kb0 + BKV);
        if (j <= wave_last) {
            const bool mask = kb0 + BKV > T || (a.causal && kb0 + BKV - 1 > wq0);
            if (mask) compute(smem + (j & 1) * STAGE, kb0, std::true_type{});
            else compute(smem + (j & 1) * STAGE, kb0, std::false_type{});
        }
        if (more) stash(smem + ((j + 1) & 1) * STAGE);
        __syncthreads();
    }

    // O^T registers: lane = query, register r of tile dt is d = 32 dt + 8 (r / 4) + 4 h2 + r % 4
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int query = wq0 + 32 * qt + l31;
        if (query >= T) continue;
        const float inv = 1.0f / l_run[qt];
        char *orow = op + int64_t(query) * a.ldo * 2;
#pragma unroll
        for (int dt = 0; dt < ND; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 v = {oacc[dt][qt][4 * g] * inv, oacc[dt][qt][4 * g + 1] * inv, oacc[dt][qt][4 * g + 2] * inv, oacc[dt][qt][4 * g + 3] * inv};
                *reinterpret_cast<u32x2 *>(orow + (32 * dt + 8 * g + 4 * h2) * 2) = pack4<DT>(v);
            }
    }
}

}  // namespace fle
