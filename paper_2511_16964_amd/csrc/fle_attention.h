// Scaled dot-product attention (forward), one pass over the keys with a running softmax.
#pragma once
#include "fle_device_common.h"

namespace fle {

typedef __attribute__((ext_vector_type(4))) short i16x4;

#ifndef FLE_ATTN_HEAD_GROUP
#define FLE_ATTN_HEAD_GROUP 8u  // heads an XCD works on at a time (see the workgroup mapping)
#endif

struct AttnArgs {
    const void *q, *k, *v;
    void *o;
    int64_t ldq, ldk, ldv, ldo;  // elements between consecutive tokens
    int64_t sbq, sbk, sbv, sbo;  // elements between consecutive sequences
    int32_t T, Tk, H, B;         // queries and keys per sequence, heads, sequences
    int32_t causal;     // 0: no mask; G >= 1: query t sees the keys below (t / G + 1) * G (G = 1: the plain causal mask)
    float scale_log2e;  // softmax scale times log2(e): the exponentials are taken in base 2
};

// The K and V of one sequence and head as buffer resources, and the copy of 1 KB of each into LDS.
struct BufferPair {
    __amdgpu_buffer_rsrc_t k, v;
    __device__ __forceinline__ void copy_1k(char *dst_k, char *dst_v, uint32_t off_k, uint32_t off_v) const {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(k, (lds_void *)dst_k, 16, off_k, 0, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(v, (lds_void *)dst_v, 16, off_v, 0, 0, 0);
    }
};

// Placement of the 16-byte chunks of a K / V row in LDS: chunk c of row r sits at position c ^ lds_swizzle(r).
// Two access patterns must spread over all banks (256 bytes per cycle): the K fragment reads (16 consecutive
// rows, the same chunk of each) and the transposing V reads (32 lanes = 4 consecutive rows x 64 contiguous
// bytes).  The first needs 16 consecutive rows to land on 16 different 16-byte positions of a 256-byte bank
// sweep, the second needs rows r .. r + 3 (r a multiple of 4) to move a 64-byte group to 4 different groups.
// D >= 128 (a row is one or two sweeps): the two low row bits go to chunk bits 3 and 2, the next two to the
// low ones.  D = 64 (two rows per sweep, 8 chunks; row parity picks the half sweep): row bit 1 goes to the
// high chunk bit, bits 2 and 3 to the low ones.  D = 32 (four rows per sweep, a row is one 64-byte group, so
// the V reads need nothing): row bits 2 and 3 pick among the four chunks.
template <int D>
__device__ __forceinline__ int lds_swizzle(int row) {
    if constexpr (D >= 128) return ((row & 3) << 2) | ((row >> 2) & 3);
    else if constexpr (D == 64) return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
    else return (row >> 2) & 3;
}

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
// A workgroup is 4 waves; a wave owns QT tiles of 32 queries (the library launches QT = 1, which keeps two
// or three waves on a SIMD) and walks the key blocks of 64 that all four waves share through LDS, double
// buffered: the next block is copied into the other stage (buffer loads that write LDS directly) while the
// current one is used; one barrier per iteration.  Rows of K / V are stored with their 16-byte
// chunks XOR-ed by lds_swizzle(row), which spreads both the row-wise reads of K and the transposing reads
// of V over all banks.  With the causal mask a wave stops computing at its last visible block and only keeps
// the barriers; the mask itself is applied on the diagonal and tail blocks only.
//
// The kernel states the occupancy it is built for (one wave per SIMD at D = 256, two at 128, three below): left to
// itself the register allocator aims one step higher, caps the ordinary VGPRs accordingly and parks the
// output accumulators in AGPRs, copying all of them in and out on every trip of the loop.
template <int DT, int D, int QT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 256 ? 1 : D == 128 ? 2 : 3, D == 256 ? 1 : D == 128 ? 2 : 3))) void flash_attention(const AttnArgs a) {
    static_assert(DT == FLE_BF16 || DT == FLE_F16, "2-byte dtypes only");
    static_assert(D == 32 || D == 64 || D == 128 || D == 256, "head dimension 32, 64, 128 or 256");
    using frag_t = typename std::conditional<DT == FLE_F16, f16x8, bf16x8>::type;
    constexpr int BKV = 64, WQ = 32 * QT, BQ = 4 * WQ;
    constexpr int NC = D / 16, ND = D / 32, RB = D * 2, CPR = D / 8;
    constexpr int STAGE = 2 * BKV * RB;
    __shared__ __attribute__((aligned(16))) char smem[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, h2 = lane >> 5;
    const int T = a.T, Tk = a.Tk;
    const int n_qb = (T + BQ - 1) / BQ;
    // Workgroup -> (sequence and head, query block).  Consecutive workgroups go to the 8 XCDs in turn, so
    // workgroup L is the (L / 8)-th one of XCD L % 8.  An XCD takes consecutive heads whole (every query block
    // of a head reads the same K and V, which then stay in that XCD's L2) and, under the causal mask, each
    // head's blocks from the longest to the shortest; handing out query blocks in plain order instead gives
    // XCD j block j of every head, i.e. all the long blocks to one XCD and all the short ones to another.
    const uint32_t n_heads = uint32_t(a.H) * uint32_t(a.B), xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    int head, qi;
    if (n_heads % 8 == 0) {
        // heads xcd * hpx .. + hpx - 1, in groups of FLE_ATTN_HEAD_GROUP heads that are worked on together
        // (their K and V share the L2), each group block-major: all its longest query blocks first
        const uint32_t hpx = n_heads / 8, gsz = FLE_ATTN_HEAD_GROUP * uint32_t(n_qb);
        const uint32_t g = slot / gsz, u = slot - g * gsz;
        const uint32_t left = hpx - g * FLE_ATTN_HEAD_GROUP, gh = left < FLE_ATTN_HEAD_GROUP ? left : FLE_ATTN_HEAD_GROUP;
        qi = int(u / gh);
        head = int(xcd * hpx + g * FLE_ATTN_HEAD_GROUP + u % gh);
    } else {
        const uint32_t n_items = n_heads * uint32_t(n_qb), per = n_items / 8, rem = n_items % 8;
        const uint32_t item = slot + xcd * per + (xcd < rem ? xcd : rem);  // XCD j owns a contiguous range of items
        head = int(item / uint32_t(n_qb));
        qi = int(item % uint32_t(n_qb));
    }
    const int qb = a.causal ? n_qb - 1 - qi : qi;
    const int q0 = qb * BQ, wq0 = q0 + wave * WQ;
    const int64_t seq = head / a.H;
    const int64_t col0 = int64_t(head % a.H) * D;
    const char *qp = reinterpret_cast<const char *>(a.q) + (seq * a.sbq + col0) * 2;
    const char *kp = reinterpret_cast<const char *>(a.k) + (seq * a.sbk + col0) * 2;
    const char *vp = reinterpret_cast<const char *>(a.v) + (seq * a.sbv + col0) * 2;
    char *op = reinterpret_cast<char *>(a.o) + (seq * a.sbo + col0) * 2;

    // Keys 0 .. limit - 1 are visible to a query; limits grow with the query index, so the last query of a
    // workgroup (of a wave) decides how many key blocks it walks and the first one whether a block needs the mask.
    // Under a mask the T queries stand at the last T of the Tk key positions.
    const int G = a.causal;
    auto limit_of = [&](int query) {
        const int lim = G ? ((query + Tk - T) / G + 1) * G : Tk;
        return lim < Tk ? lim : Tk;
    };
    const int q_last = (q0 + BQ < T ? q0 + BQ : T) - 1, w_last = (wq0 + WQ < T ? wq0 + WQ : T) - 1;
    const int n_blocks = (limit_of(q_last) + BKV - 1) / BKV;
    const int wave_last = wq0 < T ? (limit_of(w_last) + BKV - 1) / BKV - 1 : -1;  // a wave of padding rows only keeps the barriers
    const int wave_first_limit = limit_of(wq0);
    int key_limit[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) key_limit[qt] = limit_of(wq0 + 32 * qt + l31);

    // Q fragments stay in registers: B operand, lane = query, 8 consecutive d per 16-wide step
    frag_t qf[QT][NC];
    {
        const __amdgpu_buffer_rsrc_t rsrc_q = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(qp), 0, uint32_t(int64_t(T - 1) * a.ldq * 2 + RB), 0x00020000);
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            const uint32_t off = uint32_t(wq0 + 32 * qt + l31) * uint32_t(a.ldq * 2) + uint32_t(16 * h2);  // rows at or beyond T read as zeros
#pragma unroll
            for (int c = 0; c < NC; ++c) qf[qt][c] = __builtin_bit_cast(frag_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc_q, off + 32 * c, 0, 0));
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

    // Copies of one K / V block, global memory -> LDS without passing registers: one instruction moves
    // 1 KB (RPI rows) to consecutive LDS addresses, so the XOR placement is applied on the source side: the
    // lane that fills chunk position `pos` of a row fetches that row's chunk pos ^ lds_swizzle(row).  Rows at or
    // beyond Tk lie outside the buffer range and arrive as zeros.
    constexpr int RPI = 1024 / RB, NI = BKV / RPI / 4;  // rows per instruction; instructions per wave and operand
    const uint32_t nrec_k = uint32_t(int64_t(Tk - 1) * a.ldk * 2 + RB), nrec_v = uint32_t(int64_t(Tk - 1) * a.ldv * 2 + RB);
    BufferPair kv;
    kv.k = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(kp), 0, nrec_k, 0x00020000);
    kv.v = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(vp), 0, nrec_v, 0x00020000);
    uint32_t cp_k[NI], cp_v[NI];  // this lane's source offsets inside a block
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int row = (wave * NI + i) * RPI + lane / CPR, pos = lane % CPR;
        cp_k[i] = uint32_t(row) * uint32_t(a.ldk * 2) + uint32_t((pos ^ lds_swizzle<D>(row)) * 16);
        cp_v[i] = uint32_t(row) * uint32_t(a.ldv * 2) + uint32_t((pos ^ lds_swizzle<D>(row)) * 16);
    }
    auto copy_block = [&](char *stage, int kb0) {
        const uint32_t k0 = uint32_t(kb0) * uint32_t(a.ldk * 2), v0 = uint32_t(kb0) * uint32_t(a.ldv * 2);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            char *dst = stage + (wave * NI + i) * 1024;
            kv.copy_1k(dst, dst + BKV * RB, cp_k[i] + k0, cp_v[i] + v0);
        }
    };

    // Per-lane LDS byte offsets that do not change over the loop.  The swizzle of a row only depends on the
    // row's low four bits, so the constant parts of a row index (32 kt, 16 c2) are plain address immediates and
    // only the parts that enter the XOR (the chunk, and the key bit 3 of the second half-fragment) need an
    // offset register of their own.
    // K fragment (A operand): row = 32 kt + l31, 16-byte chunk 2 c + h2.
    int koff[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) koff[c] = l31 * RB + (((2 * c + h2) ^ lds_swizzle<D>(l31)) * 16);
    // V^T fragment: source lane j of a 16-lane group points at key (j >> 2) + 4 h2 (+ 8 e + 16 c2 + 32 kt), d = 16 (group & 1) + 4 (j & 3) (+ 32 dt)
    const int vj = lane & 15, vg = lane >> 4;
    const int v_key = (vj >> 2) + 4 * (vg >> 1), v_d = 16 * (vg & 1) + 4 * (vj & 3);
    int voff[ND][2];
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int key = 8 * e + v_key, d = 32 * dt + v_d;
            voff[dt][e] = BKV * RB + key * RB + (((d >> 3) ^ lds_swizzle<D>(key)) * 16) + (d & 7) * 2;
        }

    // One block of 64 keys: the scores of its two 32-key tiles (two independent MFMA chains), one update of
    // the running maximum, then exponentials and second product tile by tile in one straight-line stretch, so
    // that the scheduler can run the exponentials of the second tile under the MFMAs of the first.
    auto compute = [&](auto stage_c, int kb0, bool mask) {
        constexpr int SOFF = decltype(stage_c)::value * STAGE;  // compile-time, so that it folds into the address immediates
        f32x16 s[2][QT];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kt][qt][r] = 0.0f;
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const frag_t kf = *reinterpret_cast<const frag_t *>(smem + koff[c] + (SOFF + 32 * kt * RB));
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    if constexpr (DT == FLE_F16) s[kt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[qt][c], s[kt][qt], 0, 0, 0);
                    else s[kt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qt][c], s[kt][qt], 0, 0, 0);
                }
            }
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            if (mask) {  // diagonal and tail blocks only (uniform over the wave)
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = kb0 + 32 * kt + 8 * (r / 4) + 4 * h2 + (r % 4);
                        if (key >= key_limit[qt]) s[kt][qt][r] = -INFINITY;
                    }
            }
            float mx = s[0][qt][0];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][qt][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // The reference point of the exponentials only moves when some row's maximum has grown by more
            // than 2^8 past it (always in the first block): the probabilities of a row then reach at most 256
            // instead of 1, a common factor that the final division by the row sum removes, and in most blocks
            // no lane of the wave has to rescale its accumulators.
            const float cand = mx * a.scale_log2e;
            const bool grow = cand > m_run[qt] + 8.0f;
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                const float m_new = grow ? cand : m_run[qt];
                const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_new);
                m_run[qt] = m_new;
                l_run[qt] *= alpha;
#pragma unroll
                for (int dt = 0; dt < ND; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[dt][qt][r] *= alpha;
            }
        }
        float ps[QT];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) ps[qt] = 0.0f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            frag_t pf[QT][2];
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                const float m_ref = m_run[qt];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][qt][r], a.scale_log2e, -m_ref));
                    s[kt][qt][r] = pr;
                    ps[qt] += pr;
                }
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) {
                    const u32x2 lo = pack4<DT>(f32x4{s[kt][qt][8 * c2 + 0], s[kt][qt][8 * c2 + 1], s[kt][qt][8 * c2 + 2], s[kt][qt][8 * c2 + 3]});
                    const u32x2 hi = pack4<DT>(f32x4{s[kt][qt][8 * c2 + 4], s[kt][qt][8 * c2 + 5], s[kt][qt][8 * c2 + 6], s[kt][qt][8 * c2 + 7]});
                    pf[qt][c2] = __builtin_bit_cast(frag_t, u32x4{lo[0], lo[1], hi[0], hi[1]});
                }
            }
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int dt = 0; dt < ND; ++dt) {
                    struct { i16x4 e[2]; } part;
#pragma unroll
                    for (int e = 0; e < 2; ++e)
                        part.e[e] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) i16x4 *)(smem + voff[dt][e] + (SOFF + (32 * kt + 16 * c2) * RB)));
                    const frag_t vf = __builtin_bit_cast(frag_t, part);
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt) {
                        if constexpr (DT == FLE_F16) oacc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[qt][c2], oacc[dt][qt], 0, 0, 0);
                        else oacc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qt][c2], oacc[dt][qt], 0, 0, 0);
                    }
                }
        }
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            ps[qt] += __shfl_xor(ps[qt], 32);
            l_run[qt] += ps[qt];
        }
    };

    copy_block(smem, 0);
    wait_vmcnt<0>();
    __syncthreads();
    // two blocks per trip, so that the stage a block sits in is known at compile time
    auto block_step = [&](int j, auto stage_c) {
        constexpr int ST = decltype(stage_c)::value;
        const int kb0 = j * BKV;
        // the other stage was last read before the barrier that ended the previous block
        if (j + 1 < n_blocks) copy_block(smem + (ST ^ 1) * STAGE, kb0 + BKV);
        if (j <= wave_last) compute(stage_c, kb0, kb0 + BKV > wave_first_limit);
        wait_vmcnt<0>();
        __syncthreads();
    };
    for (int j = 0; j < n_blocks; j += 2) {
        block_step(j, std::integral_constant<int, 0>{});
        if (j + 1 < n_blocks) block_step(j + 1, std::integral_constant<int, 1>{});
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
