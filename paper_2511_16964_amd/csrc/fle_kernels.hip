// Device side of libfle: hand-written gfx950 (CDNA4) kernels and their launcher.
//
//   gemm_bf16_tiled   bf16 MFMA GEMM with the elementwise epilogue applied in registers
//   gemm_general      any shape / alignment / dtype, fp32 MFMA, in-block split-K
//   finalize_rows     second pass of a row reduction (LayerNorm / softmax) + trailing ops
//   finalize_lse      second pass of logsumexp
//
// Orientation used by both GEMM kernels: the W tile is MFMA operand A and the x tile is
// operand B, so the accumulator holds a tile of out^T.  In the MFMA result layout a lane owns
// one column and groups of four consecutive rows; with this orientation a lane therefore owns
// one output row m and groups of four consecutive n: stores, bias and residual accesses are
// 8-byte vectors, and a row reduction is in-register work plus one cross-lane exchange.
#include <hip/hip_runtime.h>

#include "fle_plan.h"

namespace fle {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) void lds_void;

struct GemmArgs {
    int64_t M, N, K;
    const void *x;
    int64_t ldx;
    const void *w;
    int64_t ldw;
    void *dst;  // where the values after the pre-ops go (nullptr: nowhere, logsumexp)
    int64_t ldd;
    int32_t dst_f32;  // dst holds fp32 regardless of the storage dtype (workspace staging)
    int32_t np;       // row-reduction partials per row
    float *partials;  // [M][np][2], or nullptr without a row op
    int32_t tiles_m, tiles_n;
    DevEpilogue epi;
};

struct FinArgs {
    int64_t M, N;
    const void *y;  // staged values: storage dtype (may alias out) or fp32
    int64_t ldy;
    int32_t y_f32;
    int32_t np, part_cols;
    const float *partials;
    void *out;
    int64_t ldo;
    DevEpilogue epi;
};

// ------------------------------------------------------------------ scalar helpers
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

__device__ __forceinline__ float ld_elem(const void *p, int64_t i, int dtype) {
    if (dtype == FLE_BF16) return bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(p)[i]);
    return reinterpret_cast<const float *>(p)[i];
}

__device__ __forceinline__ void st_elem(void *p, int64_t i, int dtype, float v) {
    if (dtype == FLE_BF16)
        reinterpret_cast<__bf16 *>(p)[i] = static_cast<__bf16>(v);
    else
        reinterpret_cast<float *>(p)[i] = v;
}

__device__ __forceinline__ f32x4 ld4_bf16(const void *p) {  // p is 8-byte aligned
    const uint2 u = *reinterpret_cast<const uint2 *>(p);
    f32x4 r;
    r[0] = __uint_as_float(u.x << 16);
    r[1] = __uint_as_float(u.x & 0xffff0000u);
    r[2] = __uint_as_float(u.y << 16);
    r[3] = __uint_as_float(u.y & 0xffff0000u);
    return r;
}

__device__ __forceinline__ float relu_f(float v) { return v < 0.0f ? 0.0f : v; }  // NaN stays NaN

__device__ __forceinline__ float gelu_erf_f(float v) { return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f)); }

// 0.5 v (1 + tanh u) == v / (1 + exp(-2u)),  u = sqrt(2/pi) (v + 0.044715 v^3)
__device__ __forceinline__ float gelu_tanh_f(float v) {
    const float u = 0.7978845608028654f * (v + 0.044715f * v * v * v);
    return v * __builtin_amdgcn_rcpf(1.0f + __expf(-2.0f * u));
}

// One elementwise op on one value at (m, n).
__device__ __forceinline__ float apply_op(const DevOp &op, float v, int64_t m, int64_t n, const void *bias, int dtype) {
    switch (op.kind) {
    case FLE_BIAS: return v + ld_elem(bias, n, dtype);
    case FLE_SCALE: return v * op.alpha;
    case FLE_RELU: return relu_f(v);
    case FLE_GELU_ERF: return gelu_erf_f(v);
    case FLE_GELU_TANH: return gelu_tanh_f(v);
    case FLE_RESIDUAL: return v + ld_elem(op.p0, m * op.ld + n, dtype);
    default: return v;
    }
}

// ------------------------------------------------------------------ row-reduction partials
// LayerNorm partial over c values: (mean, M2 = sum (v - mean)^2); the count is implied by the
// partial's position.  Softmax / logsumexp partial: (max, sum exp(v - max)).
struct Stat {
    float n, a, b;  // n = count (LayerNorm only); (a, b) = (mean, M2) or (max, sum)
};

__device__ __forceinline__ Stat combine_ln(const Stat &p, const Stat &q) {
    if (q.n == 0.0f) return p;
    if (p.n == 0.0f) return q;
    Stat r;
    r.n = p.n + q.n;
    const float d = q.a - p.a;
    r.a = p.a + d * (q.n / r.n);
    r.b = p.b + q.b + d * d * (p.n * q.n / r.n);
    return r;
}

__device__ __forceinline__ Stat combine_sm(const Stat &p, const Stat &q) {
    Stat r;
    r.n = 0.0f;
    r.a = fmaxf(p.a, q.a);
    const float sp = p.b == 0.0f ? 0.0f : p.b * __expf(p.a - r.a);
    const float sq = q.b == 0.0f ? 0.0f : q.b * __expf(q.a - r.a);
    r.b = sp + sq;
    return r;
}

// All lanes of a wave end up with the combination of every partial of `row`, in a fixed order.
template <bool LN>
__device__ __forceinline__ Stat reduce_partials(const float *partials, int64_t row, int np, int part_cols, int64_t N, int lane) {
    Stat s;
    s.n = 0.0f;
    s.a = LN ? 0.0f : -INFINITY;
    s.b = 0.0f;
    const float *pr = partials + row * np * 2;
    for (int p = lane; p < np; p += 64) {
        Stat q;
        const int64_t left = N - int64_t(p) * part_cols;
        q.n = LN ? float(left < part_cols ? left : part_cols) : 0.0f;
        q.a = pr[2 * p];
        q.b = pr[2 * p + 1];
        s = LN ? combine_ln(s, q) : combine_sm(s, q);
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        Stat o;
        o.n = __shfl_xor(s.n, d);
        o.a = __shfl_xor(s.a, d);
        o.b = __shfl_xor(s.b, d);
        const bool upper = (lane & d) != 0;  // both partners combine (lower lane, upper lane): identical results
        const Stat lo = upper ? o : s, hi = upper ? s : o;
        s = LN ? combine_ln(lo, hi) : combine_sm(lo, hi);
    }
    return s;
}

// ------------------------------------------------------------------ tiled bf16 MFMA GEMM
// Block tile BM x BN (rows of x, rows of W), K step 64, 4 waves as 2 x 2, each wave owning
// (BM/2) x (BN/2) outputs as 32x32 accumulator tiles of v_mfma_f32_32x32x16_bf16.
// Operand tiles are copied HBM -> LDS by buffer loads that write LDS directly (no registers),
// two stages deep; a stage's row is 64 bf16 = 8 chunks of 16 bytes, stored at chunk position
// c ^ g(row) with g(row) = (row & 7) ^ ((row >> 3) & 1), which spreads the 16-byte reads of an
// MFMA fragment (32 consecutive rows, same logical chunk) over all LDS banks.
template <int ROWS>
struct TileLoader {
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t off_even, off_odd;  // this lane's byte offset in the tile for even / odd 8-row groups
    uint32_t row_step;           // bytes between 8-row groups
    int wave;

    __device__ __forceinline__ void init(const void *base, int64_t ld, int64_t rows_valid, int64_t K, int wave_, int lane) {
        const int64_t rv = rows_valid < ROWS ? rows_valid : ROWS;
        const uint32_t nrec = uint32_t(((rv - 1) * ld + K) * 2);
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, nrec, 0x00020000);
        const int lr = lane >> 3, lp = lane & 7;
        const uint32_t ldb = uint32_t(ld) * 2;
        wave = wave_;
        off_even = uint32_t(wave_ * (ROWS / 4) + lr) * ldb + uint32_t((lp ^ lr) << 4);
        off_odd = uint32_t(wave_ * (ROWS / 4) + lr) * ldb + uint32_t((lp ^ lr ^ 1) << 4);
        row_step = 8 * ldb;
    }
    // Copy this wave's quarter of the [ROWS x 64] tile at column k0 into stage memory `lds`.
    __device__ __forceinline__ void issue(char *lds, uint32_t k0) const {
#pragma unroll
        for (int j = 0; j < ROWS / 32; ++j) {
            const uint32_t voff = ((j & 1) ? off_odd : off_even) + uint32_t(j) * row_step + k0 * 2;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(lds + (wave * (ROWS / 4) + j * 8) * 128), 16, voff, 0, 0, 0);
        }
    }
};

template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_bf16_tiled(const GemmArgs a) {
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    __shared__ __attribute__((aligned(1024))) char sW0[BN * 128];
    __shared__ __attribute__((aligned(1024))) char sW1[BN * 128];
    __shared__ __attribute__((aligned(1024))) char sX0[BM * 128];
    __shared__ __attribute__((aligned(1024))) char sX1[BM * 128];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t M = a.M, N = a.N;

    // Workgroup -> tile.  Consecutive workgroup ids go round-robin over the 8 XCDs, so give each
    // XCD a contiguous range of tile ids, then walk tiles in groups of 4 tile rows: the tiles
    // an XCD works on at any time share x and W panels in its own L2.
    int tile_m, tile_n;
    {
        const uint32_t G = uint32_t(a.tiles_m) * uint32_t(a.tiles_n), bid = blockIdx.x;
        const uint32_t per = G / 8, rem = G % 8, xcd = bid % 8, loc = bid / 8;
        const uint32_t id = loc + xcd * per + (xcd < rem ? xcd : rem);
        const uint32_t width = 4 * uint32_t(a.tiles_n);
        const uint32_t first_m = (id / width) * 4;
        const uint32_t gsz = (uint32_t(a.tiles_m) - first_m) < 4 ? (uint32_t(a.tiles_m) - first_m) : 4;
        tile_m = int(first_m + (id % width) % gsz);
        tile_n = int((id % width) / gsz);
    }
    const int64_t m0 = int64_t(tile_m) * BM, n0 = int64_t(tile_n) * BN;
    const int wm = wave >> 1, wn = wave & 1;

    TileLoader<BM> ldx_;
    TileLoader<BN> ldw_;
    ldx_.init(reinterpret_cast<const char *>(a.x) + m0 * a.ldx * 2, a.ldx, M - m0, a.K, wave, lane);
    ldw_.init(reinterpret_cast<const char *>(a.w) + n0 * a.ldw * 2, a.ldw, N - n0, a.K, wave, lane);

    // Fragment read offsets: lane reads row (lane & 31) of a 32-row block, logical chunk 2*kk + (lane >> 5).
    uint32_t rd_off[4];
    {
        const int g = (lane & 7) ^ ((lane >> 3) & 1), h = lane >> 5;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) rd_off[kk] = uint32_t((lane & 31) * 128 + (((2 * kk + h) ^ g) << 4));
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    auto compute = [&](const char *sW, const char *sX) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 fw[TN], fx[TM];
#pragma unroll
            for (int t = 0; t < TN; ++t) fw[t] = *reinterpret_cast<const bf16x8 *>(sW + (wn * WN + t * 32) * 128 + rd_off[kk]);
#pragma unroll
            for (int t = 0; t < TM; ++t) fx[t] = *reinterpret_cast<const bf16x8 *>(sX + (wm * WM + t * 32) * 128 + rd_off[kk]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[j], fx[i], acc[i][j], 0, 0, 0);
        }
    };

    const int KT = int(a.K / 64);
    ldw_.issue(sW0, 0);
    ldx_.issue(sX0, 0);
    for (int kt = 0; kt < KT; kt += 2) {
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's copies into stage 0 have landed
        __syncthreads();                     // everyone's have, and everyone is done reading stage 1
        if (kt + 1 < KT) {
            ldw_.issue(sW1, uint32_t(kt + 1) * 64);
            ldx_.issue(sX1, uint32_t(kt + 1) * 64);
        }
        compute(sW0, sX0);
        if (kt + 1 < KT) {
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            if (kt + 2 < KT) {
                ldw_.issue(sW0, uint32_t(kt + 2) * 64);
                ldx_.issue(sX0, uint32_t(kt + 2) * 64);
            }
            compute(sW1, sX1);
        }
    }

    // ---- epilogue, all in registers.  acc[i][j][4q+e] is out[m_i][n_(j,q) + e].
    const int h = lane >> 5;
    const int64_t m_lane = m0 + wm * WM + (lane & 31);     // + 32 i
    const int64_t n_lane = n0 + wn * WN + 4 * h;           // + 32 j + 8 q + e
    const uint16_t *bias = reinterpret_cast<const uint16_t *>(a.epi.bias);

    for (int o = 0; o < a.epi.n_pre; ++o) {
        const DevOp op = a.epi.pre[o];
        switch (op.kind) {
        case FLE_BIAS:
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t n = n_lane + 32 * j + 8 * q;
                    f32x4 bv = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (n < N) bv = ld4_bf16(bias + n);
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] += bv[e];
                }
            break;
        case FLE_SCALE:
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] *= op.alpha;
            break;
        case FLE_RELU:
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = relu_f(acc[i][j][r]);
            break;
        case FLE_GELU_ERF:
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = gelu_erf_f(acc[i][j][r]);
            break;
        case FLE_GELU_TANH:
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = gelu_tanh_f(acc[i][j][r]);
            break;
        case FLE_RESIDUAL: {
            const uint16_t *res = reinterpret_cast<const uint16_t *>(op.p0);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int64_t m = m_lane + 32 * i;
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int64_t n = n_lane + 32 * j + 8 * q;
                        if (m < M && n < N) {
                            const f32x4 rv = ld4_bf16(res + m * op.ld + n);
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] += rv[e];
                        }
                    }
            }
            break;
        }
        default: break;
        }
    }

    // ---- row-reduction partials over this wave's WN columns, from the unrounded fp32 values
    if (a.epi.row_kind >= 0) {
        const int p = int((n0 + wn * WN) / WN);
        const bool ln = a.epi.row_kind == FLE_LAYERNORM;
        const int64_t cols_left = N - (n0 + wn * WN);
        const float cnt = float(cols_left < WN ? (cols_left > 0 ? cols_left : 0) : WN);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t m = m_lane + 32 * i;
            float s0, s1;
            if (ln) {
                float sum = 0.0f;
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (n_lane + 32 * j + 8 * q < N)
#pragma unroll
                            for (int e = 0; e < 4; ++e) sum += acc[i][j][4 * q + e];
                sum += __shfl_xor(sum, 32);
                const float mean = cnt > 0.0f ? sum / cnt : 0.0f;
                float m2 = 0.0f;
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (n_lane + 32 * j + 8 * q < N)
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float d = acc[i][j][4 * q + e] - mean;
                                m2 += d * d;
                            }
                m2 += __shfl_xor(m2, 32);
                s0 = mean;
                s1 = m2;
            } else {
                float mx = -INFINITY;
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (n_lane + 32 * j + 8 * q < N)
#pragma unroll
                            for (int e = 0; e < 4; ++e) mx = fmaxf(mx, acc[i][j][4 * q + e]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                float se = 0.0f;
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (n_lane + 32 * j + 8 * q < N)
#pragma unroll
                            for (int e = 0; e < 4; ++e) se += __expf(acc[i][j][4 * q + e] - mx);
                se += __shfl_xor(se, 32);
                s0 = mx;
                s1 = se;
            }
            if (h == 0 && m < M && cols_left > 0) {
                float2 *dstp = reinterpret_cast<float2 *>(a.partials + (m * a.np + p) * 2);
                *dstp = make_float2(s0, s1);
            }
        }
    }

    // ---- store: final values (no row op) or staged values for the finalize pass
    if (a.dst) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t m = m_lane + 32 * i;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t n = n_lane + 32 * j + 8 * q;
                    if (m < M && n < N) {
                        f32x4 v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
                        if (a.dst_f32)
                            *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(a.dst) + m * a.ldd + n) = v;
                        else
                            *reinterpret_cast<bf16x4 *>(reinterpret_cast<__bf16 *>(a.dst) + m * a.ldd + n) = __builtin_convertvector(v, bf16x4);
                    }
                }
        }
    }
}

// ------------------------------------------------------------------ general GEMM (fp32 MFMA)
// Block tile 32 x 32 outputs; the 4 waves split K (wave w takes 16-wide k blocks w, w+4, ...),
// each computing the whole tile with v_mfma_f32_16x16x4_f32 (bf16 inputs are widened exactly),
// then the partial tiles are summed through LDS in a fixed order.  A lane loads 4 consecutive k
// of its row; MFMA number e consumes element e of every lane's vector, i.e. the k order inside
// a block is permuted identically for both operands, which leaves the sum unchanged.
template <bool BF16, bool VEC>
__device__ __forceinline__ f32x4 load_k4(const void *base, int64_t ld, int64_t row, int64_t rows, int64_t k, int64_t K) {
    f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
    if (row >= rows) return v;
    if (VEC) {
        if (k < K) {
            if (BF16)
                v = ld4_bf16(reinterpret_cast<const uint16_t *>(base) + row * ld + k);
            else
                v = *reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(base) + row * ld + k);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (k + e < K) v[e] = ld_elem(base, row * ld + k + e, BF16 ? FLE_BF16 : FLE_F32);
    }
    return v;
}

template <bool BF16, bool VEC>
__global__ __launch_bounds__(256) void gemm_general(const GemmArgs a) {
    __shared__ float red[4][4][64][4];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r16 = lane & 15, q4 = lane >> 4;
    const int64_t M = a.M, N = a.N, K = a.K;
    const int64_t tile_n = blockIdx.x % a.tiles_n, tile_m = blockIdx.x / a.tiles_n;
    const int64_t m0 = tile_m * 32, n0 = tile_n * 32;
    const int dtype = BF16 ? FLE_BF16 : FLE_F32;

    f32x4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int64_t KB = (K + 15) / 16;
    for (int64_t kb = wave; kb < KB; kb += 4) {
        const int64_t k = kb * 16 + 4 * q4;
        f32x4 fw[2], fx[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            fw[t] = load_k4<BF16, VEC>(a.w, a.ldw, n0 + 16 * t + r16, N, k, K);
            fx[t] = load_k4<BF16, VEC>(a.x, a.ldx, m0 + 16 * t + r16, M, k, K);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fw[j][e], fx[i][e], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) *reinterpret_cast<f32x4 *>(&red[wave][i * 2 + j][lane][0]) = acc[i][j];
    __syncthreads();
    // wave t finishes sub-tile t = 2 i + j: lane owns row m, columns n .. n+3
    const int ti = wave >> 1, tj = wave & 1;
    f32x4 v = *reinterpret_cast<const f32x4 *>(&red[0][wave][lane][0]);
#pragma unroll
    for (int ww = 1; ww < 4; ++ww) v += *reinterpret_cast<const f32x4 *>(&red[ww][wave][lane][0]);

    const int64_t m = m0 + 16 * ti + r16;
    const int64_t nb = n0 + 16 * tj;        // first column of this wave's 16-column segment
    const int64_t n = nb + 4 * q4;
    for (int o = 0; o < a.epi.n_pre; ++o) {
        const DevOp op = a.epi.pre[o];
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
    }
    if (a.dst && m < M) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (n + e < N) st_elem(a.dst, m * a.ldd + n + e, a.dst_f32 ? FLE_F32 : dtype, v[e]);
    }
}

// ------------------------------------------------------------------ finalize passes
// One workgroup per (row, 4096-column chunk).  Every wave combines the row's partials itself
// (a handful of values, identical result in every lane), then the chunk is streamed once:
// read staged y, normalise, apply the trailing elementwise ops, round, write.
template <bool VEC>
__global__ __launch_bounds__(256) void finalize_rows(const FinArgs a) {
    const int lane = threadIdx.x & 63;
    const int dtype = a.epi.dtype;
    const bool ln = a.epi.row_kind == FLE_LAYERNORM;
    const int64_t N = a.N;
    constexpr int CHUNK = 4096;
    const int64_t c0 = int64_t(blockIdx.x) * CHUNK;
    const int64_t c1 = c0 + CHUNK < N ? c0 + CHUNK : N;
    for (int64_t row = blockIdx.y; row < a.M; row += gridDim.y) {
        float sub, mul;  // out = (y - sub) * mul  (LayerNorm),  exp(y - sub) * mul  (softmax)
        if (ln) {
            const Stat s = reduce_partials<true>(a.partials, row, a.np, a.part_cols, N, lane);
            sub = s.a;
            mul = rsqrtf(s.b / float(N) + a.epi.row.alpha);
        } else {
            const Stat s = reduce_partials<false>(a.partials, row, a.np, a.part_cols, N, lane);
            sub = s.a;
            mul = 1.0f / s.b;
        }
        auto finish = [&](float y, int64_t n) -> float {
            float v;
            if (ln) {
                v = (y - sub) * mul;
                if (a.epi.row.p0) v *= ld_elem(a.epi.row.p0, n, dtype);
                if (a.epi.row.p1) v += ld_elem(a.epi.row.p1, n, dtype);
            } else {
                v = __expf(y - sub) * mul;
            }
            for (int o = 0; o < a.epi.n_post; ++o) v = apply_op(a.epi.post[o], v, row, n, a.epi.bias, dtype);
            return v;
        };
        if (VEC) {
            for (int64_t n = c0 + int64_t(threadIdx.x) * 8; n < c1; n += 256 * 8) {
                float y[8];
                if (a.y_f32) {
                    const f32x4 *src = reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(a.y) + row * a.ldy + n);
                    const f32x4 u0 = src[0], u1 = src[1];
#pragma unroll
                    for (int e = 0; e < 4; ++e) { y[e] = u0[e]; y[4 + e] = u1[e]; }
                } else if (dtype == FLE_BF16) {
                    const uint4 u = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(a.y) + row * a.ldy + n);
                    const uint32_t wv[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) { y[2 * e] = __uint_as_float(wv[e] << 16); y[2 * e + 1] = __uint_as_float(wv[e] & 0xffff0000u); }
                } else {
                    const f32x4 *src = reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(a.y) + row * a.ldy + n);
                    const f32x4 u0 = src[0], u1 = src[1];
#pragma unroll
                    for (int e = 0; e < 4; ++e) { y[e] = u0[e]; y[4 + e] = u1[e]; }
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) y[e] = finish(y[e], n + e);
                if (dtype == FLE_BF16) {
                    bf16x8 o;
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = static_cast<__bf16>(y[e]);
                    *reinterpret_cast<bf16x8 *>(reinterpret_cast<__bf16 *>(a.out) + row * a.ldo + n) = o;
                } else {
                    f32x4 *dstp = reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(a.out) + row * a.ldo + n);
                    dstp[0] = f32x4{y[0], y[1], y[2], y[3]};
                    dstp[1] = f32x4{y[4], y[5], y[6], y[7]};
                }
            }
        } else {
            for (int64_t n = c0 + threadIdx.x; n < c1; n += 256) {
                const float y = ld_elem(a.y, row * a.ldy + n, a.y_f32 ? FLE_F32 : dtype);
                st_elem(a.out, row * a.ldo + n, dtype, finish(y, n));
            }
        }
    }
}

// logsumexp: one wave per row, out[row] = max + log(sum).
__global__ __launch_bounds__(256) void finalize_lse(const FinArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t row = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (row >= a.M) return;
    const Stat s = reduce_partials<false>(a.partials, row, a.np, a.part_cols, a.N, lane);
    if (lane == 0) st_elem(a.out, row, a.epi.dtype, s.a + __logf(s.b));
}

// ------------------------------------------------------------------ launcher
static fle_status check_launch(const char *what) {
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return fail(FLE_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
    return FLE_OK;
}

fle_status launch(const fle_problem *p, const Plan &plan) {
    hipStream_t stream = reinterpret_cast<hipStream_t>(p->stream);
    const DevEpilogue &e = plan.epi;
    char *ws = reinterpret_cast<char *>(p->workspace);
    const bool bf16 = p->dtype == FLE_BF16;
    const size_t es = bf16 ? 2 : 4;

    GemmArgs g{};
    g.M = p->M; g.N = p->N; g.K = p->K;
    g.x = p->x; g.ldx = p->ldx; g.w = p->w; g.ldw = p->ldw;
    g.np = plan.np;
    g.partials = e.row_kind >= 0 ? reinterpret_cast<float *>(ws + plan.ws_part_off) : nullptr;
    g.tiles_m = int32_t(plan.tiles_m); g.tiles_n = int32_t(plan.tiles_n);
    g.epi = e;
    if (e.row_kind < 0 || plan.staging == ST_OUT) { g.dst = p->out; g.ldd = p->ldo; g.dst_f32 = 0; }
    else if (plan.staging == ST_WS) { g.dst = ws + plan.ws_y_off; g.ldd = p->N; g.dst_f32 = 1; }
    else { g.dst = nullptr; g.ldd = 0; g.dst_f32 = 0; }

    const uint32_t grid = uint32_t(plan.tiles_m * plan.tiles_n);
    if (plan.variant == V_TILED) {
        if (plan.bm == 256) hipLaunchKernelGGL((gemm_bf16_tiled<256, 256>), dim3(grid), dim3(256), 0, stream, g);
        else hipLaunchKernelGGL((gemm_bf16_tiled<128, 128>), dim3(grid), dim3(256), 0, stream, g);
    } else {
        // vector loads need 4-element groups that never straddle K and rows that keep the alignment
        const size_t va = bf16 ? 8 : 16;
        const bool vec = p->K % 4 == 0 && reinterpret_cast<uintptr_t>(p->x) % va == 0 && reinterpret_cast<uintptr_t>(p->w) % va == 0 &&
                         p->ldx % 4 == 0 && p->ldw % 4 == 0;
        if (bf16) {
            if (vec) hipLaunchKernelGGL((gemm_general<true, true>), dim3(grid), dim3(256), 0, stream, g);
            else hipLaunchKernelGGL((gemm_general<true, false>), dim3(grid), dim3(256), 0, stream, g);
        } else {
            if (vec) hipLaunchKernelGGL((gemm_general<false, true>), dim3(grid), dim3(256), 0, stream, g);
            else hipLaunchKernelGGL((gemm_general<false, false>), dim3(grid), dim3(256), 0, stream, g);
        }
    }
    fle_status s = check_launch("GEMM kernel launch");
    if (s != FLE_OK || e.row_kind < 0) return s;

    FinArgs f{};
    f.M = p->M; f.N = p->N;
    f.np = plan.np; f.part_cols = plan.part_cols;
    f.partials = g.partials;
    f.out = p->out; f.ldo = p->ldo;
    f.epi = e;
    if (e.row_kind == FLE_LOGSUMEXP) {
        hipLaunchKernelGGL(finalize_lse, dim3(uint32_t((p->M + 3) / 4)), dim3(256), 0, stream, f);
        return check_launch("logsumexp finalize launch");
    }
    f.y = g.dst; f.ldy = g.ldd; f.y_f32 = g.dst_f32;
    const size_t ysz = f.y_f32 ? 4 : es;
    const bool vec = p->N % 8 == 0 && f.ldy % 8 == 0 && p->ldo % 8 == 0 && reinterpret_cast<uintptr_t>(f.y) % (8 * ysz) == 0 &&
                     reinterpret_cast<uintptr_t>(p->out) % (8 * es) == 0;
    const dim3 fgrid(uint32_t((p->N + 4095) / 4096), uint32_t(p->M < 65535 ? p->M : 65535));
    if (vec) hipLaunchKernelGGL(finalize_rows<true>, fgrid, dim3(256), 0, stream, f);
    else hipLaunchKernelGGL(finalize_rows<false>, fgrid, dim3(256), 0, stream, f);
    return check_launch("row finalize launch");
}

}  // namespace fle
