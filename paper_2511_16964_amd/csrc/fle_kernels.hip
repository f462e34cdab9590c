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

#include <type_traits>

#include "fle_plan.h"

namespace fle {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
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
    int32_t dst_rel;  // softmax staged in bf16: store v - (maximum of v's partial), which is <= 0 and keeps exp() accurate
    int32_t np;       // row-reduction partials per row
    float *partials;  // [M][np][2], or nullptr without a row op
    int32_t tiles_m, tiles_n;
    int64_t split_stride;  // split K (gridDim.y > 1): workgroup row y owns a K range and writes dst + y * split_stride bytes
    DevEpilogue epi;
};

// Sum of the split-K slabs followed by the ops before the row op (reduce_slabs).
struct RedArgs {
    int64_t M, N;
    const float *slabs;  // [S][M][N] fp32
    int64_t stride;      // elements between slabs
    int64_t ld_slab;     // elements between slab rows (N rounded up to a multiple of 4)
    int32_t S;
    int32_t vec;         // b, residual and dst allow 4-column vector accesses
    int32_t dst_f32;
    int32_t dst_rel;     // as GemmArgs::dst_rel
    void *dst;           // as GemmArgs::dst
    int64_t ldd;
    int32_t np;
    float *partials;     // one partial per (row, 256 columns)
    DevEpilogue epi;
};

struct FinArgs {
    int64_t M, N;
    const void *y;  // staged values: storage dtype (may alias out) or fp32
    int64_t ldy;
    int32_t y_f32;
    int32_t y_rel;  // staged values are relative to the maximum of their partial (bf16 softmax)
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
    if (dtype == FLE_F16) return float(reinterpret_cast<const _Float16 *>(p)[i]);
    return reinterpret_cast<const float *>(p)[i];
}

__device__ __forceinline__ void st_elem(void *p, int64_t i, int dtype, float v) {
    if (dtype == FLE_BF16)
        reinterpret_cast<__bf16 *>(p)[i] = static_cast<__bf16>(v);
    else if (dtype == FLE_F16)
        reinterpret_cast<_Float16 *>(p)[i] = static_cast<_Float16>(v);
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

// 4 consecutive elements at element index i of p as fp32 (p + i aligned to 4 elements).  DT: fle_dtype.
template <int DT>
__device__ __forceinline__ f32x4 ld4(const void *p, int64_t i) {
    if constexpr (DT == FLE_F32) return *reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(p) + i);
    else if constexpr (DT == FLE_F16) return __builtin_convertvector(*reinterpret_cast<const f16x4 *>(reinterpret_cast<const _Float16 *>(p) + i), f32x4);
    else return ld4_bf16(reinterpret_cast<const uint16_t *>(p) + i);
}
__device__ __forceinline__ f32x4 ld4_rt(const void *p, int64_t i, int dtype) {  // dtype known at run time only
    if (dtype == FLE_F32) return ld4<FLE_F32>(p, i);
    if (dtype == FLE_F16) return ld4<FLE_F16>(p, i);
    return ld4<FLE_BF16>(p, i);
}

// 4 fp32 values rounded (to nearest even) to a 2-byte dtype and packed into 8 bytes.
template <int DT>
__device__ __forceinline__ u32x2 pack4(f32x4 v) {
    static_assert(DT == FLE_BF16 || DT == FLE_F16, "2-byte dtypes only");
    if constexpr (DT == FLE_F16) return __builtin_bit_cast(u32x2, __builtin_convertvector(v, f16x4));
    else return __builtin_bit_cast(u32x2, __builtin_convertvector(v, bf16x4));
}
__device__ __forceinline__ u32x2 pack4_rt(f32x4 v, int dtype) { return dtype == FLE_F16 ? pack4<FLE_F16>(v) : pack4<FLE_BF16>(v); }

__device__ __forceinline__ float relu_f(float v) { return v < 0.0f ? 0.0f : v; }  // NaN stays NaN

// GELU with the exact-erf definition.  erfc(|x|) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-x^2),
// t = 1 / (1 + p |x|)  (Abramowitz & Stegun 7.1.26, |error| <= 1.5e-7), and
// 1 + erf(x) = erfc(|x|) for x < 0, 2 - erfc(|x|) otherwise: no cancellation in the left tail.
__device__ __forceinline__ float gelu_erf_f(float v) {
    const float x = fabsf(v) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float p = fmaf(t, 1.061405429f, -1.453152027f);
    p = fmaf(t, p, 1.421413741f);
    p = fmaf(t, p, -0.284496736f);
    p = fmaf(t, p, 0.254829592f);
    const float c = p * t * __expf(-x * x);
    return 0.5f * v * (v < 0.0f ? c : 2.0f - c);
}

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
// LayerNorm: Chan's update, lane-serial then a butterfly.  Softmax / logsumexp: the row maximum first
// (exact in any order), then every partial sum rescaled to it once and added lane-serially and by
// butterfly: one exp per partial instead of two per pairwise combine.
template <bool LN>
__device__ __forceinline__ Stat reduce_partials(const float *partials, int64_t row, int np, int part_cols, int64_t N, int lane) {
    Stat s;
    s.n = 0.0f;
    s.a = LN ? 0.0f : -INFINITY;
    s.b = 0.0f;
    const float *pr = partials + row * np * 2;
    if (LN) {  // few partials per row (N / 64 or fewer): one load per lane and round
        for (int p = lane; p < np; p += 64) {
            Stat q;
            const int64_t left = N - int64_t(p) * part_cols;
            q.n = float(left < part_cols ? left : part_cols);
            q.a = pr[2 * p];
            q.b = pr[2 * p + 1];
            s = combine_ln(s, q);
        }
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            Stat o;
            o.n = __shfl_xor(s.n, d);
            o.a = __shfl_xor(s.a, d);
            o.b = __shfl_xor(s.b, d);
            const bool upper = (lane & d) != 0;  // both partners combine (lower lane, upper lane): identical results
            const Stat lo = upper ? o : s, hi = upper ? s : o;
            s = combine_ln(lo, hi);
        }
        return s;
    }
    // softmax / logsumexp: a lane takes partials lane, lane + 64, ...; up to 16 loads go out together so
    // that their latencies overlap (a row of a 32768-column softmax has 1024 partials, 16 per lane)
    constexpr int B = 16;
    if (np <= 64 * B) {  // one batch: keep the partials in registers between the two sweeps
        float2 buf[B];
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const int p = j * 64 + lane;
            buf[j] = make_float2(-INFINITY, 0.0f);
            if (j * 64 < np && p < np) buf[j] = *reinterpret_cast<const float2 *>(pr + 2 * p);  // outer test is wave-uniform
        }
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < B; ++j) mx = fmaxf(mx, buf[j].x);
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) mx = fmaxf(mx, __shfl_xor(mx, d));
        float sum = 0.0f;
#pragma unroll
        for (int j = 0; j < B; ++j)
            if (j * 64 < np && buf[j].y != 0.0f) sum += buf[j].y * __expf(buf[j].x - mx);
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) sum += __shfl_xor(sum, d);  // partners add the same two numbers: identical in every lane
        s.a = mx;
        s.b = sum;
        return s;
    }
    float mx = -INFINITY;
    for (int p = lane; p < np; p += 64) mx = fmaxf(mx, pr[2 * p]);
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) mx = fmaxf(mx, __shfl_xor(mx, d));
    float sum = 0.0f;
    for (int p = lane; p < np; p += 64) {
        const float2 q = *reinterpret_cast<const float2 *>(pr + 2 * p);
        if (q.y != 0.0f) sum += q.y * __expf(q.x - mx);
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) sum += __shfl_xor(sum, d);
    s.a = mx;
    s.b = sum;
    return s;
}

// ------------------------------------------------------------------ tiled MFMA GEMM (bf16 and fp32)
// Block tile BM x BN (rows of x, rows of W), K step 128 bytes (64 bf16 or 32 fp32), 4 waves as
// 2 x 2, each wave owning (BM/2) x (BN/2) outputs as 32x32 accumulator tiles of
// v_mfma_f32_32x32x16_bf16 (fp32 operands: four v_mfma_f32_32x32x2_f32 per fragment pair).
//
// Main loop.  Operand tiles go HBM -> LDS by buffer loads that write LDS directly (no
// registers), two stages deep.  A stage row is 128 bytes = 8 chunks of 16 bytes, stored at chunk
// position c ^ g(row), g(row) = (row & 7) ^ ((row >> 3) & 1): the 16-byte reads of an MFMA
// fragment (32 consecutive rows, one logical chunk) then hit every LDS bank once.  Within a
// K step the copy instructions for the next stage and the fragment reads for the next
// 16-wide k slice are issued one at a time in the gaps between MFMAs (pinned with
// sched_barrier): a wave issues in order, so a burst of memory instructions would otherwise
// leave the matrix pipe idle while the LDS and texture paths accept them.  The copies all go
// out in the first half of the K step, which gives them most of a K step to land.
//
// Epilogue.  One 32-row block of the wave's accumulators at a time is staged through LDS as
// fp32 and read back row-contiguous: a lane then owns 4 (or 2 x 4) consecutive columns of one
// row, 16 lanes cover a whole 64-column run, so bias / residual / output accesses are full
// cache lines and a row reduction is a 16-lane DPP reduction.  The residual tile is copied
// into LDS by the same direct loads, the first block before the main loop starts.
template <int ROWS>
struct TileLoader {
    static constexpr int NI = ROWS / 32;  // copy instructions per wave per stage (8 rows each)
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t off_even, off_odd;  // this lane's byte offset in the tile for its even / odd 8-row groups
    uint32_t row_step;           // bytes between 8-row groups
    int wave;
    int chunk_even;              // logical 16-byte chunk (0..7) this lane copies in its even groups (odd: ^ 1)

    // ld_bytes: distance between rows; k_bytes: length of a row (K elements), both in bytes
    __device__ __forceinline__ void init(const void *base, int64_t ld_bytes, int64_t rows_valid, int64_t k_bytes, int wave_, int lane) {
        const int64_t rv = rows_valid < ROWS ? rows_valid : ROWS;
        const uint32_t nrec = uint32_t((rv - 1) * ld_bytes + k_bytes);
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, nrec, 0x00020000);
        const int lr = lane >> 3, lp = lane & 7;
        const uint32_t ldb = uint32_t(ld_bytes);
        wave = wave_;
        const int p0 = (wave_ * (ROWS / 4) / 8) & 1;  // parity of this wave's first 8-row group
        off_even = uint32_t(wave_ * (ROWS / 4) + lr) * ldb + uint32_t((lp ^ lr ^ p0) << 4);
        off_odd = uint32_t(wave_ * (ROWS / 4) + lr) * ldb + uint32_t((lp ^ lr ^ p0 ^ 1) << 4);
        chunk_even = lp ^ lr ^ p0;
        row_step = 8 * ldb;
    }
    // Copy instruction j (8 rows x 128 bytes) of this wave's quarter of the tile at byte column k0.
    __device__ __forceinline__ void issue_one(char *lds, uint32_t k0, int j) const {
        const uint32_t voff = ((j & 1) ? off_odd : off_even) + uint32_t(j) * row_step + k0;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(lds + (wave * (ROWS / 4) + j * 8) * 128), 16, voff, 0, 0, 0);
    }
    // Same for the last, partial K step: chunks at or beyond `valid` (= remaining row bytes / 16) get
    // an out-of-range offset, for which the buffer load delivers zeros.
    __device__ __forceinline__ void issue_one_tail(char *lds, uint32_t k0, int j, int valid) const {
        uint32_t voff = ((j & 1) ? off_odd : off_even) + uint32_t(j) * row_step + k0;
        if ((chunk_even ^ (j & 1)) >= valid) voff = 0x80000000u;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(lds + (wave * (ROWS / 4) + j * 8) * 128), 16, voff, 0, 0, 0);
    }
    __device__ __forceinline__ void issue(char *lds, uint32_t k0, int valid) const {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            if (valid >= 8) issue_one(lds, k0, j);
            else issue_one_tail(lds, k0, j, valid);
        }
    }
};

template <int N>
__device__ __forceinline__ void wait_vmcnt() {  // s_waitcnt vmcnt(N), other counters untouched
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

// Sum / max over the 16 lanes of a DPP row by rotations; every lane ends with the result.
template <bool MAX>
__device__ __forceinline__ float row16_allreduce(float v) {
#define FLE_ROR(n)                                                                                              \
    {                                                                                                           \
        const float o = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + (n), 0xF, 0xF, false)); \
        v = MAX ? fmaxf(v, o) : v + o;                                                                          \
    }
    FLE_ROR(8) FLE_ROR(4) FLE_ROR(2) FLE_ROR(1)
#undef FLE_ROR
    return v;
}

// EDGE: N, the leading dimensions or the addresses of b / residual / out do not allow 4-column vector
// accesses; the epilogue then touches memory one element at a time, masked per column.
template <int BM, int BN, int DT, bool EDGE>
__device__ __forceinline__ void gemm_tiled_body(const GemmArgs &a) {
    constexpr bool F32 = DT == FLE_F32;
    constexpr int ES = F32 ? 4 : 2;  // bytes per operand element; a staged row is 128 bytes = 64 bf16 or 32 fp32
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    constexpr int SW = BN * 128, SX = BM * 128, STAGE = SW + SX;  // bytes per stage
    constexpr int NH = WN / 64;                                    // 64-column runs per wave tile
    constexpr int EP_STRIDE = WN * 4 + 16;                         // staged fp32 row + 16 bytes of bank skew
    constexpr int EP_WAVE = 32 * EP_STRIDE;
    constexpr int RES_WAVE = 32 * WN * 2;                          // one 32-row residual block per wave
    constexpr int RES1_OFF = 4 * EP_WAVE, RES0_OFF = 2 * STAGE;
    static_assert(RES1_OFF + 4 * RES_WAVE <= 2 * STAGE, "epilogue buffers must fit in the stage area");
    __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE + 4 * RES_WAVE];

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
    const int64_t m_wave = m0 + wm * WM, n_wave = n0 + wn * WN;  // origin of this wave's outputs

    // ---- residual operand of the first RESIDUAL op whose rows are 16-byte aligned: copied to LDS
    // block by block (other residual operands are read straight from memory in the epilogue)
    int res_idx = -1;
    bool has_bias = false;
    for (int o = a.epi.n_pre - 1; o >= 0; --o) {
        const DevOp &op = a.epi.pre[o];
        if (!F32 && !EDGE && op.kind == FLE_RESIDUAL && op.ld % 8 == 0 && reinterpret_cast<uintptr_t>(op.p0) % 16 == 0) res_idx = o;
        if (op.kind == FLE_BIAS) has_bias = true;
    }
    const bool wave_live = m_wave < M && n_wave < N;  // this wave owns at least one output
    __amdgpu_buffer_rsrc_t res_rsrc = __builtin_amdgcn_make_buffer_rsrc(nullptr, 0, 0, 0x00020000);
    uint32_t res_lane_off = 0, res_block_step = 0;
    if (res_idx >= 0 && wave_live) {
        const int64_t ld = a.epi.pre[res_idx].ld;
        const int64_t rows = (M - m_wave) < WM ? (M - m_wave) : WM;
        const char *base = reinterpret_cast<const char *>(a.epi.pre[res_idx].p0) + (m_wave * ld + n_wave) * 2;
        res_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(base), 0, uint32_t(((rows - 1) * ld + (N - n_wave)) * 2), 0x00020000);
        // copy instruction t of a block covers rows 4t .. 4t+3 when WN = 128 (16 lanes x 16 bytes per row),
        // rows 8t .. 8t+7 when WN = 64
        constexpr int LPR = WN / 8;  // lanes per row
        res_lane_off = uint32_t(lane / LPR) * uint32_t(ld) * 2 + uint32_t(lane % LPR) * 16;
        res_block_step = uint32_t(64 / LPR) * uint32_t(ld) * 2;
    }
    auto issue_residual = [&](int block, int buf) {
        constexpr int NI = RES_WAVE / 1024;
        char *dst = smem + (buf ? RES1_OFF : RES0_OFF) + wave * RES_WAVE;
        const uint32_t base = uint32_t(block) * 32 * uint32_t(a.epi.pre[res_idx].ld) * 2 + res_lane_off;
#pragma unroll
        for (int t = 0; t < NI; ++t)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(res_rsrc, (lds_void *)(dst + t * 1024), 16, base + uint32_t(t) * res_block_step, 0, 0, 2);  // read once: non-temporal
    };
    if (res_idx >= 0 && wave_live) issue_residual(0, 0);

    TileLoader<BM> ldx_;
    TileLoader<BN> ldw_;
    ldx_.init(reinterpret_cast<const char *>(a.x) + m0 * a.ldx * ES, a.ldx * ES, M - m0, a.K * ES, wave, lane);
    ldw_.init(reinterpret_cast<const char *>(a.w) + n0 * a.ldw * ES, a.ldw * ES, N - n0, a.K * ES, wave, lane);
    constexpr int NIW = TileLoader<BN>::NI, NIX = TileLoader<BM>::NI;

    // Fragment read offsets: lane reads row (lane & 31) of a 32-row block, logical chunk 2*kk + (lane >> 5).
    uint32_t rd_off[4];
    {
        const int g = (lane & 7) ^ ((lane >> 3) & 1), hh = lane >> 5;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) rd_off[kk] = uint32_t((lane & 31) * 128 + (((2 * kk + hh) ^ g) << 4));
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // 16 bytes of one row: 4 fp32, 8 bf16 or 8 fp16 along K
    using frag_t = typename std::conditional<F32, f32x4, typename std::conditional<DT == FLE_F16, f16x8, bf16x8>::type>::type;
    frag_t fw[2][TN], fx[2][TM];
    const int KT = int((a.K * ES + 127) / 128);
    const int tail_valid = int((a.K * ES - int64_t(KT - 1) * 128) / 16);  // 16-byte chunks of the last K step (8 = full)
    // One K step on stage kt & 1; ISSUE: also copy K step kt+1 into the other stage (masked to the
    // valid chunks when that is the partial last step).
    auto k_step = [&](int kt, auto issue_c) {
        constexpr bool ISSUE = decltype(issue_c)::value;
        const int valid = kt + 2 == KT ? tail_valid : 8;
        const char *sW = smem + (kt & 1) * STAGE, *sX = sW + SW;
        char *iW = smem + ((kt + 1) & 1) * STAGE, *iX = iW + SW;
        const uint32_t ik0 = uint32_t(kt + 1) * 128;  // byte column of the K step being copied
        wait_vmcnt<0>();                  // this wave's copies into the current stage have landed
        __builtin_amdgcn_s_barrier();     // everyone's have, and everyone is done reading the other stage
#pragma unroll
        for (int t = 0; t < TN; ++t) fw[0][t] = *reinterpret_cast<const frag_t *>(sW + (wn * WN + t * 32) * 128 + rd_off[0]);
#pragma unroll
        for (int t = 0; t < TM; ++t) fx[0][t] = *reinterpret_cast<const frag_t *>(sX + (wm * WM + t * 32) * 128 + rd_off[0]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            // 16-wide k slice kk: NMF MFMAs; in the issue slot before MFMA q goes at most one
            // fragment read of slice kk+1 and (first two slices only) one copy instruction.
            constexpr int NMF = TM * TN, NDS = TM + TN, NVM = (NIW + NIX) / 2;
            constexpr int QD = NMF / NDS, QV = NMF / NVM;  // MFMAs per fragment read / per copy instruction
            const int cur = kk & 1;
#pragma unroll
            for (int q = 0; q < NMF; ++q) {
                if (kk + 1 < 4 && q % QD == 0) {
                    const int g = q / QD;
                    if (g < TN) fw[cur ^ 1][g] = *reinterpret_cast<const frag_t *>(sW + (wn * WN + g * 32) * 128 + rd_off[(kk + 1) & 3]);
                    else fx[cur ^ 1][g - TN] = *reinterpret_cast<const frag_t *>(sX + (wm * WM + (g - TN) * 32) * 128 + rd_off[(kk + 1) & 3]);
                }
                if (ISSUE && kk < 2 && q % QV == (QV > 1 ? 1 : 0)) {
                    const int idx = kk * NVM + q / QV;
                    if (idx < NIW) ldw_.issue_one_tail(iW, ik0, idx, valid);
                    else ldx_.issue_one_tail(iX, ik0, idx - NIW, valid);
                }
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (F32) {
                    // four 32x32x2 steps; step e pairs element e of the two 16-byte groups of every row, the
                    // same K permutation for both operands
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        acc[q / TN][q % TN] = __builtin_amdgcn_mfma_f32_32x32x2f32(fw[cur][q % TN][e], fx[cur][q / TN][e], acc[q / TN][q % TN], 0, 0, 0);
                } else if constexpr (DT == FLE_F16) {
                    acc[q / TN][q % TN] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[cur][q % TN], fx[cur][q / TN], acc[q / TN][q % TN], 0, 0, 0);
                } else {
                    acc[q / TN][q % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[cur][q % TN], fx[cur][q / TN], acc[q / TN][q % TN], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // K steps kb .. ke-1 of this workgroup (all of them unless K is split over gridDim.y)
    const int kb = int(int64_t(blockIdx.y) * KT / gridDim.y), ke = int(int64_t(blockIdx.y + 1) * KT / gridDim.y);
    ldw_.issue(smem + (kb & 1) * STAGE, uint32_t(kb) * 128, kb + 1 == KT ? tail_valid : 8);
    ldx_.issue(smem + (kb & 1) * STAGE + SW, uint32_t(kb) * 128, kb + 1 == KT ? tail_valid : 8);
    {
        int kt = kb;
        for (; kt < ke - 1; ++kt) k_step(kt, std::true_type{});
        k_step(kt, std::false_type{});
    }
    __syncthreads();  // the stage area becomes epilogue scratch
    if (!wave_live) return;
    char *const dst = a.dst ? reinterpret_cast<char *>(a.dst) + int64_t(blockIdx.y) * a.split_stride : nullptr;

    // ---- epilogue
    // Final values are written once and not read again by this call: non-temporal stores keep them from
    // displacing operand panels in L2 (measured -2.4 % on the MLP block).  Values staged for the finalize
    // pass or the split-K reduction are re-read soon and stay cacheable (non-temporal costs +3 % there).
    const bool stream_out = a.epi.row_kind < 0 && gridDim.y == 1;
    const int rsub = lane >> 4;  // row within a group of 4 rows
    const int cl = lane & 15;
    char *ep = smem + wave * EP_WAVE;
    // columns of this lane in the read-back layout: run hc covers n_wave + 64 hc + 4 cl .. + 3
    int64_t n_col[NH];
    bool n_ok[NH];
    f32x4 bias_v[NH];
#pragma unroll
    for (int hc = 0; hc < NH; ++hc) {
        n_col[hc] = n_wave + 64 * hc + 4 * cl;
        n_ok[hc] = n_col[hc] < N;
        bias_v[hc] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (has_bias) {
            if constexpr (EDGE) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (n_col[hc] + e < N) bias_v[hc][e] = ld_elem(a.epi.bias, n_col[hc] + e, DT);
            } else {
                bias_v[hc] = ld4<DT>(a.epi.bias, n_ok[hc] ? n_col[hc] : N - 4);
            }
        }
    }
    const int p_idx = int(n_wave / WN);
    const int64_t cols_left = N - n_wave;
    const float cnt = float(cols_left < WN ? cols_left : WN);
    constexpr int NIT = 8;  // 4 rows per iteration

#pragma unroll 1
    for (int i = 0; i < TM; ++i) {
        const int64_t m_blk = m_wave + 32 * i;
        if (m_blk >= M) break;
        if (res_idx >= 0) {
            wait_vmcnt<0>();  // residual block i is in LDS (and this wave's earlier stores are done)
            if (i + 1 < TM && m_blk + 32 < M) issue_residual(i + 1, (i + 1) & 1);
        }
        // accumulators of row block i -> LDS, row (lane & 31), columns 32 j + 8 q + 4 h .. + 3
        {
            char *wr = ep + (lane & 31) * EP_STRIDE + (lane >> 5) * 16;
            auto put = [&](auto ic) {
                constexpr int I = decltype(ic)::value;
                if constexpr (I < TM) {
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            *reinterpret_cast<f32x4 *>(wr + (32 * j + 8 * q) * 4) = f32x4{acc[I][j][4 * q], acc[I][j][4 * q + 1], acc[I][j][4 * q + 2], acc[I][j][4 * q + 3]};
                }
            };
            switch (i) {
            case 0: put(std::integral_constant<int, 0>{}); break;
            case 1: put(std::integral_constant<int, 1>{}); break;
            case 2: put(std::integral_constant<int, 2>{}); break;
            default: put(std::integral_constant<int, 3>{}); break;
            }
        }
        // read back row-contiguous: v[it][hc] = row 4 it + rsub, columns of run hc
        f32x4 v[NIT][NH];
#pragma unroll
        for (int it = 0; it < NIT; ++it)
#pragma unroll
            for (int hc = 0; hc < NH; ++hc) v[it][hc] = *reinterpret_cast<const f32x4 *>(ep + (4 * it + rsub) * EP_STRIDE + hc * 256 + cl * 16);

        for (int o = 0; o < a.epi.n_pre; ++o) {
            const DevOp op = a.epi.pre[o];
            switch (op.kind) {
            case FLE_BIAS:
#pragma unroll
                for (int it = 0; it < NIT; ++it)
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc) v[it][hc] += bias_v[hc];
                break;
            case FLE_SCALE:
#pragma unroll
                for (int it = 0; it < NIT; ++it)
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc) v[it][hc] *= op.alpha;
                break;
            case FLE_RELU:
#pragma unroll
                for (int it = 0; it < NIT; ++it)
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc)
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[it][hc][e] = relu_f(v[it][hc][e]);
                break;
            case FLE_GELU_ERF:
#pragma unroll
                for (int it = 0; it < NIT; ++it)
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc)
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[it][hc][e] = gelu_erf_f(v[it][hc][e]);
                break;
            case FLE_GELU_TANH:
#pragma unroll
                for (int it = 0; it < NIT; ++it)
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc)
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[it][hc][e] = gelu_tanh_f(v[it][hc][e]);
                break;
            case FLE_RESIDUAL:
                if (o == res_idx) {  // staged in LDS: [32 rows][WN] bf16
                    const char *rb = smem + ((i & 1) ? RES1_OFF : RES0_OFF) + wave * RES_WAVE;
#pragma unroll
                    for (int it = 0; it < NIT; ++it)
#pragma unroll
                        for (int hc = 0; hc < NH; ++hc) v[it][hc] += ld4<DT>(rb + (4 * it + rsub) * (WN * 2) + hc * 128 + cl * 8, 0);
                } else {  // a further residual operand: straight from memory, clamped to stay in bounds
#pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        const int64_t m = m_blk + 4 * it + rsub;
                        const int64_t mc = m < M ? m : M - 1;
#pragma unroll
                        for (int hc = 0; hc < NH; ++hc) {
                            if constexpr (EDGE) {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (n_col[hc] + e < N) v[it][hc][e] += ld_elem(op.p0, mc * op.ld + n_col[hc] + e, DT);
                            } else {
                                v[it][hc] += ld4<DT>(op.p0, mc * op.ld + (n_ok[hc] ? n_col[hc] : N - 4));
                            }
                        }
                    }
                }
                break;
            default: break;
            }
        }

        // row-reduction partials over this wave's WN columns, from the unrounded fp32 values
        float part_max[NIT];  // softmax: the partial's maximum per row of this block
        if (a.epi.row_kind >= 0) {
            const bool ln = a.epi.row_kind == FLE_LAYERNORM;
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int64_t m = m_blk + 4 * it + rsub;
                float s0, s1;
                if (ln) {
                    float sum = 0.0f;
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc)
                        if (n_ok[hc]) {
                            if constexpr (EDGE) {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (n_col[hc] + e < N) sum += v[it][hc][e];
                            } else {
                                sum += (v[it][hc][0] + v[it][hc][1]) + (v[it][hc][2] + v[it][hc][3]);
                            }
                        }
                    sum = row16_allreduce<false>(sum);
                    const float mean = sum / cnt;
                    float m2 = 0.0f;
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc)
                        if (n_ok[hc])
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (!EDGE || n_col[hc] + e < N) m2 += (v[it][hc][e] - mean) * (v[it][hc][e] - mean);
                    m2 = row16_allreduce<false>(m2);
                    s0 = mean;
                    s1 = m2;
                } else {
                    float mx = -INFINITY;
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc)
                        if (n_ok[hc]) {
                            if constexpr (EDGE) {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (n_col[hc] + e < N) mx = fmaxf(mx, v[it][hc][e]);
                            } else {
                                mx = fmaxf(fmaxf(mx, fmaxf(v[it][hc][0], v[it][hc][1])), fmaxf(v[it][hc][2], v[it][hc][3]));
                            }
                        }
                    mx = row16_allreduce<true>(mx);
                    float se = 0.0f;
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc)
                        if (n_ok[hc])
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (!EDGE || n_col[hc] + e < N) se += __expf(v[it][hc][e] - mx);
                    se = row16_allreduce<false>(se);
                    s0 = mx;
                    s1 = se;
                }
                part_max[it] = s0;
                if (cl == 0 && m < M) *reinterpret_cast<float2 *>(a.partials + (m * a.np + p_idx) * 2) = make_float2(s0, s1);
            }
            if (a.dst_rel) {
#pragma unroll
                for (int it = 0; it < NIT; ++it)
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc) v[it][hc] -= part_max[it];
            }
        }

        // store: final values (no row op) or staged values for the finalize pass
        if (a.dst) {
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int64_t m = m_blk + 4 * it + rsub;
#pragma unroll
                for (int hc = 0; hc < NH; ++hc)
                    if (m < M && n_ok[hc]) {
                        if constexpr (EDGE) {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (n_col[hc] + e < N) st_elem(dst, m * a.ldd + n_col[hc] + e, a.dst_f32 ? FLE_F32 : DT, v[it][hc][e]);
                        } else if (F32 || a.dst_f32) {
                            f32x4 *q = reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(dst) + m * a.ldd + n_col[hc]);
                            if (stream_out) __builtin_nontemporal_store(v[it][hc], q);
                            else *q = v[it][hc];
                        } else {
                            u32x2 *q = reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(dst) + m * a.ldd + n_col[hc]);
                            constexpr int DT2 = F32 ? FLE_BF16 : DT;  // (this branch is never taken for fp32 problems)
                            if (stream_out) __builtin_nontemporal_store(pack4<DT2>(v[it][hc]), q);
                            else *q = pack4<DT2>(v[it][hc]);
                        }
                    }
            }
        }
    }
}

// 256 x 256: one workgroup per CU (160 KB of LDS, 512 registers per lane).  DT: fle_dtype of the operands.
// fp32 operands run on the same tiles: a K step is 32 elements and each fragment pair feeds four
// v_mfma_f32_32x32x2_f32 (64 cycles each), so the loop is bound by the matrix pipe with room to spare.
template <int DT, bool EDGE>
__global__ __launch_bounds__(256) void gemm_tiled_256(const GemmArgs a) { gemm_tiled_body<256, 256, DT, EDGE>(a); }
// 128 x 128: two workgroups per CU (80 KB of LDS each), so at most 256 registers per lane.
template <int DT, bool EDGE>
__global__ __launch_bounds__(256, 2) void gemm_tiled_128(const GemmArgs a) { gemm_tiled_body<128, 128, DT, EDGE>(a); }


// ------------------------------------------------------------------ skinny bf16 GEMM (M <= 64)
// HBM-bound: W streams through once and the matrix pipe is nearly idle, so the design goal is
// bytes in flight.  One workgroup owns 128 rows of W (columns of out) and all of K; each of its
// 4 waves copies and consumes its own 32 W rows, the small x tile is shared.  The LDS ring is
// NST stages of (128 + 32 TMB) x 64 bf16, NST-1 of them in flight (about 100 KB of W per CU,
// what 8 TB/s x ~2 us of latency / 256 CUs asks for).  Same swizzle and orientation as the
// tiled kernel; the wave tile is 32 TMB x 32, so the epilogue stays in the MFMA register layout.
template <int TMB, int BK, int DT>
__device__ __forceinline__ void gemm_bf16_skinny_body(const GemmArgs &a) {
    static_assert(DT == FLE_BF16 || DT == FLE_F16, "2-byte operands only");
    using frag_t = typename std::conditional<DT == FLE_F16, f16x8, bf16x8>::type;
    constexpr int BM = 32 * TMB, BN = 128;
    constexpr int RB = BK * 2;                 // bytes per staged row
    constexpr int CPR = BK / 8, RPI = 64 / CPR;  // 16-byte chunks per row, rows per copy instruction
    constexpr int KPS = BK / 16;               // 16-wide k slices per stage
    constexpr int SW = BN * RB, SX = BM * RB, STAGE = SW + SX;
    constexpr int NST = (160 * 1024) / STAGE < 8 ? (160 * 1024) / STAGE : 8;
    constexpr int NIW = 32 / RPI, NIX = (8 * TMB) / RPI, LPS = NIW + NIX;  // copy instructions per wave per stage
    static_assert(NST >= 2 && NIX >= 1 && (NST - 2) * LPS < 64, "ring does not fit the counters");
    __shared__ __attribute__((aligned(1024))) char smem[NST * STAGE];
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
    auto sw = [](int row) { return BK == 64 ? ((row & 7) ^ ((row >> 3) & 1)) : (row & 15); };
    const int lr = lane / CPR, lp = lane % CPR;
    __amdgpu_buffer_rsrc_t rw, rx;
    {
        const int64_t wrows = (N - n0) < BN ? (N - n0) : BN, xrows = (M - m0) < BM ? (M - m0) : BM;
        rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(reinterpret_cast<const char *>(a.w) + n0 * a.ldw * 2), 0,
                                               uint32_t(((wrows - 1) * a.ldw + a.K) * 2), 0x00020000);
        rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(reinterpret_cast<const char *>(a.x) + m0 * a.ldx * 2), 0,
                                               uint32_t(((xrows - 1) * a.ldx + a.K) * 2), 0x00020000);
    }
    const uint32_t ldwb = uint32_t(a.ldw) * 2, ldxb = uint32_t(a.ldx) * 2;
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
                if constexpr (DT == FLE_F16) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw, fx, acc[t], 0, 0, 0);
                else acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, fx, acc[t], 0, 0, 0);
            }
        }
    };
    // K stages kt .. KT-1 of this workgroup (all of them unless K is split over gridDim.y)
    const int KA = int(a.K / BK);
    int kt = int(int64_t(blockIdx.y) * KA / gridDim.y);
    const int KT = int(int64_t(blockIdx.y + 1) * KA / gridDim.y);
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
                    if (a.dst_f32)
                        *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(dst) + m * a.ldd + n) = v;
                    else
                        *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(dst) + m * a.ldd + n) = pack4<DT>(v);
                }
            }
        }
    }
}
template <int TMB, int BK, int DT>
__global__ __launch_bounds__(256) void gemm_bf16_skinny(const GemmArgs a) { gemm_bf16_skinny_body<TMB, BK, DT>(a); }

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

// ------------------------------------------------------------------ finalize passes
// One wave per (row, 2048-column chunk).  The wave combines the row's partials itself (one
// per lane, then a fixed butterfly: identical result in every lane), issues all of its
// 16-byte loads of staged y at once, normalises, applies the trailing elementwise ops, rounds
// and writes 16-byte vectors.
__device__ __forceinline__ void ld8(const void *p, int64_t i, int dtype, float (&v)[8]) {  // 8 elements at index i
    if (dtype == FLE_F32) {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(p) + i);
        const f32x4 u0 = src[0], u1 = src[1];
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[e] = u0[e]; v[4 + e] = u1[e]; }
    } else if (dtype == FLE_F16) {
        const f16x8 u = *reinterpret_cast<const f16x8 *>(reinterpret_cast<const _Float16 *>(p) + i);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = float(u[e]);
    } else {
        const uint4 u = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(p) + i);
        const uint32_t wv[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[2 * e] = __uint_as_float(wv[e] << 16); v[2 * e + 1] = __uint_as_float(wv[e] & 0xffff0000u); }
    }
}
// 8 fp32 values rounded to a 2-byte dtype, stored as one 16-byte vector at element index i.
__device__ __forceinline__ void st8_2byte(void *p, int64_t i, int dtype, const float (&v)[8]) {
    u32x4 o;
    if (dtype == FLE_F16) {
        f16x8 h;
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = static_cast<_Float16>(v[e]);
        o = __builtin_bit_cast(u32x4, h);
    } else {
        bf16x8 h;
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = static_cast<__bf16>(v[e]);
        o = __builtin_bit_cast(u32x4, h);
    }
    *reinterpret_cast<u32x4 *>(reinterpret_cast<uint16_t *>(p) + i) = o;
}

// LNK: LayerNorm (true) or softmax (false); separate kernels so that each gets its own register budget.
template <bool VEC, bool LNK>
__global__ __launch_bounds__(256) void finalize_rows(const FinArgs a) {
    constexpr int CH = 2048, IT = CH / 512;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int dtype = a.epi.dtype;
    const bool f32 = dtype == FLE_F32;
    constexpr bool ln = LNK;
    const int64_t N = a.N;
    const int64_t chunks = (N + CH - 1) / CH, items = a.M * chunks;
    for (int64_t item = int64_t(blockIdx.x) * 4 + wave; item < items; item += int64_t(gridDim.x) * 4) {
        const int64_t row = item / chunks, c0 = (item % chunks) * CH;
        const int64_t c1 = c0 + CH < N ? c0 + CH : N;
        float y[IT][8];
        if (VEC) {  // issue the loads before the partials are combined
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                const int64_t n = c0 + it * 512 + lane * 8;
                if (n < c1) ld8(a.y, row * a.ldy + n, a.y_f32 ? FLE_F32 : dtype, y[it]);
            }
        }
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
        auto post = [&](float v, int64_t n) -> float {
            for (int o = 0; o < a.epi.n_post; ++o) v = apply_op(a.epi.post[o], v, row, n, a.epi.bias, dtype);
            return v;
        };
        if (VEC) {
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                const int64_t n = c0 + it * 512 + lane * 8;
                if (n < c1) {
                    float *v = y[it];
                    if (ln) {
                        float g[8], be[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) { g[e] = 1.0f; be[e] = 0.0f; }
                        if (a.epi.row.p0) ld8(a.epi.row.p0, n, dtype, g);
                        if (a.epi.row.p1) ld8(a.epi.row.p1, n, dtype, be);
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = (v[e] - sub) * mul * g[e] + be[e];
                    } else {
                        // staged relative to the maximum of the partial the 8 columns lie in (part_cols is a multiple of 8)
                        const float shift = a.y_rel ? sub - a.partials[(row * a.np + n / a.part_cols) * 2] : sub;
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = __expf(v[e] - shift) * mul;
                    }
                    if (a.epi.n_post > 0) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = post(v[e], n + e);
                    }
                    if (f32) {
                        f32x4 *dstp = reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(a.out) + row * a.ldo + n);
                        dstp[0] = f32x4{v[0], v[1], v[2], v[3]};
                        dstp[1] = f32x4{v[4], v[5], v[6], v[7]};
                    } else {
                        st8_2byte(a.out, row * a.ldo + n, dtype, y[it]);
                    }
                }
            }
        } else {
            auto one = [&](int64_t n) {  // one element
                const float yv = ld_elem(a.y, row * a.ldy + n, a.y_f32 ? FLE_F32 : dtype);
                float v;
                if (ln) {
                    v = (yv - sub) * mul;
                    if (a.epi.row.p0) v *= ld_elem(a.epi.row.p0, n, dtype);
                    if (a.epi.row.p1) v += ld_elem(a.epi.row.p1, n, dtype);
                } else {
                    const float shift = a.y_rel ? sub - a.partials[(row * a.np + n / a.part_cols) * 2] : sub;
                    v = __expf(yv - shift) * mul;
                }
                st_elem(a.out, row * a.ldo + n, dtype, post(v, n));
            };
            // bf16 rows whose staged values and outputs share their offset within a 16-byte line (always so
            // when staged in out itself): skip h elements to the next line boundary, then whole lines as
            // 16-byte vectors.  Chunk k takes elements h + 2048 k ... of the row, chunk 0 also the first h.
            const uintptr_t ya = reinterpret_cast<uintptr_t>(a.y) + uintptr_t(row * a.ldy) * 2;
            const uintptr_t oa = reinterpret_cast<uintptr_t>(a.out) + uintptr_t(row * a.ldo) * 2;
            if (!f32 && !a.y_f32 && ((ya ^ oa) & 15) == 0 && (ya & 1) == 0) {
                const int h = int(((16 - (ya & 15)) & 15) >> 1);
                if (c0 == 0 && lane < h && lane < N) one(lane);
#pragma unroll
                for (int it = 0; it < IT; ++it) {
                    const int64_t n = h + c0 + (it * 64 + lane) * 8;
                    if (n + 8 <= N) {
                        float v[8];
                        ld8(a.y, row * a.ldy + n, dtype, v);
                        if (ln) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                v[e] = (v[e] - sub) * mul;
                                if (a.epi.row.p0) v[e] *= ld_elem(a.epi.row.p0, n + e, dtype);
                                if (a.epi.row.p1) v[e] += ld_elem(a.epi.row.p1, n + e, dtype);
                            }
                        } else {
                            float s0 = sub, s1 = sub;
                            const int64_t p0 = n / a.part_cols, p1 = (n + 7) / a.part_cols;  // the 8 columns may straddle two partials
                            if (a.y_rel) {
                                s0 = sub - a.partials[(row * a.np + p0) * 2];
                                s1 = sub - a.partials[(row * a.np + p1) * 2];
                            }
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] = __expf(v[e] - ((n + e) / a.part_cols == p0 ? s0 : s1)) * mul;
                        }
                        if (a.epi.n_post > 0) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] = post(v[e], n + e);
                        }
                        st8_2byte(a.out, row * a.ldo + n, dtype, v);
                    } else {
                        for (int64_t nn = n; nn < N; ++nn) one(nn);  // the row's last, partial line (one lane at most)
                    }
                }
            } else {
                for (int64_t n = c0 + lane; n < c1; n += 64) one(n);
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

// ------------------------------------------------------------------ split-K reduction
// One wave per (row, 256-column chunk), a lane per 4 consecutive columns: sums the S fp32 slabs
// in slab order, applies the ops that precede the row op, writes the value (final, or staged
// for the finalize pass) and, with a row op, the chunk's partial.
template <bool MAX>
__device__ __forceinline__ float wave_allreduce(float v) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float o = __shfl_xor(v, d);
        v = MAX ? fmaxf(v, o) : v + o;
    }
    return v;
}

__global__ __launch_bounds__(256) void reduce_slabs(const RedArgs a) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t N = a.N;
    const int dtype = a.epi.dtype;
    const bool f32 = dtype == FLE_F32;
    const bool vec = a.vec != 0;  // 4-column vector accesses to b, residual and dst are possible
    const int64_t chunks = (N + 255) / 256, items = a.M * chunks;
    for (int64_t item = int64_t(blockIdx.x) * 4 + wave; item < items; item += int64_t(gridDim.x) * 4) {
        const int64_t row = item / chunks, c0 = (item % chunks) * 256;
        const int64_t n = c0 + lane * 4;
        const bool ok = n < N;  // at least the first of this lane's four columns exists
        bool okc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) okc[e] = n + e < N;
        f32x4 v = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (ok) {
            const float *src = a.slabs + row * a.ld_slab + n;  // slab rows are padded to whole groups of four
            int s = 0;
            for (; s + 4 <= a.S; s += 4) {
                const f32x4 u0 = *reinterpret_cast<const f32x4 *>(src + (s + 0) * a.stride);
                const f32x4 u1 = *reinterpret_cast<const f32x4 *>(src + (s + 1) * a.stride);
                const f32x4 u2 = *reinterpret_cast<const f32x4 *>(src + (s + 2) * a.stride);
                const f32x4 u3 = *reinterpret_cast<const f32x4 *>(src + (s + 3) * a.stride);
                v = (((v + u0) + u1) + u2) + u3;
            }
            for (; s < a.S; ++s) v += *reinterpret_cast<const f32x4 *>(src + s * a.stride);
            auto add4 = [&](const void *ptr, int64_t idx) {
                if (vec) {
                    v += ld4_rt(ptr, idx, dtype);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (okc[e]) v[e] += ld_elem(ptr, idx + e, dtype);
                }
            };
            for (int o = 0; o < a.epi.n_pre; ++o) {
                const DevOp op = a.epi.pre[o];
                switch (op.kind) {
                case FLE_BIAS: add4(a.epi.bias, n); break;
                case FLE_SCALE: v *= op.alpha; break;
                case FLE_RELU:
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = relu_f(v[e]);
                    break;
                case FLE_GELU_ERF:
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = gelu_erf_f(v[e]);
                    break;
                case FLE_GELU_TANH:
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = gelu_tanh_f(v[e]);
                    break;
                case FLE_RESIDUAL: add4(op.p0, row * op.ld + n); break;
                default: break;
                }
            }
        }
        if (a.epi.row_kind >= 0) {
            float s0, s1;
            if (a.epi.row_kind == FLE_LAYERNORM) {
                const float cnt = float(N - c0 < 256 ? N - c0 : 256);
                float sum = 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (okc[e]) sum += v[e];
                const float mean = wave_allreduce<false>(sum) / cnt;
                float m2 = 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (okc[e]) m2 += (v[e] - mean) * (v[e] - mean);
                s0 = mean;
                s1 = wave_allreduce<false>(m2);
            } else {
                float mx = -INFINITY;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (okc[e]) mx = fmaxf(mx, v[e]);
                mx = wave_allreduce<true>(mx);
                float se = 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (okc[e]) se += __expf(v[e] - mx);
                s0 = mx;
                s1 = wave_allreduce<false>(se);
            }
            if (lane == 0) *reinterpret_cast<float2 *>(a.partials + (row * a.np + c0 / 256) * 2) = make_float2(s0, s1);
            if (a.dst_rel) v -= s0;
        }
        if (a.dst && ok) {
            const bool d32 = a.dst_f32 || f32;
            if (!vec) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (okc[e]) st_elem(a.dst, row * a.ldd + n + e, d32 ? FLE_F32 : dtype, v[e]);
            } else if (d32) {
                *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(a.dst) + row * a.ldd + n) = v;
            } else {
                *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(a.dst) + row * a.ldd + n) = pack4_rt(v, dtype);
            }
        }
    }
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
    const bool bf16 = p->dtype != FLE_F32;  // 2-byte operands (bf16 or fp16)
    const size_t es = bf16 ? 2 : 4;

    GemmArgs g{};
    g.M = p->M; g.N = p->N; g.K = p->K;
    g.x = p->x; g.ldx = p->ldx; g.w = p->w; g.ldw = p->ldw;
    g.np = plan.np;
    g.partials = e.row_kind >= 0 ? reinterpret_cast<float *>(ws + plan.ws_part_off) : nullptr;
    g.tiles_m = int32_t(plan.tiles_m); g.tiles_n = int32_t(plan.tiles_n);
    g.epi = e;
    if (e.row_kind < 0 || plan.staging == ST_OUT) { g.dst = p->out; g.ldd = p->ldo; g.dst_f32 = 0; g.dst_rel = plan.stage_rel; }
    else if (plan.staging == ST_WS) { g.dst = ws + plan.ws_y_off; g.ldd = p->N; g.dst_f32 = 1; }
    else { g.dst = nullptr; g.ldd = 0; g.dst_f32 = 0; }

    // Split K: the GEMM writes bare fp32 slabs; reduce_slabs takes over dst, the pre-ops and the partials.
    RedArgs r{};
    const bool split = plan.split_k > 1;
    if (split) {
        r.M = p->M; r.N = p->N;
        r.slabs = reinterpret_cast<const float *>(ws + plan.ws_slab_off);
        r.ld_slab = (p->N + 3) / 4 * 4;
        r.stride = p->M * r.ld_slab;
        r.vec = plan.edge ? 0 : 1;
        r.S = plan.split_k;
        r.dst = g.dst; r.ldd = g.ldd; r.dst_f32 = g.dst_f32; r.dst_rel = g.dst_rel;
        r.np = plan.np; r.partials = g.partials;
        r.epi = e;
        g.dst = ws + plan.ws_slab_off; g.ldd = r.ld_slab; g.dst_f32 = 1; g.dst_rel = 0;
        g.split_stride = r.stride * int64_t(sizeof(float));
        g.partials = nullptr;
        g.epi.n_pre = 0; g.epi.n_post = 0; g.epi.row_kind = -1;
    }
    // skinny kernel: W tiles in groups of 8 (one per XCD), each with all its row blocks
    const int64_t wgs = plan.variant == V_SKINNY ? (plan.tiles_n + 7) / 8 * 8 * plan.tiles_m : plan.tiles_m * plan.tiles_n;
    const dim3 grid{uint32_t(wgs), uint32_t(plan.split_k)};
    if (plan.variant == V_SKINNY) {
        auto pick = [&](auto dt_c) -> void (*)(GemmArgs) {
            constexpr int DT = decltype(dt_c)::value;
            if (plan.bm == 32) return plan.bk == 256 ? gemm_bf16_skinny<1, 256, DT> : plan.bk == 128 ? gemm_bf16_skinny<1, 128, DT> : gemm_bf16_skinny<1, 64, DT>;
            return gemm_bf16_skinny<2, 128, DT>;  // row blocks of 64: only with the 128-wide K step (the planner never asks for another)
        };
        void (*kern)(GemmArgs) = p->dtype == FLE_F16 ? pick(std::integral_constant<int, FLE_F16>{}) : pick(std::integral_constant<int, FLE_BF16>{});
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, g);
    } else if (plan.variant == V_TILED) {
        // split K writes fp32 slabs with a padded leading dimension: vector stores whatever out looks like
        const bool edge = plan.edge && !split;
        void (*kern)(GemmArgs);
        auto pick = [&](auto dt_c) -> void (*)(GemmArgs) {
            constexpr int DT = decltype(dt_c)::value;
            if (plan.bm == 256) return edge ? gemm_tiled_256<DT, true> : gemm_tiled_256<DT, false>;
            return edge ? gemm_tiled_128<DT, true> : gemm_tiled_128<DT, false>;
        };
        if (p->dtype == FLE_F32) kern = pick(std::integral_constant<int, FLE_F32>{});
        else if (p->dtype == FLE_F16) kern = pick(std::integral_constant<int, FLE_F16>{});
        else kern = pick(std::integral_constant<int, FLE_BF16>{});
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, g);
    } else {
        // vector loads need 4-element groups that never straddle K and rows that keep the alignment
        const size_t va = bf16 ? 8 : 16;
        const bool vec = p->K % 4 == 0 && reinterpret_cast<uintptr_t>(p->x) % va == 0 && reinterpret_cast<uintptr_t>(p->w) % va == 0 &&
                         p->ldx % 4 == 0 && p->ldw % 4 == 0;
        auto pick = [&](auto dt_c) -> void (*)(GemmArgs) {
            constexpr int DT = decltype(dt_c)::value;
            if (plan.bm == 32) return vec ? gemm_general<DT, true, 2> : gemm_general<DT, false, 2>;
            return vec ? gemm_general<DT, true, 1> : gemm_general<DT, false, 1>;
        };
        void (*kern)(GemmArgs) = p->dtype == FLE_F32 ? pick(std::integral_constant<int, FLE_F32>{})
                                 : p->dtype == FLE_F16 ? pick(std::integral_constant<int, FLE_F16>{}) : pick(std::integral_constant<int, FLE_BF16>{});
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, g);
    }
    fle_status s = check_launch("GEMM kernel launch");
    if (s == FLE_OK && split) {
        const int64_t want = (p->M * ((p->N + 255) / 256) + 3) / 4;
        hipLaunchKernelGGL(reduce_slabs, dim3(uint32_t(want < (int64_t(1) << 20) ? want : (int64_t(1) << 20))), dim3(256), 0, stream, r);
        s = check_launch("split-K reduction launch");
    }
    if (s != FLE_OK || e.row_kind < 0) return s;

    FinArgs f{};
    f.M = p->M; f.N = p->N;
    f.np = plan.np; f.part_cols = plan.part_cols;
    f.partials = split ? r.partials : g.partials;
    f.out = p->out; f.ldo = p->ldo;
    f.epi = e;
    if (e.row_kind == FLE_LOGSUMEXP) {
        hipLaunchKernelGGL(finalize_lse, dim3(uint32_t((p->M + 3) / 4)), dim3(256), 0, stream, f);
        return check_launch("logsumexp finalize launch");
    }
    if (split) { f.y = r.dst; f.ldy = r.ldd; f.y_f32 = r.dst_f32; }
    else { f.y = g.dst; f.ldy = g.ldd; f.y_f32 = g.dst_f32; }
    f.y_rel = plan.stage_rel;
    const size_t ysz = f.y_f32 ? 4 : es;
    const bool vec = p->N % 8 == 0 && f.ldy % 8 == 0 && p->ldo % 8 == 0 && reinterpret_cast<uintptr_t>(f.y) % (8 * ysz) == 0 &&
                     reinterpret_cast<uintptr_t>(p->out) % (8 * es) == 0;
    // vector path also needs 16-byte aligned gamma / beta
    const bool gb_ok = reinterpret_cast<uintptr_t>(e.row.p0) % (8 * es) == 0 && reinterpret_cast<uintptr_t>(e.row.p1) % (8 * es) == 0;
    const int64_t items = p->M * ((p->N + 2047) / 2048);
    const int64_t want = (items + 3) / 4;
    const dim3 fgrid(uint32_t(want < (int64_t(1) << 20) ? want : (int64_t(1) << 20)));
    void (*fin)(FinArgs);
    if (e.row_kind == FLE_LAYERNORM) fin = (vec && gb_ok) ? finalize_rows<true, true> : finalize_rows<false, true>;
    else fin = (vec && gb_ok) ? finalize_rows<true, false> : finalize_rows<false, false>;
    hipLaunchKernelGGL(fin, fgrid, dim3(256), 0, stream, f);
    return check_launch("row finalize launch");
}

}  // namespace fle
