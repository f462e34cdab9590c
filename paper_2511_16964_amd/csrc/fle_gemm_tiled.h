// The tiled MFMA GEMM (bf16, fp16, fp32, fp8 and block-scaled fp8 operands) with the fused epilogue.
#pragma once
#include "fle_device_common.h"

namespace fle {

// ------------------------------------------------------------------ tiled MFMA GEMM
// Block tile BM x BN (rows of x, rows of W), K step 128 bytes of every row (64 bf16 / fp16, 32 fp32, 128 fp8),
// 4 waves as 2 x 2, each wave owning (BM/2) x (BN/2) outputs: as 16x16 accumulator tiles of
// v_mfma_f32_16x16x32_bf16 / _f16 for the 2-byte dtypes, as 32x32 tiles of v_mfma_f32_32x32x2_f32 (four per
// fragment pair) for fp32 and of v_mfma_f32_32x32x64_f8f6f4 (plain or block-scaled) for fp8.
//
// Main loop.  Operand tiles go HBM -> LDS by buffer loads that write LDS directly (no
// registers), two stages deep.  A stage row is 128 bytes = 8 chunks of 16 bytes, stored at chunk
// position c ^ g(row), g(row) = (row & 7) ^ ((row >> 3) & 1): the 16-byte reads of an MFMA
// fragment (consecutive rows, one logical chunk) then hit every LDS bank once.  Within a
// K step the copy instructions for a later stage and the fragment reads for the next
// k slice are issued one at a time in the gaps between MFMAs (pinned with
// sched_barrier): a wave issues in order, so a burst of memory instructions would otherwise
// leave the matrix pipe idle while the LDS and texture paths accept them.  Each of the three
// loops below says where its copies and reads go and why.
//
// Epilogue.  One 32-row block of the wave's accumulators at a time is staged through LDS as
// fp32 and read back row-contiguous: a lane then owns 4 (or 2 x 4) consecutive columns of one
// row, 16 lanes cover a whole 64-column run, so bias / residual / output accesses are full
// cache lines and a row reduction is a 16-lane DPP reduction.  (Stores straight from the
// accumulators' layout, 16 rows x 32 bytes per instruction, skip the 3.3 us that the LDS trip
// costs a 256 x 256 tile and were still slower: 97.7 against 96.3 us on 4096^3.)  The residual
// tile is copied into LDS by the same direct loads, block by block, the first one behind the
// first barrier of the main loop.
// AUX: cache policy bits of the copy instructions (2 = non-temporal, for a panel that is read once).
template <int ROWS, int AUX = 0>
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
    // Copy instruction j (8 rows x 128 bytes) of this wave's quarter of the tile at byte column k0.  k0 travels
    // as the instruction's scalar offset, so the per-lane offset does not change from one K step to the next
    // and the main loop spends no vector ALU work on addresses.
    __device__ __forceinline__ void issue_one(char *lds, uint32_t k0, int j) const {
        const uint32_t voff = ((j & 1) ? off_odd : off_even) + uint32_t(j) * row_step;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(lds + (wave * (ROWS / 4) + j * 8) * 128), 16, voff, k0, 0, AUX);
    }
    // Same for the last, partial K step: chunks at or beyond `valid` (= remaining row bytes / 16) get
    // an out-of-range offset, for which the buffer load delivers zeros.
    __device__ __forceinline__ void issue_one_tail(char *lds, uint32_t k0, int j, int valid) const {
        uint32_t voff = ((j & 1) ? off_odd : off_even) + uint32_t(j) * row_step;
        if ((chunk_even ^ (j & 1)) >= valid) voff = 0x80000000u;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(lds + (wave * (ROWS / 4) + j * 8) * 128), 16, voff, k0, 0, AUX);
    }
    __device__ __forceinline__ void issue(char *lds, uint32_t k0, int valid) const {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            if (valid >= 8) issue_one(lds, k0, j);
            else issue_one_tail(lds, k0, j, valid);
        }
    }
};

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

// 4 packed 2-byte values as fp32.
template <int DT>
__device__ __forceinline__ f32x4 unpack4(u32x2 u) {
    static_assert(DT == FLE_BF16 || DT == FLE_F16, "2-byte dtypes only");
    if constexpr (DT == FLE_F16) {
        return __builtin_convertvector(__builtin_bit_cast(f16x4, u), f32x4);
    } else {
        f32x4 r;
        r[0] = __uint_as_float(u[0] << 16);
        r[1] = __uint_as_float(u[0] & 0xffff0000u);
        r[2] = __uint_as_float(u[1] << 16);
        r[3] = __uint_as_float(u[1] & 0xffff0000u);
        return r;
    }
}

// acc += A B on v_mfma_f32_16x16x32_bf16 / _f16 with the accumulator tied to one place in the accumulation
// registers.  (Through the compiler's builtin the 64 four-register accumulators of a 128 x 128 wave tile are
// shuffled between register files on every trip of the K loop: the instruction's result need not overwrite its
// addend, and the allocator uses that freedom.)  a, b: 16 bytes of one row each, 8 consecutive k.
template <int DT>
__device__ __forceinline__ void mfma_16x16x32(f32x4 &acc, const u32x4 &a, const u32x4 &b) {
    if constexpr (DT == FLE_F16) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// The output tile a workgroup computes: its origin, the first row past the rows it may touch (the
// end of the matrix, or of the row group that owns the tile), and the W and bias of that owner.
struct TileRef {
    int64_t m0, n0, m_end;
    const void *w, *bias;
};

// Workgroup id -> tile of a tiles_m x tiles_n grid.  Consecutive workgroup ids go round-robin over
// the 8 XCDs, so give each XCD a contiguous range of tile ids, then walk tiles in groups of 4 tile
// rows: the tiles an XCD works on at any time share x and W panels in its own L2.
__device__ __forceinline__ void tile_of_workgroup(uint32_t bid, uint32_t tiles_m, uint32_t tiles_n, int &tile_m, int &tile_n) {
    const uint32_t G = tiles_m * tiles_n;
    const uint32_t per = G / 8, rem = G % 8, xcd = bid % 8, loc = bid / 8;
    const uint32_t id = loc + xcd * per + (xcd < rem ? xcd : rem);
    const uint32_t width = 4 * tiles_n;
    const uint32_t first_m = (id / width) * 4;
    const uint32_t gsz = (tiles_m - first_m) < 4 ? (tiles_m - first_m) : 4;
    tile_m = int(first_m + (id % width) % gsz);
    tile_n = int((id % width) / gsz);
}

template <int BM>
__device__ __forceinline__ TileRef whole_matrix_tile(const GemmArgs &a) {
    int tile_m, tile_n;
    tile_of_workgroup(blockIdx.x, uint32_t(a.tiles_m), uint32_t(a.tiles_n), tile_m, tile_n);
    return TileRef{int64_t(tile_m) * BM, int64_t(tile_n) * BM, a.M, a.w, a.epi.bias};
}

// Grouped problems: the rows of x / out / residual are cut into consecutive groups by a device array
// of offsets, and group g multiplies by its own W (and adds its own bias).
struct GroupArgs {
    const int64_t *row_offsets;  // [n_groups + 1], device memory
    int32_t n_groups;
    int64_t w_stride_bytes;      // from one group's W (bias) to the next group's
    int64_t b_stride_bytes;
};

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = uint32_t(__shfl_up(int(v), d, 64));
        if (lane >= d) v += o;
    }
    return v;
}

__device__ __forceinline__ int64_t wave_pick_i64(int64_t v, int src) {
    const uint32_t lo = uint32_t(__builtin_amdgcn_readfirstlane(__shfl(int(uint32_t(v)), src, 64)));
    const uint32_t hi = uint32_t(__builtin_amdgcn_readfirstlane(__shfl(int(uint32_t(uint64_t(v) >> 32)), src, 64)));
    return int64_t((uint64_t(hi) << 32) | lo);
}

// Workgroup id -> tile of a grouped problem.  Group g owns ceil(rows_g / BM) tile rows, which start at
// the group's first row, so no tile straddles two groups.  The offsets live in device memory (a router
// kernel usually writes them), so every workgroup derives the mapping itself: each lane takes one
// group, a wave prefix sum over the groups' tile rows gives the total (for the XCD-aware id -> tile
// mapping) and then the group holding this workgroup's tile row.  Offsets are clamped to [0, M] and
// to be non-decreasing, so whatever the array holds, every access stays inside the operands.
// Returns false for the surplus workgroups of the launch (the grid is sized for the worst case).
template <int BM>
__device__ __forceinline__ bool grouped_tile(const GemmArgs &a, const GroupArgs &ga, TileRef &t) {
    const int lane = threadIdx.x & 63;
    const int64_t M = a.M;
    const int G = ga.n_groups;
    auto group_rows = [&](int g, int64_t &b, int64_t &e) -> uint32_t {  // tile rows of group g (0 beyond the last group)
        b = e = 0;
        if (g >= G) return 0u;
        b = ga.row_offsets[g];
        e = ga.row_offsets[g + 1];
        b = b < 0 ? 0 : (b > M ? M : b);
        e = e < b ? b : (e > M ? M : e);
        return uint32_t((e - b + BM - 1) / BM);
    };
    uint32_t total = 0;
    for (int c = 0; c < G; c += 64) {
        int64_t b, e;
        const uint32_t incl = wave_inclusive_scan(group_rows(c + lane, b, e), lane);
        total += uint32_t(__builtin_amdgcn_readfirstlane(__shfl(int(incl), 63, 64)));
    }
    const uint32_t tiles_n = uint32_t(a.tiles_n);
    if (blockIdx.x >= total * tiles_n) return false;
    int tile_m, tile_n;
    tile_of_workgroup(blockIdx.x, total, tiles_n, tile_m, tile_n);
    uint32_t base = 0;
    for (int c = 0; c < G; c += 64) {
        int64_t b, e;
        const uint32_t mine = group_rows(c + lane, b, e);
        const uint32_t incl = wave_inclusive_scan(mine, lane);
        const uint64_t hit = __ballot(base + incl > uint32_t(tile_m));
        if (hit) {
            const int src = __builtin_ctzll(hit);
            const uint32_t first = base + uint32_t(__builtin_amdgcn_readfirstlane(__shfl(int(incl - mine), src, 64)));  // first tile row of the group
            const int64_t gb = wave_pick_i64(b, src), ge = wave_pick_i64(e, src);
            const int64_t g = c + src;
            t.m0 = gb + int64_t(uint32_t(tile_m) - first) * BM;
            t.m_end = ge;
            if (t.m0 >= ge) return false;  // only if a malformed array made the 32-bit tile counts wrap
            t.n0 = int64_t(tile_n) * BM;
            t.w = reinterpret_cast<const char *>(a.w) + g * ga.w_stride_bytes;
            t.bias = a.epi.bias ? reinterpret_cast<const char *>(a.epi.bias) + g * ga.b_stride_bytes : nullptr;
            return true;
        }
        base += uint32_t(__builtin_amdgcn_readfirstlane(__shfl(int(incl), 63, 64)));
    }
    return false;  // not reached: tile_m < total
}

// EDGE: N, the leading dimensions or the addresses of b / residual / out do not allow 4-column vector
// accesses; the epilogue then touches memory one element at a time, masked per column.
// W_NT: the W panel is read by this workgroup only (grouped problems with about one tile row per group), so
// its copies carry the non-temporal hint and do not displace other data from L2 and the Infinity Cache.
// MF: shape of the MFMA tiles of the main loop, 32 (v_mfma_f32_32x32x16, k slices of 16, four per K step) or, for
// the 2-byte dtypes, 16 (v_mfma_f32_16x16x32, k slices of 32, two per K step: twice as many issue slots between
// matrix instructions for the same fragment reads and copies, and half the accumulator traffic per flop).
// C1: (MF = 16) how many of a K step's copy instructions go out in the slice right behind the barrier; the
// rest follow in the next slice.
// MX: (fp8 operands) every 32 consecutive k of a row of x and of W share a power-of-two scale, one E8M0 byte each:
// the OCP microscaling format, multiplied on the matrix instruction's scaled form.
template <int BM, int BN, int DT, bool EDGE, bool W_NT = false, int MF = 32, int C1 = -1, bool MX = false>
__device__ __forceinline__ void gemm_tiled_body(const GemmArgs &a, const TileRef &t) {
    constexpr bool F32 = DT == FLE_F32, F8 = DT == FLE_F8E4M3;
    static_assert(!MX || F8, "block scales exist for fp8 operands");
    static_assert(MF == 32 || (MF == 16 && !F32 && !F8), "16x16 tiles exist for the 2-byte dtypes");
    constexpr int DTE = F8 ? FLE_BF16 : DT;     // dtype of b, the residual and store operands and out (fp8 problems: bf16)
    constexpr int ES = F32 ? 4 : F8 ? 1 : 2;    // bytes per operand element; a staged row is 128 bytes = 128 fp8, 64 bf16 or 32 fp32
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
    const int64_t M = t.m_end, N = a.N;  // M: first row past the rows this tile may touch

    const int64_t m0 = t.m0, n0 = t.n0;
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

    TileLoader<BM> ldx_;
    TileLoader<BN, W_NT ? 2 : 0> ldw_;
    ldx_.init(reinterpret_cast<const char *>(a.x) + m0 * a.ldx * ES, a.ldx * ES, M - m0, a.K * ES, wave, lane);
    ldw_.init(reinterpret_cast<const char *>(t.w) + n0 * a.ldw * ES, a.ldw * ES, N - n0, a.K * ES, wave, lane);
    constexpr int NIW = TileLoader<BN>::NI, NIX = TileLoader<BM>::NI;

    // 16 bytes of one row: 4 fp32, 8 bf16 or 8 fp16 along K
    using frag_t = typename std::conditional<F32, f32x4, typename std::conditional<DT == FLE_F16, f16x8, bf16x8>::type>::type;
    const int KT = int((a.K * ES + 127) / 128);
    const int tail_valid = int((a.K * ES - int64_t(KT - 1) * 128) / 16);  // 16-byte chunks of the last K step (8 = full)
    // K steps kb .. ke-1 of this workgroup (all of them unless K is split over gridDim.y).
    const int kb = int(int64_t(blockIdx.y) * KT / gridDim.y), ke = int(int64_t(blockIdx.y + 1) * KT / gridDim.y);
    auto valid_of = [&](int step) { return step + 1 == KT ? tail_valid : 8; };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    constexpr int TM16 = WM / 16, TN16 = WN / 16;
    f32x16 acc[MF == 32 ? TM : 1][MF == 32 ? TN : 1];
    f32x4 acc16[MF == 16 ? TM16 : 1][MF == 16 ? TN16 : 1];
    if constexpr (F8) {
        // ---- main loop on 32x32x64 tiles (fp8 operands).  A K step (128 bytes of every row) is two k slices of 64;
        // a fragment (32 rows x 64 k) is 32 bytes per lane, read as two 16-byte pieces: row (lane & 31), chunks
        // 4 s + hh and 4 s + 2 + hh of slice s, hh = lane >> 5, which is where the instruction expects them (16 k
        // values of the slice's first half, then 16 of its second); lanes l and l + 32, which the LDS serves in
        // the same cycle, then read chunks one apart: no bank conflicts under the row swizzle.  16 matrix instructions of 64 cycles per slice move the
        // same bytes through LDS as the 2-byte loop's 64 of 16 cycles, for twice the products.  The schedule is
        // that loop's: fragments one slice ahead, wait and barrier between the two slices of a step, the copies
        // of the step after next right behind the barrier.
        // (The 16x16x128 shape needs its fragments a whole K step ahead, 192 registers of them next to 256
        // accumulators: it spilled.)
        uint32_t rd_off[2][2];  // [slice][piece]
        {
            const int r = lane & 31, g = (r & 7) ^ ((r >> 3) & 1), hh = lane >> 5;
#pragma unroll
            for (int sl = 0; sl < 2; ++sl)
#pragma unroll
                for (int e = 0; e < 2; ++e) rd_off[sl][e] = uint32_t(r * 128 + (((4 * sl + 2 * e + hh) ^ g) << 4));
        }
        // Block scales.  With the pieces as above, the first 16 bytes of a lane lie in the slice's first block of 32
        // k values and the second 16 bytes in its second block, for both lane halves, and the instruction takes the
        // scale of a row's first block from that row's lane in the lower half and the scale of its second block
        // from its lane in the upper half (established with single non-unit scales and single non-zero k
        // positions).  The scale bytes of a K step (4 blocks) are one dword per row, read from memory a K step
        // ahead; lanes of the upper half shift theirs down a byte, and the instruction picks byte 2 s: block
        // 2 s + hh.  Rows beyond the tile's valid rows read zero: 2^-127 times operand bytes that are zero as well.
        [[maybe_unused]] uint32_t sw_cur[TN], sx_cur[TM], sw_nxt[TN], sx_nxt[TM], sw_nx2[TN], sx_nx2[TM];
        [[maybe_unused]] __amdgpu_buffer_rsrc_t sw_rsrc = __builtin_amdgcn_make_buffer_rsrc(nullptr, 0, 0, 0x00020000), sx_rsrc = sw_rsrc;
        [[maybe_unused]] uint32_t sc_row = 0, sc_shift = 0;
        if constexpr (MX) {
            const int64_t ks = a.K / 32;  // bytes per row of scales
            const int64_t rows_w = (N - n0) < BN ? (N - n0) : BN, rows_x = (M - m0) < BM ? (M - m0) : BM;
            sw_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(reinterpret_cast<const char *>(a.w_scale) + n0 * ks), 0, uint32_t((rows_w > 0 ? rows_w : 0) * ks), 0x00020000);
            sx_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(reinterpret_cast<const char *>(a.x_scale) + m0 * ks), 0, uint32_t((rows_x > 0 ? rows_x : 0) * ks), 0x00020000);
            sc_row = uint32_t(lane & 31) * uint32_t(ks);
            sc_shift = uint32_t(lane >> 5) * 8;
        }
        // The scales of step kt + 2 are requested in the middle of step kt, behind the copies of its first slice, and
        // the wait in front of the barrier leaves exactly these TN + TM loads in flight (loads complete in order):
        // they have a step and a half to arrive, and no wait ever includes a request that has only just gone out.
        auto load_scales = [&](int kt, uint32_t (&dw)[TN], uint32_t (&dx)[TM]) {
            if constexpr (MX) {
                const uint32_t ks = uint32_t(a.K / 32);
#pragma unroll
                for (int j = 0; j < TN; ++j) dw[j] = __builtin_amdgcn_raw_buffer_load_b32(sw_rsrc, int(sc_row + uint32_t(wn * WN + j * 32) * ks), kt * 4, 0);
#pragma unroll
                for (int i = 0; i < TM; ++i) dx[i] = __builtin_amdgcn_raw_buffer_load_b32(sx_rsrc, int(sc_row + uint32_t(wm * WM + i * 32) * ks), kt * 4, 0);
            }
        };
        auto take_scales = [&]() {  // this step's scales, and the next step's move up
            if constexpr (MX) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    sw_cur[j] = sw_nxt[j] >> sc_shift;
                    sw_nxt[j] = sw_nx2[j];
                }
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    sx_cur[i] = sx_nxt[i] >> sc_shift;
                    sx_nxt[i] = sx_nx2[i];
                }
            }
        };
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
        typedef __attribute__((ext_vector_type(8))) int i32x8;
        struct Frag { u32x4 lo, hi; };
        Frag fw[2][TN], fx[2][TM];
        constexpr int NMF = TM * TN, NRD = 2 * (TM + TN);  // MFMAs per slice, 16-byte reads per slice
        constexpr int NCP = NIW + NIX;
        constexpr int NC1 = C1 < 0 ? (NCP * 3) / 4 : C1;
        auto slice = [&](auto sl_c, auto read_c, auto first_c, auto count_c, auto full_c, const char *rW, const char *rX, int rs,
                         char *iW, char *iX, uint32_t ik0, int valid) {
            constexpr int SL = decltype(sl_c)::value, FIRST = decltype(first_c)::value, COUNT = decltype(count_c)::value;
            constexpr bool READ = decltype(read_c)::value, FULL = decltype(full_c)::value;
#pragma unroll
            for (int q = 0; q < NMF; ++q) {
#pragma unroll
                for (int r = 0; r < NRD; ++r) {  // read r (piece e of fragment g of the next slice) goes out before MFMA r NMF / NRD
                    if (!READ || (r * NMF) / NRD != q) continue;
                    const int g = r / 2, e = r % 2;
                    const u32x4 v = g < TN ? *reinterpret_cast<const u32x4 *>(rW + (wn * WN + (g % TN) * 32) * 128 + rd_off[rs][e])
                                           : *reinterpret_cast<const u32x4 *>(rX + (wm * WM + ((g - TN) % TM) * 32) * 128 + rd_off[rs][e]);
                    Frag &f = g < TN ? fw[SL ^ 1][g % TN] : fx[SL ^ 1][(g - TN) % TM];
                    if (e == 0) f.lo = v; else f.hi = v;
                }
#pragma unroll
                for (int c = 0; c < COUNT; ++c) {  // copy c goes out before MFMA c (as many per slot as it takes when there are fewer slots):
                    if ((c < NMF ? c : c % NMF) != q) continue;  // a matrix instruction lasts as long as the texture path needs for one copy of each wave
                    const int idx = FIRST + c;
                    if constexpr (FULL) {
                        if (idx < NIW) ldw_.issue_one(iW, ik0, idx);
                        else ldx_.issue_one(iX, ik0, idx - NIW);
                    } else {
                        if (idx < NIW) ldw_.issue_one_tail(iW, ik0, idx, valid);
                        else ldx_.issue_one_tail(iX, ik0, idx - NIW, valid);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                const Frag &fa = fw[SL][q % TN], &fb = fx[SL][q / TN];
                if constexpr (MX)
                    acc[q / TN][q % TN] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        __builtin_bit_cast(i32x8, __builtin_shufflevector(fa.lo, fa.hi, 0, 1, 2, 3, 4, 5, 6, 7)),
                        __builtin_bit_cast(i32x8, __builtin_shufflevector(fb.lo, fb.hi, 0, 1, 2, 3, 4, 5, 6, 7)), acc[q / TN][q % TN], 0, 0,
                        2 * SL, int(sw_cur[q % TN]), 2 * SL, int(sx_cur[q / TN]));
                else
                    acc[q / TN][q % TN] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        __builtin_bit_cast(i32x8, __builtin_shufflevector(fa.lo, fa.hi, 0, 1, 2, 3, 4, 5, 6, 7)),
                        __builtin_bit_cast(i32x8, __builtin_shufflevector(fb.lo, fb.hi, 0, 1, 2, 3, 4, 5, 6, 7)), acc[q / TN][q % TN], 0, 0, 0, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        using CNT1 = std::integral_constant<int, NC1>;
        if constexpr (MX) {
#pragma unroll
            for (int j = 0; j < TN; ++j) sw_nx2[j] = 0;
#pragma unroll
            for (int i = 0; i < TM; ++i) sx_nx2[i] = 0;
        }
        load_scales(kb, sw_nxt, sx_nxt);
        if (kb + 1 < ke) load_scales(kb + 1, sw_nx2, sx_nx2);
        ldw_.issue(smem + (kb & 1) * STAGE, uint32_t(kb) * 128, valid_of(kb));
        ldx_.issue(smem + (kb & 1) * STAGE + SW, uint32_t(kb) * 128, valid_of(kb));
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (res_idx >= 0 && wave_live) issue_residual(0, 0);  // (behind the first stage: the wait above does not include it)
        {
            const char *sW = smem + (kb & 1) * STAGE, *sX = sW + SW;
#pragma unroll
            for (int g = 0; g < TN; ++g) {
                fw[0][g].lo = *reinterpret_cast<const u32x4 *>(sW + (wn * WN + g * 32) * 128 + rd_off[0][0]);
                fw[0][g].hi = *reinterpret_cast<const u32x4 *>(sW + (wn * WN + g * 32) * 128 + rd_off[0][1]);
            }
#pragma unroll
            for (int g = 0; g < TM; ++g) {
                fx[0][g].lo = *reinterpret_cast<const u32x4 *>(sX + (wm * WM + g * 32) * 128 + rd_off[0][0]);
                fx[0][g].hi = *reinterpret_cast<const u32x4 *>(sX + (wm * WM + g * 32) * 128 + rd_off[0][1]);
            }
            if (kb + 1 < ke) {
                char *iW = smem + ((kb + 1) & 1) * STAGE, *iX = iW + SW;
#pragma unroll
                for (int idx = 0; idx < NC1; ++idx) {
                    if (idx < NIW) ldw_.issue_one_tail(iW, uint32_t(kb + 1) * 128, idx, valid_of(kb + 1));
                    else ldx_.issue_one_tail(iX, uint32_t(kb + 1) * 128, idx - NIW, valid_of(kb + 1));
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        auto k_step = [&](int kt, auto more_c, auto more2_c, auto full_c) {
            constexpr bool MORE = decltype(more_c)::value, MORE2 = decltype(more2_c)::value;
            char *cW = smem + (kt & 1) * STAGE, *cX = cW + SW;
            char *nW = smem + ((kt + 1) & 1) * STAGE, *nX = nW + SW;
            take_scales();
            slice(I0{}, std::true_type{}, CNT1{}, std::integral_constant<int, MORE ? NCP - NC1 : 0>{}, full_c, cW, cX, 1, nW, nX, uint32_t(kt + 1) * 128, valid_of(kt + 1));
            if constexpr (MX && MORE2) load_scales(kt + 2, sw_nx2, sx_nx2);
            if constexpr (MORE) {
                wait_vmcnt<(MX && MORE2) ? TN + TM : 0>();
                __builtin_amdgcn_s_waitcnt(0xC07F);
                __builtin_amdgcn_s_barrier();
            }
            slice(I1{}, std::integral_constant<bool, MORE>{}, I0{}, std::integral_constant<int, MORE2 ? NC1 : 0>{}, full_c, nW, nX, 0, cW, cX, uint32_t(kt + 2) * 128, valid_of(kt + 2));
        };
        int kt = kb;
        for (; kt + 3 < ke; ++kt) k_step(kt, std::true_type{}, std::true_type{}, std::true_type{});
        if (kt + 2 < ke) {
            k_step(kt, std::true_type{}, std::true_type{}, std::false_type{});
            ++kt;
        }
        if (kt + 1 < ke) {
            k_step(kt, std::true_type{}, std::false_type{}, std::false_type{});
            ++kt;
        }
        k_step(kt, std::false_type{}, std::false_type{}, std::false_type{});
    } else if constexpr (MF == 16) {
        // ---- main loop on 16x16x32 tiles.  A K step is two k slices of 32; a fragment (16 rows x 32 k) is one
        // 16-byte read per lane: row (lane & 15) and one of the four chunks of slice s.  The instruction takes the k
        // values of lanes 16 h .. 16 h + 15 as one group of 8, and a sum over k does not care which group holds
        // which chunk as long as both operands agree, so group h reads chunk kq(h) = 0, 2, 1, 3: the LDS serves a
        // 16-byte read of lanes l and l + 32 in the same cycle, and with chunks two apart in those two lane
        // groups the row swizzle sent them to the same banks (measured: 8.7e6 conflict cycles per 4096^3 call, the
        // LDS twice as long busy; chunks one apart: none).
        uint32_t rd_off[2];
        {
            const int r = lane & 15, g = (r & 7) ^ ((r >> 3) & 1);
            const int h = lane >> 4, kq = ((h & 1) << 1) | (h >> 1);
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) rd_off[sl] = uint32_t(r * 128 + (((4 * sl + kq) ^ g) << 4));
        }
#pragma unroll
        for (int i = 0; i < TM16; ++i)
#pragma unroll
            for (int j = 0; j < TN16; ++j) {
                acc16[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                // The zeros are written here, in front of the wait states below.  Left free, the compiler may sink
                // each write to just before the first matrix instruction that reads it (seen when the first K steps
                // were peeled out of the loop); that instruction is inline asm, so the hazard recognizer puts no wait
                // states between the two and the instruction reads a stale accumulator.
                asm volatile("" : "+a"(acc16[i][j]));
            }
        asm volatile("s_nop 7");
        u32x4 fw[2][TN16], fx[2][TM16];
        constexpr int NMF = TM16 * TN16, NDS = TM16 + TN16, QD = NMF / NDS;  // MFMAs per slice, fragment reads per slice, MFMAs per read
        constexpr int NCP = NIW + NIX;                                        // copy instructions per K step
        constexpr int NC1 = C1 < 0 ? (NCP * 3) / 4 : C1;                      // ... of which in the slice behind the barrier
        constexpr int CSTEP = NMF / (NC1 > 0 ? NC1 : 1) >= 3 ? 3 : NMF / (NC1 > 0 ? NC1 : 1) >= 2 ? 2 : 1;  // MFMAs from one copy to the next
        static_assert(NC1 >= 0 && NC1 <= NCP && CSTEP * (NC1 - 1) + 1 < NMF && CSTEP * (NCP - NC1 - 1) + 1 < NMF, "copy placement");
        // Slice SL of the stage being multiplied: NMF MFMAs on the fragments in buffer SL.  In the issue slots
        // between them go, one at a time, (READ) the fragment reads of the slice that is multiplied next (slice rs
        // of the stage at (rW, rX)) into the other buffer, and copy instructions FIRST .. FIRST + COUNT - 1 of one
        // K step into the stage at (iW, iX), one every CSTEP MFMAs from the start of the slice: a stage has one K
        // step from the barrier that frees it to the barrier that needs it, the texture path takes half of that
        // to accept the step's copies, and what is left is the time the last copy has to land.  Measured against
        // an even spread over the slice (4096^3): 172 k -> 152 k cycles in the loop; the clock, which the chip lowers
        // as the loop gets denser, gives back more than half of that (1.91 -> 1.76 GHz; 104.9 -> 100.3 us).
        auto slice = [&](auto sl_c, auto read_c, auto first_c, auto count_c, auto full_c, const char *rW, const char *rX, int rs,
                         char *iW, char *iX, uint32_t ik0, int valid) {
            constexpr int SL = decltype(sl_c)::value, FIRST = decltype(first_c)::value, COUNT = decltype(count_c)::value;
            constexpr bool READ = decltype(read_c)::value, FULL = decltype(full_c)::value;
#pragma unroll
            for (int q = 0; q < NMF; ++q) {
                if (READ && q % QD == 0) {
                    const int g = q / QD;
                    if (g < TN16) fw[SL ^ 1][g] = *reinterpret_cast<const u32x4 *>(rW + (wn * WN + g * 16) * 128 + rd_off[rs]);
                    else fx[SL ^ 1][g - TN16] = *reinterpret_cast<const u32x4 *>(rX + (wm * WM + (g - TN16) * 16) * 128 + rd_off[rs]);
                }
                if (COUNT > 0 && q % CSTEP == 1 % CSTEP && q / CSTEP < COUNT) {  // copy c of this slice goes out before MFMA CSTEP c + 1
                    const int idx = FIRST + q / CSTEP;
                    if constexpr (FULL) {
                        if (idx < NIW) ldw_.issue_one(iW, ik0, idx);
                        else ldx_.issue_one(iX, ik0, idx - NIW);
                    } else {
                        if (idx < NIW) ldw_.issue_one_tail(iW, ik0, idx, valid);
                        else ldx_.issue_one_tail(iX, ik0, idx - NIW, valid);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                mfma_16x16x32<DT>(acc16[q / TN16][q % TN16], fw[SL][q % TN16], fx[SL][q / TN16]);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        using CNT1 = std::integral_constant<int, NC1>;
        // The loop is rotated by one slice against the K steps: the wait for the next stage and the workgroup
        // barrier sit between the two slices of a step.  By then every fragment of the current stage is in
        // registers (its second slice was read during the first), so the stage may be overwritten; the second
        // slice runs on registers alone and covers the first fragment reads of the next stage and the first NC1
        // copies of the step after it, the other copies go out at the start of the next step's first slice.
        ldw_.issue(smem + (kb & 1) * STAGE, uint32_t(kb) * 128, valid_of(kb));
        ldx_.issue(smem + (kb & 1) * STAGE + SW, uint32_t(kb) * 128, valid_of(kb));
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (res_idx >= 0 && wave_live) issue_residual(0, 0);  // (behind the first stage: the wait above does not include it)
        {
            const char *sW = smem + (kb & 1) * STAGE, *sX = sW + SW;
#pragma unroll
            for (int g = 0; g < TN16; ++g) fw[0][g] = *reinterpret_cast<const u32x4 *>(sW + (wn * WN + g * 16) * 128 + rd_off[0]);
#pragma unroll
            for (int g = 0; g < TM16; ++g) fx[0][g] = *reinterpret_cast<const u32x4 *>(sX + (wm * WM + g * 16) * 128 + rd_off[0]);
            if (kb + 1 < ke) {  // first copies of the second step (later steps: during the second slice of the step before)
                char *iW = smem + ((kb + 1) & 1) * STAGE, *iX = iW + SW;
#pragma unroll
                for (int idx = 0; idx < NC1; ++idx) {
                    if (idx < NIW) ldw_.issue_one_tail(iW, uint32_t(kb + 1) * 128, idx, valid_of(kb + 1));
                    else ldx_.issue_one_tail(iX, uint32_t(kb + 1) * 128, idx - NIW, valid_of(kb + 1));
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        auto k_step = [&](int kt, auto more_c, auto more2_c, auto full_c) {
            constexpr bool MORE = decltype(more_c)::value, MORE2 = decltype(more2_c)::value;
            char *cW = smem + (kt & 1) * STAGE, *cX = cW + SW;        // the stage being multiplied
            char *nW = smem + ((kt + 1) & 1) * STAGE, *nX = nW + SW;  // the stage of the next step
            slice(I0{}, std::true_type{}, CNT1{}, std::integral_constant<int, MORE ? NCP - NC1 : 0>{}, full_c, cW, cX, 1, nW, nX, uint32_t(kt + 1) * 128, valid_of(kt + 1));
            if constexpr (MORE) {
                wait_vmcnt<0>();                          // this wave's copies of the next stage have landed ...
                __builtin_amdgcn_s_waitcnt(0xC07F);       // ... and its last fragment reads of this stage have returned
                __builtin_amdgcn_s_barrier();             // everyone's have: the next stage is complete, this one is free
            }
            slice(I1{}, std::integral_constant<bool, MORE>{}, I0{}, std::integral_constant<int, MORE2 ? NC1 : 0>{}, full_c, nW, nX, 0, cW, cX, uint32_t(kt + 2) * 128, valid_of(kt + 2));
        };
        int kt = kb;
        for (; kt + 3 < ke; ++kt) k_step(kt, std::true_type{}, std::true_type{}, std::true_type{});
        if (kt + 2 < ke) {
            k_step(kt, std::true_type{}, std::true_type{}, std::false_type{});
            ++kt;
        }
        if (kt + 1 < ke) {
            k_step(kt, std::true_type{}, std::false_type{}, std::false_type{});
            ++kt;
        }
        k_step(kt, std::false_type{}, std::false_type{}, std::false_type{});
        // (the matrix instructions above are opaque to the compiler's hazard recognizer: keep the wait states
        // that an accumulator read behind the last of them needs)
        asm volatile("s_nop 7");
        asm volatile("s_nop 7");
        asm volatile("s_nop 7");
    } else {
        // Fragment read offsets: lane reads row (lane & 31) of a 32-row block, logical chunk 2*kk + (lane >> 5).
        uint32_t rd_off[4];
        {
            const int g = (lane & 7) ^ ((lane >> 3) & 1), hh = lane >> 5;
    #pragma unroll
            for (int kk = 0; kk < 4; ++kk) rd_off[kk] = uint32_t((lane & 31) * 128 + (((2 * kk + hh) ^ g) << 4));
        }

    #pragma unroll
        for (int i = 0; i < TM; ++i)
    #pragma unroll
            for (int j = 0; j < TN; ++j)
    #pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

        frag_t fw[2][TN], fx[2][TM];
        // One 16-wide k slice KK of the stage at (sW, sX): NMF MFMAs on the fragments in buffer KK & 1.  In the
        // issue slots between them go, one at a time, (READ) the fragment reads of the slice that is multiplied
        // next, slice (KK + 1) & 3 of the stage at (rW, rX), into the other buffer, and (HALF = 1 or 2) the first
        // or second half of the copy instructions of one K step into the stage at (iW, iX) (masked to the valid
        // chunks when that is the partial last step).
        auto slice = [&](auto kk_c, auto read_c, auto half_c, auto full_c, const char *sW, const char *sX, const char *rW, const char *rX,
                         char *iW, char *iX, uint32_t ik0, int valid) {
            constexpr int KK = decltype(kk_c)::value, HALF = decltype(half_c)::value;
            constexpr bool FULL = decltype(full_c)::value;  // the copied step is known to be a whole one: no masking of chunks
            constexpr bool READ = decltype(read_c)::value;
            constexpr int NMF = TM * TN, NDS = TM + TN, NVM = (NIW + NIX) / 2;
            constexpr int QD = NMF / NDS, QV = NMF / NVM;  // MFMAs per fragment read / per copy instruction
            constexpr int cur = KK & 1;
            (void)sW; (void)sX;
    #pragma unroll
            for (int q = 0; q < NMF; ++q) {
                if (READ && q % QD == 0) {
                    const int g = q / QD;
                    if (g < TN) fw[cur ^ 1][g] = *reinterpret_cast<const frag_t *>(rW + (wn * WN + g * 32) * 128 + rd_off[(KK + 1) & 3]);
                    else fx[cur ^ 1][g - TN] = *reinterpret_cast<const frag_t *>(rX + (wm * WM + (g - TN) * 32) * 128 + rd_off[(KK + 1) & 3]);
                }
                if (HALF != 0 && q % QV == (QV > 1 ? 1 : 0)) {
                    const int idx = (HALF - 1) * NVM + q / QV;
                    if constexpr (FULL) {
                        if (idx < NIW) ldw_.issue_one(iW, ik0, idx);
                        else ldx_.issue_one(iX, ik0, idx - NIW);
                    } else {
                        if (idx < NIW) ldw_.issue_one_tail(iW, ik0, idx, valid);
                        else ldx_.issue_one_tail(iX, ik0, idx - NIW, valid);
                    }
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
        };

        // K steps kb .. ke-1 of this workgroup (all of them unless K is split over gridDim.y).
        //
        // The loop is rotated by one slice against the K steps.  The wait for the next stage and the workgroup
        // barrier sit between slices 2 and 3 of a step, not at its end: by then every fragment of the current
        // stage is in registers (so the stage may be overwritten) and the copies of the next stage have had two
        // slices to land.  Slice 3 then runs on registers alone and covers the first fragment reads of the next
        // stage and the first half of the copies of the step after it; the other half goes out during slice 0.
        // No MFMA ever waits right behind the barrier for an LDS read.
        ldw_.issue(smem + (kb & 1) * STAGE, uint32_t(kb) * 128, valid_of(kb));
        ldx_.issue(smem + (kb & 1) * STAGE + SW, uint32_t(kb) * 128, valid_of(kb));
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (res_idx >= 0 && wave_live) issue_residual(0, 0);  // (behind the first stage: the wait above does not include it)
        {
            const char *sW = smem + (kb & 1) * STAGE, *sX = sW + SW;
    #pragma unroll
            for (int t = 0; t < TN; ++t) fw[0][t] = *reinterpret_cast<const frag_t *>(sW + (wn * WN + t * 32) * 128 + rd_off[0]);
    #pragma unroll
            for (int t = 0; t < TM; ++t) fx[0][t] = *reinterpret_cast<const frag_t *>(sX + (wm * WM + t * 32) * 128 + rd_off[0]);
            if (kb + 1 < ke) {  // first half of the copies of the second step (later steps: during slice 3 of the step before)
                char *iW = smem + ((kb + 1) & 1) * STAGE, *iX = iW + SW;
                constexpr int NVM = (NIW + NIX) / 2;
    #pragma unroll
                for (int idx = 0; idx < NVM; ++idx) {
                    if (idx < NIW) ldw_.issue_one_tail(iW, uint32_t(kb + 1) * 128, idx, valid_of(kb + 1));
                    else ldx_.issue_one_tail(iX, uint32_t(kb + 1) * 128, idx - NIW, valid_of(kb + 1));
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // One K step: MORE: a next step exists (second half of its copies in slice 0, wait and barrier before
        // slice 3, its first fragments read in slice 3); MORE2: so does the one after it (first half of its copies
        // in slice 3).  The flags are compile-time so that the loop body is one straight-line sequence.
        auto k_step = [&](int kt, auto more_c, auto more2_c, auto full_c) {
            constexpr bool MORE = decltype(more_c)::value, MORE2 = decltype(more2_c)::value;
            char *cW = smem + (kt & 1) * STAGE, *cX = cW + SW;        // the stage being multiplied
            char *nW = smem + ((kt + 1) & 1) * STAGE, *nX = nW + SW;  // the stage of the next step
            slice(I0{}, std::true_type{}, std::integral_constant<int, MORE ? 2 : 0>{}, full_c, cW, cX, cW, cX, nW, nX, uint32_t(kt + 1) * 128, valid_of(kt + 1));
            slice(I1{}, std::true_type{}, I0{}, full_c, cW, cX, cW, cX, nW, nX, 0u, 8);
            slice(I2{}, std::true_type{}, I0{}, full_c, cW, cX, cW, cX, nW, nX, 0u, 8);
            if constexpr (MORE) {
                wait_vmcnt<0>();                          // this wave's copies of the next stage have landed ...
                __builtin_amdgcn_s_waitcnt(0xC07F);       // ... and its last fragment reads of this stage have returned
                __builtin_amdgcn_s_barrier();             // everyone's have: the next stage is complete, this one is free
            }
            slice(I3{}, std::integral_constant<bool, MORE>{}, std::integral_constant<int, MORE2 ? 1 : 0>{}, full_c, cW, cX, nW, nX, cW, cX, uint32_t(kt + 2) * 128, valid_of(kt + 2));
        };
        {
            int kt = kb;
            // steps whose copies (for steps kt + 1 and kt + 2) cannot touch the last, possibly partial K step
            for (; kt + 3 < ke; ++kt) k_step(kt, std::true_type{}, std::true_type{}, std::true_type{});
            if (kt + 2 < ke) {
                k_step(kt, std::true_type{}, std::true_type{}, std::false_type{});
                ++kt;
            }
            if (kt + 1 < ke) {
                k_step(kt, std::true_type{}, std::false_type{}, std::false_type{});
                ++kt;
            }
            k_step(kt, std::false_type{}, std::false_type{}, std::false_type{});
        }
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
                    if (n_col[hc] + e < N) bias_v[hc][e] = ld_elem(t.bias, n_col[hc] + e, DTE);
            } else {
                bias_v[hc] = ld4<DTE>(t.bias, n_ok[hc] ? n_col[hc] : N - 4);
            }
        }
    }
    const int p_idx = int(n_wave / WN);
    const int64_t cols_left = N - n_wave;
    const float cnt = float(cols_left < WN ? cols_left : WN);
    const float inv_cnt = 1.0f / cnt;  // (exact for a full wave tile; the partial's M2 is taken about the mean as computed, so an ulp in it costs nothing)

    // One 32-row block.  FULL: all of this wave's rows and columns lie inside the matrix, and nothing in the block
    // is masked: every store is issued, unconditionally, so their number is known (see the residual below).
    auto block = [&](const int i, auto full_c) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full_c)::value;
        const int64_t m_blk = m_wave + 32 * i;
        // accumulators of row block i -> LDS.  32x32 tiles: row (lane & 31), columns 32 j + 8 q + 4 h .. + 3;
        // 16x16 tiles (two tile rows per block): row 16 t + (lane & 15), columns 16 j + 4 (lane >> 4) .. + 3
        {
            char *wr = MF == 16 ? ep + (lane & 15) * EP_STRIDE + (lane >> 4) * 16 : ep + (lane & 31) * EP_STRIDE + (lane >> 5) * 16;
            auto put = [&](auto ic) __attribute__((always_inline)) {
                constexpr int I = decltype(ic)::value;
                if constexpr (I < TM) {
                    if constexpr (MF == 16) {
#pragma unroll
                        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                            for (int j = 0; j < TN16; ++j) *reinterpret_cast<f32x4 *>(wr + tt * 16 * EP_STRIDE + 16 * j * 4) = acc16[2 * I + tt][j];
                    } else {
#pragma unroll
                        for (int j = 0; j < TN; ++j)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                *reinterpret_cast<f32x4 *>(wr + (32 * j + 8 * q) * 4) = f32x4{acc[I][j][4 * q], acc[I][j][4 * q + 1], acc[I][j][4 * q + 2], acc[I][j][4 * q + 3]};
                    }
                    asm volatile("; accumulator block %0" ::"n"(I));  // (keeps the four cases of the switch below apart: merged, they would index the accumulators at run time, which sends them to scratch memory)
                }
            };
            switch (i) {
            case 0: put(std::integral_constant<int, 0>{}); break;
            case 1: put(std::integral_constant<int, 1>{}); break;
            case 2: put(std::integral_constant<int, 2>{}); break;
            default: put(std::integral_constant<int, 3>{}); break;
            }
        }
        // The residual of this block, out of LDS into registers, then the copy of the next block's.  The copy of
        // this block went out a block ago, in front of that block's stores; vector memory instructions complete in
        // the order of issue, so waiting until no more than those stores are outstanding (8 NH of them, when
        // nothing was masked) is waiting for the copy, and the stores stay in flight.  (Waiting for everything
        // cost 7.8 of the epilogue's 16.6 us on the 4096^3 chain: a round trip to memory in every block.)
        u32x2 rv[F32 ? 1 : 8][F32 ? 1 : NH];
        if constexpr (!F32) {
            if (res_idx >= 0) {
                if (FULL && a.dst) wait_vmcnt<8 * NH>();
                else wait_vmcnt<0>();
                const char *rb = smem + ((i & 1) ? RES1_OFF : RES0_OFF) + wave * RES_WAVE;
#pragma unroll
                for (int it = 0; it < 8; ++it)
#pragma unroll
                    for (int hc = 0; hc < NH; ++hc) rv[it][hc] = *reinterpret_cast<const u32x2 *>(rb + (4 * it + rsub) * (WN * 2) + hc * 128 + cl * 8);
                if (i + 1 < TM && (FULL || m_blk + 32 < M)) issue_residual(i + 1, (i + 1) & 1);
            }
        }

        // The two 16-row halves of the block one after the other (half the values in registers at a time).
        auto half_pass = [&](auto hf_c) __attribute__((always_inline)) {
            constexpr int HF = decltype(hf_c)::value;
            constexpr int NIT = 4;  // 4 rows per iteration
            // read back row-contiguous: v[it][hc] = row 16 HF + 4 it + rsub, columns of run hc
            f32x4 v[NIT][NH];
    #pragma unroll
            for (int it = 0; it < NIT; ++it)
    #pragma unroll
                for (int hc = 0; hc < NH; ++hc) v[it][hc] = *reinterpret_cast<const f32x4 *>(ep + (16 * HF + 4 * it + rsub) * EP_STRIDE + hc * 256 + cl * 16);
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
                    if (o == res_idx) {  // staged through LDS
                        if constexpr (!F32) {
    #pragma unroll
                            for (int it = 0; it < NIT; ++it)
    #pragma unroll
                                for (int hc = 0; hc < NH; ++hc) v[it][hc] += unpack4<DTE>(rv[4 * HF + it][hc]);
                        }
                    } else {  // a further residual operand: straight from memory, clamped to stay in bounds
    #pragma unroll
                        for (int it = 0; it < NIT; ++it) {
                            const int64_t m = m_blk + 16 * HF + 4 * it + rsub;
                            const int64_t mc = m < M ? m : M - 1;
    #pragma unroll
                            for (int hc = 0; hc < NH; ++hc) {
                                if constexpr (EDGE) {
    #pragma unroll
                                    for (int e = 0; e < 4; ++e)
                                        if (n_col[hc] + e < N) v[it][hc][e] += ld_elem(op.p0, mc * op.ld + n_col[hc] + e, DTE);
                                } else {
                                    v[it][hc] += ld4<DTE>(op.p0, mc * op.ld + (n_ok[hc] ? n_col[hc] : N - 4));
                                }
                            }
                        }
                    }
                    break;
                case FLE_STORE:  // a copy of the values as they stand, rounded to the dtype; rows and columns inside the matrix only
    #pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        const int64_t m = m_blk + 16 * HF + 4 * it + rsub;
    #pragma unroll
                        for (int hc = 0; hc < NH; ++hc)
                            if (FULL || (m < M && n_ok[hc])) {
                                if constexpr (EDGE) {
    #pragma unroll
                                    for (int e = 0; e < 4; ++e)
                                        if (n_col[hc] + e < N) st_elem(const_cast<void *>(op.p0), m * op.ld + n_col[hc] + e, DTE, v[it][hc][e]);
                                } else if constexpr (F32) {
                                    *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(const_cast<void *>(op.p0)) + m * op.ld + n_col[hc]) = v[it][hc];
                                } else {
                                    constexpr int DT2 = F32 ? FLE_BF16 : DTE;
                                    *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(const_cast<void *>(op.p0)) + m * op.ld + n_col[hc]) = pack4<DT2>(v[it][hc]);
                                }
                            }
                    }
                    break;
                default: break;
                }
            }

            // row-reduction partials over this wave's WN columns, from the unrounded fp32 values.  (The choice between the
            // two kinds of partial is made once, around the four row groups, not inside each: the compiler then interleaves
            // the four chains of cross-lane steps, each of which waits two cycles on the one before.)
            float part_max[NIT];  // softmax: the partial's maximum per row of this block
            if (a.epi.row_kind >= 0) {
                const bool ln = a.epi.row_kind == FLE_LAYERNORM;
                float s0[NIT], s1[NIT];
                if (ln) {
                    float sum[NIT];
    #pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        sum[it] = 0.0f;
    #pragma unroll
                        for (int hc = 0; hc < NH; ++hc)
                            if (FULL || n_ok[hc]) {
                                if constexpr (EDGE) {
    #pragma unroll
                                    for (int e = 0; e < 4; ++e)
                                        if (n_col[hc] + e < N) sum[it] += v[it][hc][e];
                                } else {
                                    sum[it] += (v[it][hc][0] + v[it][hc][1]) + (v[it][hc][2] + v[it][hc][3]);
                                }
                            }
                    }
    #pragma unroll
                    for (int it = 0; it < NIT; ++it) s0[it] = row16_allreduce<false>(sum[it]) * inv_cnt;
    #pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        float m2 = 0.0f;
    #pragma unroll
                        for (int hc = 0; hc < NH; ++hc)
                            if (FULL || n_ok[hc])
    #pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (!EDGE || n_col[hc] + e < N) m2 += (v[it][hc][e] - s0[it]) * (v[it][hc][e] - s0[it]);
                        s1[it] = m2;
                    }
    #pragma unroll
                    for (int it = 0; it < NIT; ++it) s1[it] = row16_allreduce<false>(s1[it]);
                } else {
    #pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        float mx = -INFINITY;
    #pragma unroll
                        for (int hc = 0; hc < NH; ++hc)
                            if (FULL || n_ok[hc]) {
                                if constexpr (EDGE) {
    #pragma unroll
                                    for (int e = 0; e < 4; ++e)
                                        if (n_col[hc] + e < N) mx = fmaxf(mx, v[it][hc][e]);
                                } else {
                                    mx = fmaxf(fmaxf(mx, fmaxf(v[it][hc][0], v[it][hc][1])), fmaxf(v[it][hc][2], v[it][hc][3]));
                                }
                            }
                        s0[it] = mx;
                    }
    #pragma unroll
                    for (int it = 0; it < NIT; ++it) s0[it] = row16_allreduce<true>(s0[it]);
    #pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        float se = 0.0f;
    #pragma unroll
                        for (int hc = 0; hc < NH; ++hc)
                            if (FULL || n_ok[hc])
    #pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (!EDGE || n_col[hc] + e < N) se += __expf(v[it][hc][e] - s0[it]);
                        s1[it] = se;
                    }
    #pragma unroll
                    for (int it = 0; it < NIT; ++it) s1[it] = row16_allreduce<false>(s1[it]);
                }
    #pragma unroll
                for (int it = 0; it < NIT; ++it) {
                    const int64_t m = m_blk + 16 * HF + 4 * it + rsub;
                    part_max[it] = s0[it];
                    if (cl == 0 && (FULL || m < M)) *reinterpret_cast<float2 *>(a.partials + (m * a.np + p_idx) * 2) = make_float2(s0[it], s1[it]);
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
                    const int64_t m = m_blk + 16 * HF + 4 * it + rsub;
    #pragma unroll
                    for (int hc = 0; hc < NH; ++hc)
                        if (FULL || (m < M && n_ok[hc])) {
                            if constexpr (EDGE) {
    #pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (n_col[hc] + e < N) st_elem(dst, m * a.ldd + n_col[hc] + e, a.dst_f32 ? FLE_F32 : DTE, v[it][hc][e]);
                            } else if (F32 || a.dst_f32) {
                                f32x4 *q = reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(dst) + m * a.ldd + n_col[hc]);
                                if (stream_out) __builtin_nontemporal_store(v[it][hc], q);
                                else *q = v[it][hc];
                            } else {
                                u32x2 *q = reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(dst) + m * a.ldd + n_col[hc]);
                                constexpr int DT2 = F32 ? FLE_BF16 : DTE;  // (this branch is never taken for fp32 problems)
                                if (stream_out) __builtin_nontemporal_store(pack4<DT2>(v[it][hc]), q);
                                else *q = pack4<DT2>(v[it][hc]);
                            }
                        }
                }
            }
        };
        half_pass(I0{});
        half_pass(I1{});
    };
    if (!EDGE && m_wave + WM <= M && n_wave + WN <= N) {
#pragma unroll 1
        for (int i = 0; i < TM; ++i) block(i, std::true_type{});
    } else {
#pragma unroll 1
        for (int i = 0; i < TM && m_wave + 32 * i < M; ++i) block(i, std::false_type{});
    }
}

// 256 x 256: one workgroup per CU (160 KB of LDS, 512 registers per lane).  DT: fle_dtype of the operands.
// fp32 operands run on the same tiles: a K step is 32 elements and each fragment pair feeds four
// v_mfma_f32_32x32x2_f32 (64 cycles each), so the loop is bound by the matrix pipe with room to spare.
template <int DT, bool EDGE, int MF = (DT == FLE_F32 || DT == FLE_F8E4M3 ? 32 : 16), int C1 = -1, bool MX = false>
__global__ __launch_bounds__(256) void gemm_tiled_256(const GemmArgs a) { gemm_tiled_body<256, 256, DT, EDGE, false, MF, C1, MX>(a, whole_matrix_tile<256>(a)); }
// 128 x 128: two workgroups per CU (80 KB of LDS each), so at most 256 registers per lane.
template <int DT, bool EDGE, int MF = (DT == FLE_F32 || DT == FLE_F8E4M3 ? 32 : 16), int C1 = -1, bool MX = false>
__global__ __launch_bounds__(256, 2) void gemm_tiled_128(const GemmArgs a) { gemm_tiled_body<128, 128, DT, EDGE, false, MF, C1, MX>(a, whole_matrix_tile<128>(a)); }

// Grouped forms: the same tiles, with the tile -> rows mapping taken from the group offsets.
template <int DT, bool EDGE>
__global__ __launch_bounds__(256) void gemm_tiled_grouped_256(const GemmArgs a, const GroupArgs ga) {
    TileRef t;
    if (!grouped_tile<256>(a, ga, t)) return;
    gemm_tiled_body<256, 256, DT, EDGE, false, (DT == FLE_F32 || DT == FLE_F8E4M3 ? 32 : 16)>(a, t);
}
template <int DT, bool EDGE, bool W_NT>
__global__ __launch_bounds__(256, 2) void gemm_tiled_grouped_128(const GemmArgs a, const GroupArgs ga) {
    TileRef t;
    if (!grouped_tile<128>(a, ga, t)) return;
    gemm_tiled_body<128, 128, DT, EDGE, W_NT, (DT == FLE_F32 || DT == FLE_F8E4M3 ? 32 : 16)>(a, t);
}

}  // namespace fle
