// Deferred-epilogue persistent 8-bit "NT" GEMM for gfx950 (FP8 E4M3 / INT8):
// the large-shape kernel of the per-tensor FP8 linear (Sec. 4.3) and of the
// W8A8 linear (Sec. 4.4) when M and N are multiples of 256 and K of 128.
//
// One workgroup of four waves per CU (one wave per SIMD, so a wave may hold
// 512 registers): a 256x256 output tile, each wave a 128x128 sub-tile = 4x4
// MFMA blocks of 32x32 = 256 accumulator registers.  Operands stream through
// two 64 KB LDS stages of 128 bytes of K (direct-to-LDS loads, whole 128-byte
// lines per row), as one uninterrupted stream over all the tiles a workgroup
// owns: the loads of the next tile's first stages are issued while the current
// tile is still being multiplied.
//
// A wave issues one instruction every four cycles and a 32x32x64 MFMA keeps the
// matrix pipe busy for 64, so an MFMA "slot" has room for about sixteen
// instructions: everything besides the MFMAs (fragment reads, operand loads,
// the whole epilogue) is cut into pieces of a few instructions and dealt out
// over the slots.
//
//  * Operand stream: the B half of an LDS stage has been read by slot 16 of the
//    stage, the A half by slot 28; each half gets its own workgroup barrier and
//    is refilled right behind it, at most one load instruction per slot.  The
//    wait in front of the second barrier leaves the youngest eight loads in
//    flight, so the load pipe never drains.
//  * Epilogue: a block of accumulators is final after its MFMA in the tile's
//    last K slab.  From two slots later on it is scaled and rounded to bf16 in
//    place (half a block per slot, into 128 packed registers; the accumulator
//    reads are issued back to back, a read followed at once by its use stalls),
//    and the next tile's first MFMA on that block starts from zero (no
//    clearing).  The packed values are written out *during the next tile*, a
//    few instructions per slot: a lane of the MFMA layout holds four consecutive
//    columns of a row and lane + 32 the next four, so one v_permlane32_swap per
//    register pair gives every lane eight consecutive columns (16 bytes) to
//    store; the TWEO penalty terms (Sec. 3.3; the term of the value as stored)
//    are added from the same registers.  No LDS round trip: extra LDS
//    instructions cost the matrix pipe about 25 cycles each.
//
// Fragments are single-buffered in registers and refilled just in time: the
// A fragment of row i+1 is read while row i multiplies, the B fragment j of the
// next K slab is read right after its last use in the current slab.
#pragma once
#include <utility>
#include "gemm_common.h"

namespace tweo {

// MT: 32-row blocks per wave along M (4: 256x256 tile, 3: 192x256 tile, for row counts that
// 256 quantises badly, e.g. weight gradients with fewer tiles than CUs).  The 192-row variant
// also takes a ragged last row of tiles (M not a multiple of 192): rows past M are loaded as
// copies of the last valid row and neither stored nor counted in the penalty.
template <int MT_>
struct DeferTile {
    static constexpr int MT = MT_, NB = MT * 4;           // MFMA blocks per wave: MT x 4
    static constexpr int BM = MT * 64, BN = 256, BK = 128, NWAVES = 4, THREADS = 256;
    static constexpr int A_BYTES = BM * BK, STAGE_BYTES = (BM + BN) * BK;
    static constexpr int STAGE_STRIDE = 65536;            // power of two: buffers are toggled by XOR
    static constexpr int LDS_BYTES = 2 * STAGE_STRIDE;
    static constexpr int SLAB = NB, SLOTS = 2 * NB;       // MFMA slots per K slab / per stage
    static constexpr int NA = BM / 32, NBP = BN / 32;     // operand pieces per wave per stage
    static constexpr int STEPS_PER_BLOCK = 8;             // micro-steps of writing a block out
    static constexpr int DRAIN_STEPS = NB * STEPS_PER_BLOCK;
    static constexpr int HALVES = 2 * NB;                 // half blocks to convert per tile
    static constexpr int PARTIALS_PER_WG = NWAVES;       // one fp32 sum per wave
    static constexpr bool EDGE = MT == 3;                 // M may end inside the last row of tiles
    static_assert(STAGE_BYTES <= STAGE_STRIDE && LDS_BYTES <= 160 * 1024, "LDS capacity");
    static_assert(SLAB + NBP <= SLOTS - 4 && NA / 2 <= 4, "operand pieces fit their slots");
    // Half block h of the finishing tile is converted in this slot, counted from the start of
    // the tile's last stage (slots SLOTS.. are the next tile's first stage).  Block b = h/2 gets
    // its last MFMA in slot SLAB + b and its first MFMA of the next tile in slot SLOTS + b: the
    // conversions are spread over the slots SLAB + 2 .. SLOTS + NB - 2.
    static constexpr int convert_slot(int h) { return SLAB + 2 + h * (2 * NB - 3) / (2 * NB); }
    // Slots of a stage that issue an operand load, and the slots left for the write-out: a
    // 16-byte-per-lane store of 32 different rows keeps the address unit busy for as long as four
    // operand loads, so the two are kept apart.
    __host__ __device__ __attribute__((always_inline)) static constexpr bool load_slot(int t)
    {
        return t < NA / 2 || (t >= SLAB && t < SLAB + NBP) || (t >= SLOTS - 4 && t < SLOTS - 4 + NA / 2);
    }
    static constexpr int FREE = SLOTS - NA - NBP;         // slots without a load, per stage
    __host__ __device__ __attribute__((always_inline)) static constexpr int clamp(int v, int hi) { return v < 0 ? 0 : (v > hi ? hi : v); }
    __host__ __device__ __attribute__((always_inline)) static constexpr int free_index(int t)                // how many of them lie before slot t
    {
        return t - clamp(t, NA / 2) - clamp(t - SLAB, NBP) - clamp(t - (SLOTS - 4), NA / 2);
    }
};

// Where the write-out of a tile happens inside the first D stages of the next one (LINES).  Per
// pair of neighbouring blocks there are 20 arithmetic micro-steps (penalty terms, lane exchanges)
// and 4 stores.  The arithmetic is dealt evenly over all slots from slot 2 on; a store goes to the
// first slot without an operand load (the two share the address unit) after its pair's arithmetic,
// one store per slot.  alu_lo/alu_hi: the arithmetic steps of slot s; store: the store of slot s or -1.
template <typename T, int D>
struct DrainPlan {
    static constexpr int NSLOT = D * T::SLOTS, PAIRS = T::NB / 2, ALU = PAIRS * 20, STORES = PAIRS * 4;
    int alu_lo[NSLOT], alu_hi[NSLOT], store[NSLOT];
    bool ok;
};
template <typename T, int D>
constexpr DrainPlan<T, D> make_drain_plan()
{
    using P = DrainPlan<T, D>;
    constexpr int FIRST = 2;
    // the arithmetic ends as late as still leaves store slots for the last pairs (the last slots
    // of a stage carry loads)
    for (int end = P::NSLOT - 8; end > P::NSLOT / 2; --end) {
        P p{};
        int at[P::ALU] = {};
        for (int a = 0; a < P::ALU; ++a)
            at[a] = FIRST + (int)((long long)a * (end - FIRST) / P::ALU);
        for (int s = 0, a = 0; s < P::NSLOT; ++s) {
            p.alu_lo[s] = a;
            while (a < P::ALU && at[a] == s)
                ++a;
            p.alu_hi[s] = a;
            p.store[s] = -1;
        }
        int s = 0;
        p.ok = true;
        for (int st = 0; st < P::STORES && p.ok; ++st) {
            const int ready = at[(st / 4) * 20 + 19] + 1;  // the slot after the pair's last exchange
            if (s < ready)
                s = ready;
            while (s < P::NSLOT && T::load_slot(s % T::SLOTS))
                ++s;
            if (s >= P::NSLOT)
                p.ok = false;
            else
                p.store[s++] = st;
        }
        if (p.ok)
            return p;
    }
    P bad{};
    bad.ok = false;
    return bad;
}

template <typename T, int D>
struct DrainPlanOf {  // evaluated once per tile shape and D, not once per slot body
    static constexpr DrainPlan<T, D> value = make_drain_plan<T, D>();
};

// PMODE: 4 = TWEO penalty with p = 4 (the paper's setting), 0 = none.  D: number of stages of
// the next tile over which the write-out of a tile is spread (3, 5, 7 or 15; needs K >= 128 * (D + 1):
// the tile's last stage, which converts its own blocks, takes no part in it).
// calls f(integral_constant<int, 0>), f(integral_constant<int, 1>), ... in order
template <typename F, int... Is>
__device__ __forceinline__ void for_each_constant(std::integer_sequence<int, Is...>, F &f)
{
    (f(std::integral_constant<int, Is>{}), ...);
}

// A_E5M2 (FP8 only): the A operand holds E5M2 codes (the gradient of the HYBRID recipe, Sec. 4.3);
// B is always E4M3.  The MFMA takes the format of each source from a modifier.
// LINES: the write-out regroups the packed values among lanes first, so that the four lanes of a
// quad store 64 contiguous bytes of one row and the matching quad of the other half-wave the next
// 64 (whole 128-byte lines, 8 rows per instruction); otherwise a lane stores 16 bytes of its own
// row (32 rows per instruction: 2.25 times the time in the store path, measured on stores that
// hit in L2).
// KSPLIT: g.ksplit workgroups share a tile; workgroup id = split * tiles + tile multiplies its run
// of K stages (at least two) and leaves the fp32 sums in g.ksplit_out in the order the lanes hold
// them (unit, wave, block, quarter, lane: every store instruction writes 1 KB contiguously);
// splitk_reduce_defer_kernel adds the runs in index order, rounds and writes the output.  One
// unit per workgroup, so nothing is deferred.
template <bool INT8, int PMODE, int D, int MT, bool A_E5M2 = false, bool LINES = true, bool KSPLIT = false>
__global__ __launch_bounds__(256, 1) void gemm_nt_defer_kernel(GemmDev g)
{
    using T = DeferTile<MT>;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = wave >> 1, wn = wave & 1;
    const int l31 = lane & 31, lh = lane >> 5;
    const int n_tiles = g.tiles_m * g.tiles_n;
    const int total = KSPLIT ? n_tiles * g.ksplit : n_tiles;
    // persistent schedule: round r hands tile ids [r*G, (r+1)*G) to the G workgroups; inside a
    // round each XCD (workgroup index mod 8) gets a contiguous run of ids
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, per_xcd = G >> 3, rem_xcd = G & 7;
    const int slot = xcd * per_xcd + (xcd < rem_xcd ? xcd : rem_xcd) + (blockIdx.x >> 3);
    if (slot >= total)
        return;
    int kt = g.K / T::BK, k_first = 0;
    if constexpr (KSPLIT) {
        const int split = slot / n_tiles, base = kt / g.ksplit, rem = kt % g.ksplit;
        k_first = split * base + (split < rem ? split : rem);
        kt = base + (split < rem ? 1 : 0);
    }

    float alpha;
    if constexpr (INT8)
        alpha = g.alpha;
    else
        alpha = (*g.s0) * (*g.s1);

    // ---- operand stream (direct-to-LDS loads), running ahead of the MFMAs -----------------
    // One instruction of a wave fills 1 KB = 8 rows x 128 B; lane -> (row, 16-byte chunk), the
    // chunk XOR-swizzled with (row/2)%8.  Piece p of an operand is its rows (p*4 + wave)*8.. .
    // A and B are two streams of their own over (tile, stage): the B half of an LDS stage is
    // released (and refilled) earlier than the A half.  An instruction costs three issue slots:
    // LDS destination = constant + buffer offset, one wait state, the load with a per-piece
    // row offset register and the stream's scalar address.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const int dma_row = lane >> 3, dma_p = lane & 7;
    uint32_t voffs[8];
    const uint32_t dma_chunk = (uint32_t)((dma_p ^ ((dma_row >> 1) + 4 * (wave & 1))) << 4);
#pragma unroll
    for (int p8 = 0; p8 < 8; ++p8)
        voffs[p8] = (uint32_t)(p8 * 32 + wave * 8 + dma_row) * (uint32_t)g.K + dma_chunk;
    // A rows of a ragged last tile are clamped to the last valid one (EDGE only)
    uint32_t voffs_a[T::EDGE ? T::NA : 1];
    struct Stream {
        const uint8_t *ptr;  // first row of the tile's panel, at the stage to load next
        int s;               // that stage
        uint32_t bufoff;     // LDS buffer it goes to: 0 or STAGE_STRIDE
    };
    Stream sa, sb;
    // Where this workgroup's tiles lie, 64 of them at a time: lane r holds the operand offsets of
    // its tile number vec_r0 + r (id = slot + number * G), worked out by the vector unit once; at a
    // tile boundary the scalar side fetches one lane's values instead of dividing (the divisions
    // of the id raster cost both streams about 250 cycles per tile when done in scalar code).
    uint32_t ta_lo = 0, ta_hi = 0, tb_lo = 0, tb_hi = 0;
    int tvalid = 0, tmv = 0, tnv = 0, vec_r0 = 0;
    auto tiles_fill = [&](int r0) {
        const int id_l = KSPLIT ? slot % n_tiles : slot + (r0 + lane) * G;
        int tm = 0, tn = 0;
        if (id_l < (KSPLIT ? n_tiles : total))
            tile_from_id(id_l, g.tiles_m, g.tiles_n, tm, tn);
        const uint64_t oa = (uint64_t)tm * T::BM * (uint64_t)g.K, ob = (uint64_t)tn * T::BN * (uint64_t)g.K;
        ta_lo = (uint32_t)oa;
        ta_hi = (uint32_t)(oa >> 32);
        tb_lo = (uint32_t)ob;
        tb_hi = (uint32_t)(ob >> 32);
        tvalid = g.M - tm * T::BM;
        tmv = tm;
        tnv = tn;
        vec_r0 = r0;
    };
    auto tile_a = [&](int r) {
        const int l = r - vec_r0;
        return g.A + (((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)ta_hi, l) << 32) |
                      (uint32_t)__builtin_amdgcn_readlane((int)ta_lo, l)) + (int64_t)k_first * T::BK;
    };
    auto tile_b = [&](int r) {
        const int l = r - vec_r0;
        return g.B + (((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)tb_hi, l) << 32) |
                      (uint32_t)__builtin_amdgcn_readlane((int)tb_lo, l)) + (int64_t)k_first * T::BK;
    };
    auto set_voffs_a = [&](int valid) {  // EDGE: rows past the matrix load the last valid one
        if constexpr (T::EDGE) {
#pragma unroll
            for (int p8 = 0; p8 < T::NA; ++p8) {
                const int r = p8 * 32 + wave * 8 + dma_row;
                voffs_a[p8] = (uint32_t)(r < valid ? r : valid - 1) * (uint32_t)g.K + dma_chunk;
            }
        }
    };
    // the tile the streams move on to while tile number r - 1 is multiplied
    const uint8_t *next_a = nullptr, *next_b = nullptr;
    int next_valid = 0, next_tm = 0, next_tn = 0;
    bool has_next = false;
    auto plan_next = [&](int r) {
        has_next = !KSPLIT && slot + r * G < total;
        if (has_next) {
            if (r - vec_r0 >= kWave)
                tiles_fill(r);
            next_a = tile_a(r);
            next_b = tile_b(r);
            next_valid = __builtin_amdgcn_readlane(tvalid, r - vec_r0);
            next_tm = __builtin_amdgcn_readlane(tmv, r - vec_r0);
            next_tn = __builtin_amdgcn_readlane(tnv, r - vec_r0);
        }
    };
    // Past the workgroup's last stage a stream keeps re-reading that stage (in bounds) into
    // buffers nobody multiplies from any more: the main loop stays free of branches.
    auto stream_advance = [&](Stream &st, bool is_b) {
        st.bufoff ^= T::STAGE_STRIDE;
        if (st.s + 1 < kt) {
            ++st.s;
            st.ptr += T::BK;
        } else if (has_next) {
            st.ptr = is_b ? next_b : next_a;
            st.s = 0;
            if (!is_b)
                set_voffs_a(next_valid);
        }
    };
    auto dma_piece_a = [&](int p8) {
        const uint32_t dst0 = lds_base + (p8 * 4 + wave) * 1024;
        asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
                     :
                     : "s"(dst0), "s"(sa.bufoff), "v"(T::EDGE ? voffs_a[T::EDGE ? p8 : 0] : voffs[p8]), "s"(sa.ptr)
                     : "memory", "m0", "scc");
    };
    auto dma_piece_b = [&](int p8) {
        const uint32_t dst0 = lds_base + T::A_BYTES + (p8 * 4 + wave) * 1024;
        asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
                     :
                     : "s"(dst0), "s"(sb.bufoff), "v"(voffs[p8]), "s"(sb.ptr)
                     : "memory", "m0", "scc");
    };

    // ---- fragment addressing ---------------------------------------------------------------
    // lane (l31, lh) reads row l31 of a 32-row block; logical chunks of slab kk:
    // FP8 4kk+2lh, 4kk+2lh+1 (32 contiguous bytes of K); INT8 4kk+lh and 4kk+2+lh
    const int sw = (l31 >> 1) & 7;
    uint32_t pa[2][2], pb[2][2];  // [slab][half]: byte offsets into smem, stage 0
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int c0 = INT8 ? 4 * kk + lh : 4 * kk + 2 * lh;
        const int c1 = INT8 ? 4 * kk + 2 + lh : 4 * kk + 2 * lh + 1;
        pa[kk][0] = (wm * MT * 32 + l31) * T::BK + ((c0 ^ sw) << 4);
        pa[kk][1] = (wm * MT * 32 + l31) * T::BK + ((c1 ^ sw) << 4);
        pb[kk][0] = T::A_BYTES + (wn * 128 + l31) * T::BK + ((c0 ^ sw) << 4);
        pb[kk][1] = T::A_BYTES + (wn * 128 + l31) * T::BK + ((c1 ^ sw) << 4);
    }
    auto flip_stage = [&]() {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                pa[kk][h] ^= T::STAGE_STRIDE;
                pb[kk][h] ^= T::STAGE_STRIDE;
            }
    };
    v8i fa[2], fb[4];
    auto load_a = [&](v8i &f, int kk, int i) {
        const v4i x = *(const v4i *)(smem + pa[kk][0] + i * 32 * T::BK);
        const v4i y = *(const v4i *)(smem + pa[kk][1] + i * 32 * T::BK);
        f = v8i{x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
    };
    auto load_b = [&](v8i &f, int kk, int j) {
        const v4i x = *(const v4i *)(smem + pb[kk][0] + j * 32 * T::BK);
        const v4i y = *(const v4i *)(smem + pb[kk][1] + j * 32 * T::BK);
        f = v8i{x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
    };

    using acc_t = typename std::conditional<INT8, v16i, v16f>::type;
    acc_t acc[MT][4];
    // The MFMAs are written as asm with accumulator-register constraints: the 256 accumulators
    // fill the accumulation register file exactly, and only a hard constraint keeps the register
    // allocator from parking blocks in VGPRs and copying them around every use.  Consecutive
    // MFMAs never touch the same block (a block recurs after 16), and the fragments come straight
    // from LDS reads (the compiler's own s_waitcnt covers asm operands).  The one software-visible
    // hazard, reading a block right after its last MFMA, is avoided by the schedule: a block is
    // converted at least two slots after that MFMA was issued.
    // the A fragment of row i of slab kk sits in fa[(kk * MT + i) % 2]
    auto mfma = [&](int kk, int i, int j) {
        const int ab = (kk * MT + i) & 1;
        if constexpr (INT8) {
            const v4i a0 = {fa[ab][0], fa[ab][1], fa[ab][2], fa[ab][3]};
            const v4i a1 = {fa[ab][4], fa[ab][5], fa[ab][6], fa[ab][7]};
            const v4i b0 = {fb[j][0], fb[j][1], fb[j][2], fb[j][3]};
            const v4i b1 = {fb[j][4], fb[j][5], fb[j][6], fb[j][7]};
            asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0\n\tv_mfma_i32_32x32x32_i8 %0, %3, %4, %0"
                         : "+a"(acc[i][j])
                         : "v"(b0), "v"(a0), "v"(b1), "v"(a1));
        } else {
            if constexpr (A_E5M2)
                asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0 blgp:1" : "+a"(acc[i][j]) : "v"(fb[j]), "v"(fa[ab]));
            else
                asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fb[j]), "v"(fa[ab]));
        }
    };
    // first MFMA of a block in a tile: accumulates onto zero
    auto mfma_first = [&](int kk, int i, int j) {
        const int ab = (kk * MT + i) & 1;
        if constexpr (INT8) {
            const v4i a0 = {fa[ab][0], fa[ab][1], fa[ab][2], fa[ab][3]};
            const v4i a1 = {fa[ab][4], fa[ab][5], fa[ab][6], fa[ab][7]};
            const v4i b0 = {fb[j][0], fb[j][1], fb[j][2], fb[j][3]};
            const v4i b1 = {fb[j][4], fb[j][5], fb[j][6], fb[j][7]};
            asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, 0\n\tv_mfma_i32_32x32x32_i8 %0, %3, %4, %0"
                         : "=&a"(acc[i][j])
                         : "v"(b0), "v"(a0), "v"(b1), "v"(a1));
        } else {
            if constexpr (A_E5M2)
                asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, 0 blgp:1" : "=&a"(acc[i][j]) : "v"(fb[j]), "v"(fa[ab]));
            else
                asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, 0" : "=&a"(acc[i][j]) : "v"(fb[j]), "v"(fa[ab]));
        }
    };

    // ---- deferred epilogue -----------------------------------------------------------------
    // packed[i][j][2q+h]: bf16 pair (rows l31, columns j*32 + 8q + 4lh + 2h, +1) of block (i, j)
    uint32_t packed[MT][4][8];
    float pen = 0.0f;
    // half h of block b = h/2 (i = b/4, j = b%4): accumulator words 8*(h%2) .. +7
    auto convert_half = [&](int h) {
        const int i = h >> 3, j = (h >> 1) & 3, q0 = (h & 1) * 2;  // block h/2 = 4i + j
        typedef typename std::conditional<INT8, int, float>::type word_t;
        word_t t[8];
        asm volatile("v_accvgpr_read_b32 %0, %8\n\tv_accvgpr_read_b32 %1, %9\n\t"
                     "v_accvgpr_read_b32 %2, %10\n\tv_accvgpr_read_b32 %3, %11\n\t"
                     "v_accvgpr_read_b32 %4, %12\n\tv_accvgpr_read_b32 %5, %13\n\t"
                     "v_accvgpr_read_b32 %6, %14\n\tv_accvgpr_read_b32 %7, %15"
                     : "=v"(t[0]), "=v"(t[1]), "=v"(t[2]), "=v"(t[3]), "=v"(t[4]), "=v"(t[5]), "=v"(t[6]), "=v"(t[7])
                     : "a"(acc[i][j][4 * q0 + 0]), "a"(acc[i][j][4 * q0 + 1]), "a"(acc[i][j][4 * q0 + 2]),
                       "a"(acc[i][j][4 * q0 + 3]), "a"(acc[i][j][4 * q0 + 4]), "a"(acc[i][j][4 * q0 + 5]),
                       "a"(acc[i][j][4 * q0 + 6]), "a"(acc[i][j][4 * q0 + 7]));
#pragma unroll
        for (int d = 0; d < 4; ++d)
            packed[i][j][2 * q0 + d] = pack_bf16x2((float)t[2 * d] * alpha, (float)t[2 * d + 1] * alpha);
        // make the four results exist here, not whenever the instruction selector gets round to
        // them (pure arithmetic floats past fences)
        asm volatile(""
                     : "+v"(packed[i][j][2 * q0]), "+v"(packed[i][j][2 * q0 + 1]),
                       "+v"(packed[i][j][2 * q0 + 2]), "+v"(packed[i][j][2 * q0 + 3]));
    };
    auto pen_word = [&](uint32_t d) {  // two stored values
        if constexpr (PMODE == 4) {
            const float t0 = bf16lo_to_f32(d), t1 = bf16hi_to_f32(d);
            const float a0 = t0 * t0, a1 = t1 * t1;
            pen = __builtin_fmaf(a0, a0, pen);
            pen = __builtin_fmaf(a1, a1, pen);
            // keep the arithmetic in this MFMA slot (otherwise it sinks to wherever the sum is
            // finally needed, out of the MFMAs' shadow)
            asm volatile("" : "+v"(pen));
        }
    };
    // Stores walk the wave's sub-tile with one scalar pointer (first row of the band of blocks
    // being written); block column and column half go into the instruction's offset field.
    // Lane (row l31, half lh) stores the 16 bytes at row l31, columns 8*lh .. 8*lh+7 of a half.
    const uint8_t *sp = nullptr;
    const int64_t rows32 = (int64_t)g.N * 64;
    const uint32_t out_lane = (uint32_t)l31 * (uint32_t)g.N * 2u + (uint32_t)lh * 16u;
    int prow_left = 0;  // EDGE: rows of the wave's sub-tile inside the matrix, for the tile in `packed`
    auto store_begin = [&](int tm, int tn) {
        if constexpr (T::EDGE)
            prow_left = g.M - tm * T::BM - wm * MT * 32;
        sp = (const uint8_t *)g.out +
             (((int64_t)tm * T::BM + wm * MT * 32) * g.N + (int64_t)tn * T::BN + wn * 128) * 2;
    };
    // Micro-step q of writing a tile out: block q / 8 (in conversion order), column half
    // P = (q % 8) / 4 (register words 4P .. 4P+3 = columns 16P .. 16P+15 of the block).  Step 0
    // of a half exchanges words between lane and lane + 32 (word 4P+2 of the lower lanes <-> word
    // 4P of the upper ones, likewise 4P+3 <-> 4P+1), after which the four words of a lane are
    // eight consecutive columns; steps 1 and 2 add the penalty terms; step 3 stores.
    auto drain_step = [&](int q) {
        const int b = q / T::STEPS_PER_BLOCK, i = b >> 2, j = b & 3;
        const int P = (q % T::STEPS_PER_BLOCK) >> 2, k = q & 3;
        uint32_t *w = &packed[i][j][4 * P];
        const bool row_ok = !T::EDGE || i * 32 + l31 < prow_left;
        if (k == 0) {
            // the swap reads its operands early: two wait states after a vector-ALU write (the
            // compiler may have placed a register copy right in front of this statement)
            asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %2\n\tv_permlane32_swap_b32 %1, %3"
                         : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]));
        } else if (k == 1) {
            if (PMODE != 0 && row_ok) {
                pen_word(w[0]);
                pen_word(w[1]);
            }
        } else if (k == 2) {
            if (PMODE != 0 && row_ok) {
                pen_word(w[2]);
                pen_word(w[3]);
            }
        } else if (row_ok) {
            const v4i v = {(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
            // a store of more than 8 bytes reads its data late: nothing may write those
            // registers in the next wait states (the compiler does not know this is a store)
            asm volatile("global_store_dwordx4 %0, %1, %2 offset:%3\n\ts_nop 1"
                         :
                         : "v"(out_lane), "v"(v), "s"(sp), "n"(j * 64 + P * 32)
                         : "memory");
        }
        if (k == 3 && j == 3 && P == 1)
            sp += rows32;
    };
    // LINES.  Arithmetic step a works on the pair of neighbouring blocks c = a / 20 (blocks 2c,
    // 2c+1 of band i: 64 columns = one 128-byte line per row), r = a % 20, with A, B the register
    // arrays of blocks 2c and 2c+1:
    //  r = 0..15  word w = r/2: penalty terms of A[w] (even r) / of B[w] (odd r), after which B[w]
    //             of the lower half-wave is exchanged with A[w] of the upper one.  After the eight
    //             exchanges lane (row, lh) holds all 32 columns of its row in block 2c+lh: 16-byte
    //             piece u = words {A[2u], A[2u+1], B[2u], B[2u+1]}.
    //  r = 16..19 dword r-16 of the four pieces: 4x4 transposition over the lanes of a quad, after
    //             which piece register u of lane a holds piece a of row 4*(row/4) + u.
    // Store step st: pair st / 4, u = st % 4: a quad writes 64 contiguous bytes of row
    // 4*(row/4) + u, the two half-waves the two halves of the line.
    const uint32_t out_quad = (uint32_t)(l31 & ~3) * (uint32_t)g.N * 2u + (uint32_t)lh * 64u + (uint32_t)(l31 & 3) * 16u;
    const int64_t row_bytes = (int64_t)g.N * 2;
    const QuadMasks qmasks = quad_masks();
    auto drain_alu = [&](int a) {
        const int c = a / 20, r = a % 20, i = c >> 1, jp = c & 1;
        uint32_t *A = packed[i][2 * jp], *B = packed[i][2 * jp + 1];
        if (r < 16) {
            const int w = r >> 1;
            if (PMODE != 0 && (!T::EDGE || i * 32 + l31 < prow_left))
                pen_word((r & 1) ? B[w] : A[w]);
            // the swap reads its operands early, and what follows may read its results early
            if (r & 1)
                asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(A[w]), "+v"(B[w]));
        } else {
            const int d = r - 16;
            uint32_t *src = (d & 2) ? B : A;
            quad_transpose(src[(d & 1)], src[2 + (d & 1)], src[4 + (d & 1)], src[6 + (d & 1)], qmasks);
        }
    };
    auto drain_store = [&](int st) {
        const int c = st / 4, u = st % 4, i = c >> 1, jp = c & 1;
        uint32_t *A = packed[i][2 * jp], *B = packed[i][2 * jp + 1];
        if (!T::EDGE || i * 32 + (l31 & ~3) + u < prow_left) {
            const v4i v = {(int)A[2 * u], (int)A[2 * u + 1], (int)B[2 * u], (int)B[2 * u + 1]};
            const uint8_t *spu = sp + u * row_bytes;
            // a store of more than 8 bytes reads its data late: nothing may write those
            // registers in the next wait states (the compiler does not know this is a store)
            // "nt": the output is not read again by this kernel; with whole lines per store the
            // streaming hint lets the memory side write them out while the GEMM still runs
            // instead of during the next kernel (measured: LLaMA block step -1.7 %, ViT -3.4 %)
            asm volatile("global_store_dwordx4 %0, %1, %2 offset:%3 nt\n\ts_nop 1"
                         :
                         : "v"(out_quad), "v"(v), "s"(spu), "n"(jp * 128)
                         : "memory");
        }
        if (u == 3 && jp == 1)
            sp += rows32;
    };

    // The penalty terms are summed per lane over every tile of the workgroup (a few thousand
    // fp32 terms), reduced over the wave once, at the end, and written as
    // partials[workgroup][wave]; the finishing kernel adds them in index order in fp64.
    // Sum of a^4 here, times 1/(tau+eps)^4 at the end.
    auto pen_flush = [&]() {
        if constexpr (PMODE != 0) {
            const float it2 = g.inv_tau * g.inv_tau;
            const float v = wave_reduce_sum(pen * (it2 * it2));
            if (lane == 0)
                g.partials[blockIdx.x * T::PARTIALS_PER_WG + wave] = v;
        }
    };

    // ---- one stage: 2 slabs x 16 MFMA slots ------------------------------------------------
    // On entry fa[0] and fb[0..3] hold the fragments of slab 0 (row 0 / all columns) of this
    // stage.  DR >= 0: this is stage DR of a tile whose predecessor is being written out: the
    // micro-steps are dealt evenly over the slots of the first D stages, from slot 2 on.  FIRST: a
    // tile starts (1: the workgroup's first tile, 2: a later one, which also converts the last
    // half blocks of its predecessor).  LAST: a tile ends: its blocks are converted as they finish.
    constexpr int W = D * T::FREE;
    // The slot number is a compile-time constant of each slot's body (the bodies are stamped out
    // from an integer sequence): which pieces a slot carries is decided by the front end, not
    // left to constant propagation through unrolled loops.
    auto stage = [&](auto dr_c, auto first_c, auto last_c) {
        constexpr int DR = decltype(dr_c)::value, FIRST = decltype(first_c)::value;
        constexpr bool LAST = decltype(last_c)::value;
        auto slot_body = [&](auto t_c) {
                {
                    constexpr int t = decltype(t_c)::value;
                    constexpr int kk = t / T::SLAB, i = (t % T::SLAB) / 4, j = t % 4;
                    if constexpr (t == T::SLAB) {
                        // every wave has read the B half of this stage (its slab-1 fragments were
                        // requested in the last four slots of slab 0): the half can be refilled
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                        block_barrier();
                    }
                    if constexpr (t == T::SLOTS - 4) {
                        // every LDS read of this stage has been issued: wait for them and for this
                        // wave's share of the next stage (everything but the eight B pieces of the
                        // stage after next, the youngest loads), then publish
                        asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
                        block_barrier();
                        flip_stage();
                    }
                    if constexpr (FIRST != 0 && kk == 0)
                        mfma_first(kk, i, j);
                    else
                        mfma(kk, i, j);
                    if constexpr (j == 0) {
                        if constexpr (i < MT - 1)
                            load_a(fa[(kk * MT + i + 1) & 1], kk, i + 1);
                        else
                            load_a(fa[((kk ^ 1) * MT) & 1], kk ^ 1, 0);  // next slab (after the flip: next stage)
                    }
                    if constexpr (i == MT - 1)
                        load_b(fb[j], kk ^ 1, j);
                    // operand stream, at most one piece per slot: A of the next stage (second
                    // half of its pieces) in the first slots, B of the stage after next right
                    // behind the first barrier (which released its buffer half), A of the stage
                    // after next (first half) behind the second barrier
                    if constexpr (t < T::NA / 2) {
                        dma_piece_a(T::NA / 2 + t);
                        if constexpr (t == T::NA / 2 - 1)
                            stream_advance(sa, false);
                    } else if constexpr (t >= T::SLAB && t < T::SLAB + T::NBP) {
                        dma_piece_b(t - T::SLAB);
                        if constexpr (t == T::SLAB + T::NBP - 1)
                            stream_advance(sb, true);
                    } else if constexpr (t >= T::SLOTS - 4 && t < T::SLOTS - 4 + T::NA / 2) {
                        dma_piece_a(t - (T::SLOTS - 4));
                    }
                    // conversion of the tile that ends here / ended in the previous stage
#pragma unroll
                    for (int h = 0; h < T::HALVES; ++h)
                        if ((LAST && T::convert_slot(h) == t) || (FIRST == 2 && T::convert_slot(h) == t + T::SLOTS))
                            convert_half(h);
                    // write-out of the previous tile
                    if constexpr (DR >= 0 && LINES) {
                        using Plan = DrainPlanOf<T, D>;
                        static_assert(Plan::value.ok, "the write-out fits the first D stages");
                        constexpr int ds = DR * T::SLOTS + t;
                        constexpr int a_lo = Plan::value.alu_lo[ds], a_hi = Plan::value.alu_hi[ds], st = Plan::value.store[ds];
                        static_assert(a_hi - a_lo <= 3, "at most three arithmetic steps per slot");
                        if constexpr (a_lo < a_hi)
                            drain_alu(a_lo);
                        if constexpr (a_lo + 1 < a_hi)
                            drain_alu(a_lo + 1);
                        if constexpr (a_lo + 2 < a_hi)
                            drain_alu(a_lo + 2);
                        if constexpr (st >= 0)
                            drain_store(st);
                    } else if constexpr (DR >= 0 && !T::load_slot(t)) {
                        constexpr int w = DR * T::FREE + T::free_index(t);
                        constexpr int q_lo = (w * T::DRAIN_STEPS + W - 1) / W;
                        constexpr int q_hi = ((w + 1) * T::DRAIN_STEPS + W - 1) / W;
                        static_assert(T::DRAIN_STEPS <= 3 * W, "at most three micro-steps per slot");
                        if constexpr (q_lo < q_hi)
                            drain_step(q_lo);
                        if constexpr (q_lo + 1 < q_hi)
                            drain_step(q_lo + 1);
                        if constexpr (q_lo + 2 < q_hi)
                            drain_step(q_lo + 2);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
        };
        for_each_constant(std::make_integer_sequence<int, T::SLOTS>{}, slot_body);
    };
    using std::integral_constant;
    using std::true_type;
    using std::false_type;
    typedef integral_constant<int, -1> no_drain;
    typedef integral_constant<int, 0> mid;

    // ---- prologue: stage 0 whole, B of stage 1, the first half of the A pieces of stage 1 ----
    tiles_fill(0);
    sa.bufoff = sb.bufoff = 0;
    sa.s = sb.s = 0;
    sa.ptr = tile_a(0);
    sb.ptr = tile_b(0);
    set_voffs_a(__builtin_amdgcn_readlane(tvalid, 0));
    const int first_tm = __builtin_amdgcn_readlane(tmv, 0), first_tn = __builtin_amdgcn_readlane(tnv, 0);
    plan_next(1);
#pragma unroll
    for (int p8 = 0; p8 < T::NA; ++p8)
        dma_piece_a(p8);
    stream_advance(sa, false);
#pragma unroll
    for (int r = 0; r < 2; ++r) {
#pragma unroll
        for (int p8 = 0; p8 < T::NBP; ++p8)
            dma_piece_b(p8);
        stream_advance(sb, true);
    }
#pragma unroll
    for (int p8 = 0; p8 < T::NA / 2; ++p8)
        dma_piece_a(p8);
    wait_vmcnt<T::NBP + T::NA / 2>();
    block_barrier();
    load_a(fa[0], 0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        load_b(fb[j], 0, j);

    if constexpr (KSPLIT) {
        stage(no_drain{}, integral_constant<int, 1>{}, false_type{});
        for (int s = 1; s < kt; ++s)
            stage(no_drain{}, mid{}, false_type{});
        // the last MFMAs are still in the pipe (the hardware does not interlock an accumulator
        // read written as asm against them): a few hundred cycles
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7\n\ts_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
        wait_vmcnt<0>();
        float4 *dst = (float4 *)g.ksplit_out + ((int64_t)slot * T::NWAVES + wave) * (T::NB * 4 * kWave) + lane;
#pragma unroll
        for (int b = 0; b < T::NB; ++b)
#pragma unroll
            for (int hq = 0; hq < 2; ++hq) {
                float t[8];
                asm volatile("v_accvgpr_read_b32 %0, %8\n\tv_accvgpr_read_b32 %1, %9\n\t"
                             "v_accvgpr_read_b32 %2, %10\n\tv_accvgpr_read_b32 %3, %11\n\t"
                             "v_accvgpr_read_b32 %4, %12\n\tv_accvgpr_read_b32 %5, %13\n\t"
                             "v_accvgpr_read_b32 %6, %14\n\tv_accvgpr_read_b32 %7, %15"
                             : "=v"(t[0]), "=v"(t[1]), "=v"(t[2]), "=v"(t[3]), "=v"(t[4]), "=v"(t[5]), "=v"(t[6]), "=v"(t[7])
                             : "a"(acc[b >> 2][b & 3][8 * hq + 0]), "a"(acc[b >> 2][b & 3][8 * hq + 1]),
                               "a"(acc[b >> 2][b & 3][8 * hq + 2]), "a"(acc[b >> 2][b & 3][8 * hq + 3]),
                               "a"(acc[b >> 2][b & 3][8 * hq + 4]), "a"(acc[b >> 2][b & 3][8 * hq + 5]),
                               "a"(acc[b >> 2][b & 3][8 * hq + 6]), "a"(acc[b >> 2][b & 3][8 * hq + 7]));
                dst[(b * 4 + 2 * hq) * kWave] = make_float4(t[0], t[1], t[2], t[3]);
                dst[(b * 4 + 2 * hq + 1) * kWave] = make_float4(t[4], t[5], t[6], t[7]);
            }
        return;
    }
    // first tile: nothing to write out yet
    int id = slot;
    {
        const int tm = first_tm, tn = first_tn;
        stage(no_drain{}, integral_constant<int, 1>{}, false_type{});
        for (int s = 1; s < kt - 1; ++s)
            stage(no_drain{}, mid{}, false_type{});
        stage(no_drain{}, mid{}, true_type{});
        store_begin(tm, tn);
    }
    // every further tile writes its predecessor out during its first D stages
    int round = 0;
    for (id += G; id < total; id += G) {
        const int tm = next_tm, tn = next_tn;  // what the last plan_next fetched: this tile
        ++round;
        plan_next(round + 1);
        stage(integral_constant<int, 0>{}, integral_constant<int, 2>{}, false_type{});
        stage(integral_constant<int, 1>{}, mid{}, false_type{});
        stage(integral_constant<int, 2>{}, mid{}, false_type{});
        if constexpr (D >= 5) {
            stage(integral_constant<int, 3>{}, mid{}, false_type{});
            stage(integral_constant<int, 4>{}, mid{}, false_type{});
        }
        if constexpr (D >= 7) {
            stage(integral_constant<int, 5>{}, mid{}, false_type{});
            stage(integral_constant<int, 6>{}, mid{}, false_type{});
        }
        if constexpr (D >= 15) {
            stage(integral_constant<int, 7>{}, mid{}, false_type{});
            stage(integral_constant<int, 8>{}, mid{}, false_type{});
            stage(integral_constant<int, 9>{}, mid{}, false_type{});
            stage(integral_constant<int, 10>{}, mid{}, false_type{});
            stage(integral_constant<int, 11>{}, mid{}, false_type{});
            stage(integral_constant<int, 12>{}, mid{}, false_type{});
            stage(integral_constant<int, 13>{}, mid{}, false_type{});
            stage(integral_constant<int, 14>{}, mid{}, false_type{});
        }
        for (int s = D; s < kt - 1; ++s)
            stage(no_drain{}, mid{}, false_type{});
        stage(no_drain{}, mid{}, true_type{});
        store_begin(tm, tn);
    }
    // The workgroup's last tile: the rest of its conversion, then its write-out with nothing to
    // hide it under.  Here every CU of the chip stores at the same time, and 16-byte pieces would
    // queue up at the L2s (eight times the requests of whole lines).  The LDS is idle now, so a
    // band of the wave's sub-tile (32 rows x 128 columns) goes through a wave-private 32 KB of
    // the stage buffers and comes back with 16 lanes per row: whole 128-byte lines per store.
#pragma unroll
    for (int h = 0; h < T::HALVES; ++h)
        if (T::convert_slot(h) >= T::SLOTS) {
            convert_half(h);
            __builtin_amdgcn_sched_barrier(0);
        }
    wait_vmcnt<0>();  // the operand stream's last (unused) loads have landed in the stage buffers
    block_barrier();  // ... and every wave is done reading them
    {
        constexpr int ROW = 256 + 16;  // bytes: 128 bf16 + padding
        uint8_t *tb = smem + wave * 32768;
        uint8_t *tb_wr = tb + l31 * ROW + lh * 8;
        const uint8_t *tb_rd = tb + (lane >> 4) * ROW + (lane & 15) * 16;
        const uint32_t lane_off = (uint32_t)(lane >> 4) * (uint32_t)g.N * 2u + (uint32_t)(lane & 15) * 16u;
        const int64_t rows4 = (int64_t)g.N * 8;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *(uint2 *)(tb_wr + j * 64 + q * 16) = make_uint2(packed[i][j][2 * q], packed[i][j][2 * q + 1]);
#pragma unroll
            for (int ps = 0; ps < 8; ++ps) {
                const v4i d = *(const v4i *)(tb_rd + ps * 4 * ROW);
                if (!T::EDGE || i * 32 + ps * 4 + (lane >> 4) < prow_left) {
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        pen_word((uint32_t)d[w]);
                    asm volatile("global_store_dwordx4 %0, %1, %2 nt\n\ts_nop 1" : : "v"(lane_off), "v"(d), "s"(sp) : "memory");
                }
                sp += rows4;
            }
        }
    }
    pen_flush();
}

}  // namespace tweo
