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
// What is new here is where the epilogue runs.  When a tile's last MFMA is
// done, the accumulators are scaled and rounded to bf16 in place (128 packed
// registers) and the next tile's MFMAs start at once; the packed values are
// written out *during the first stages of the next tile*: a few instructions
// after each MFMA pass them through a wave-private LDS strip (so that stores
// cover whole 128-byte lines), add their TWEO penalty terms (Sec. 3.3; the
// term of the value as stored) and store them.  The matrix pipe therefore only
// waits for the conversion, not for the LDS round trip, the stores or the
// penalty arithmetic.
//
// Fragments are single-buffered in registers and refilled just in time: the
// A fragment of row i+1 is read while row i multiplies, the B fragment j of the
// next K slab is read right after its last use in the current slab.  One
// workgroup barrier per stage, placed before the last MFMA row of the stage:
// at that point every LDS read of the stage has been issued and waited for, so
// the barrier both publishes the next stage and frees this one for the loads
// of the stage after next.
#pragma once
#include "gemm_common.h"

namespace tweo {

struct DeferTile {
    static constexpr int BM = 256, BN = 256, BK = 128, NWAVES = 4, THREADS = 256;
    static constexpr int A_BYTES = BM * BK, STAGE_BYTES = (BM + BN) * BK;
    static constexpr int STRIP_ROW = 128 + 16;            // 64 bf16 + padding (conflict-free)
    static constexpr int STRIP_BYTES = 32 * STRIP_ROW;    // one 32x64 unit per wave
    static constexpr int STRIP_OFFSET = 2 * STAGE_BYTES;
    static constexpr int LDS_BYTES = STRIP_OFFSET + NWAVES * STRIP_BYTES;
    static constexpr int PIECES = 16;                     // DMA instructions per wave per stage
    static constexpr int UNITS = 8;                       // 32x64 output units per wave per tile
    static constexpr int PARTIALS_PER_WG = NWAVES;       // one fp32 sum per wave
    static_assert(LDS_BYTES <= 160 * 1024, "LDS capacity");
};

// PMODE: 4 = TWEO penalty with p = 4 (the paper's setting), 0 = none.  UPS: output units drained
// per stage of the next tile, 1 (needs K >= 1024) or 2 (needs K >= 512).
template <bool INT8, int PMODE, int UPS>
__global__ __launch_bounds__(DeferTile::THREADS, 1) void gemm_nt_defer_kernel(GemmDev g)
{
    using T = DeferTile;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = wave >> 1, wn = wave & 1;
    const int l31 = lane & 31, lh = lane >> 5;
    const int total = g.tiles_m * g.tiles_n;
    // persistent schedule: round r hands tile ids [r*G, (r+1)*G) to the G workgroups; inside a
    // round each XCD (workgroup index mod 8) gets a contiguous run of ids
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, per_xcd = G >> 3, rem_xcd = G & 7;
    const int slot = xcd * per_xcd + (xcd < rem_xcd ? xcd : rem_xcd) + (blockIdx.x >> 3);
    const int kt = g.K / T::BK;
    if (slot >= total)
        return;

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
#pragma unroll
    for (int p8 = 0; p8 < 8; ++p8)
        voffs[p8] = (uint32_t)(p8 * 32 + wave * 8 + dma_row) * (uint32_t)g.K +
                    (uint32_t)((dma_p ^ ((dma_row >> 1) + 4 * (wave & 1))) << 4);
    struct Stream {
        const uint8_t *ptr;  // first row of the tile's panel, at the stage to load next
        int s, id;           // that stage and its tile id
        uint32_t bufoff;     // LDS buffer it goes to: 0 or STAGE_BYTES
    };
    Stream sa, sb;
    auto stream_set = [&](Stream &st, bool is_b) {
        int tm, tn;
        tile_from_id(st.id, g.tiles_m, g.tiles_n, tm, tn);
        st.ptr = is_b ? g.B + (int64_t)tn * T::BN * g.K : g.A + (int64_t)tm * T::BM * g.K;
        st.s = 0;
    };
    // Past the workgroup's last stage a stream keeps re-reading that stage (in bounds) into
    // buffers nobody multiplies from any more: the main loop stays free of branches.
    auto stream_advance = [&](Stream &st, bool is_b) {
        st.bufoff ^= T::STAGE_BYTES;
        if (st.s + 1 < kt) {
            ++st.s;
            st.ptr += T::BK;
        } else if (st.id + G < total) {
            st.id += G;
            stream_set(st, is_b);
        }
    };
    auto dma_piece_a = [&](int p8) {
        const uint32_t dst0 = lds_base + (p8 * 4 + wave) * 1024;
        asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
                     :
                     : "s"(dst0), "s"(sa.bufoff), "v"(voffs[p8]), "s"(sa.ptr)
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
        pa[kk][0] = (wm * 128 + l31) * T::BK + ((c0 ^ sw) << 4);
        pa[kk][1] = (wm * 128 + l31) * T::BK + ((c1 ^ sw) << 4);
        pb[kk][0] = T::A_BYTES + (wn * 128 + l31) * T::BK + ((c0 ^ sw) << 4);
        pb[kk][1] = T::A_BYTES + (wn * 128 + l31) * T::BK + ((c1 ^ sw) << 4);
    }
    auto flip_stage = [&]() {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                pa[kk][h] ^= T::STAGE_BYTES;
                pb[kk][h] ^= T::STAGE_BYTES;
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
    acc_t acc[4][4];
    // The MFMAs are written as asm with accumulator-register constraints: the 256 accumulators
    // fill the accumulation register file exactly, and only a hard constraint keeps the register
    // allocator from parking blocks in VGPRs and copying them around every use.  Consecutive
    // MFMAs never touch the same block (a block recurs after 16), and the fragments come straight
    // from LDS reads (the compiler's own s_waitcnt covers asm operands); the one software-visible
    // hazard, reading a block right after its last MFMA, is covered by the no-ops in convert().
    auto mfma = [&](int i, int j) {
        if constexpr (INT8) {
            const v4i a0 = {fa[i & 1][0], fa[i & 1][1], fa[i & 1][2], fa[i & 1][3]};
            const v4i a1 = {fa[i & 1][4], fa[i & 1][5], fa[i & 1][6], fa[i & 1][7]};
            const v4i b0 = {fb[j][0], fb[j][1], fb[j][2], fb[j][3]};
            const v4i b1 = {fb[j][4], fb[j][5], fb[j][6], fb[j][7]};
            asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0\n\tv_mfma_i32_32x32x32_i8 %0, %3, %4, %0"
                         : "+a"(acc[i][j])
                         : "v"(b0), "v"(a0), "v"(b1), "v"(a1));
        } else {
            asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fb[j]), "v"(fa[i & 1]));
        }
    };
    // A block is cleared by a multiplication of zeros: it runs on the matrix pipe, under the
    // conversion arithmetic of the other blocks.  The zero register is written once, here (the
    // compiler cannot re-create it next to a use: an MFMA must not read a register in the
    // cycles right after a vector-ALU write, and nothing pads asm statements).
    uint32_t zero_lo, zero_hi;
    asm volatile("v_mov_b32 %0, 0\n\tv_mov_b32 %1, 0\n\ts_nop 4" : "=v"(zero_lo), "=v"(zero_hi));
    auto clear_block = [&](int i, int j) {
        if constexpr (INT8) {
            const long z = (long)(((uint64_t)zero_hi << 32) | zero_lo);
            asm volatile("s_nop 4\n\tv_mfma_i32_32x32x16_i8 %0, %1, %1, 0" : "=a"(acc[i][j]) : "v"(z));
        } else {
            asm volatile("s_nop 4\n\tv_mfma_f32_32x32x2_f32 %0, %1, %1, 0" : "=a"(acc[i][j]) : "v"(zero_lo));
        }
    };

    // ---- deferred epilogue -----------------------------------------------------------------
    // packed[i][j][2q+h]: bf16 pair (rows l31, columns j*32 + 8q + 4lh + 2h, +1) of block (i, j)
    uint32_t packed[4][4][8];
    float pen = 0.0f;
    int ptm = 0, ptn = 0;  // tile whose values sit in `packed`
    uint8_t *strip = smem + T::STRIP_OFFSET + wave * T::STRIP_BYTES;
    uint8_t *strip_wr = strip + l31 * T::STRIP_ROW + lh * 8;
    const uint8_t *strip_rd = strip + (lane >> 3) * T::STRIP_ROW + (lane & 7) * 16;
    const uint32_t out_lane = ((uint32_t)(lane >> 3) * (uint32_t)g.N + (uint32_t)(lane & 7) * 8u) * 2u;
    auto convert = [&]() {
        // the last MFMA (16 passes) must have written its block before it is read
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        uint32_t chain = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // One block at a time: the empty asm ties the reads of this block behind the
                // last value of the previous one (otherwise all 256 accumulators are copied to
                // VGPRs up front and spill).
                asm volatile("" : "+a"(acc[i][j]), "+v"(chain));
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    packed[i][j][2 * q + 0] = pack_bf16x2((float)acc[i][j][4 * q + 0] * alpha,
                                                          (float)acc[i][j][4 * q + 1] * alpha);
                    packed[i][j][2 * q + 1] = pack_bf16x2((float)acc[i][j][4 * q + 2] * alpha,
                                                          (float)acc[i][j][4 * q + 3] * alpha);
                }
                // ... and this one makes the eight results exist here, not whenever the
                // instruction selector gets round to them (pure arithmetic floats past fences)
                asm volatile(""
                             : "+v"(packed[i][j][0]), "+v"(packed[i][j][1]), "+v"(packed[i][j][2]),
                               "+v"(packed[i][j][3]), "+v"(packed[i][j][4]), "+v"(packed[i][j][5]),
                               "+v"(packed[i][j][6]), "+v"(packed[i][j][7]));
                chain = packed[i][j][7];
                clear_block(i, j);
                __builtin_amdgcn_sched_barrier(0);
            }
    };
    // unit u = (band i = u/2, column half jh = u%2): 32 rows x 64 columns of the wave's sub-tile
    auto unit_write = [&](int u) {
        const int i = u >> 1, jh = u & 1;
#pragma unroll
        for (int jl = 0; jl < 2; ++jl)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(uint2 *)(strip_wr + jl * 64 + q * 16) =
                    make_uint2(packed[i][2 * jh + jl][2 * q], packed[i][2 * jh + jl][2 * q + 1]);
    };
    v4i dr[2];  // values of the pass being written out, and of the next one (read ahead)
    auto unit_read = [&](int ps) { dr[ps & 1] = *(const v4i *)(strip_rd + ps * 8 * T::STRIP_ROW); };
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
    auto unit_store = [&](int u, int ps) {
        const int i = u >> 1, jh = u & 1;
        const int64_t row = (int64_t)ptm * T::BM + wm * 128 + i * 32 + ps * 8;
        const int64_t col = (int64_t)ptn * T::BN + wn * 128 + jh * 64;
        // scalar base + one shared 32-bit lane offset: no per-store address registers
        const uint8_t *base = (const uint8_t *)g.out + (row * g.N + col) * 2;
#ifndef EXP_NOSTORE
        asm volatile("global_store_dwordx4 %0, %1, %2" : : "v"(out_lane), "v"(dr[ps & 1]), "s"(base) : "memory");
#else
        asm volatile("; no store %0 %1 %2" : : "v"(out_lane), "v"(dr[ps & 1]), "s"(base) : "memory");
#endif
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
    // Micro-steps of draining, one per MFMA slot.  A unit: step 0 writes it to the strip, step 1
    // reads pass 0 back; then each pass takes 4 (UPS == 1) or 2 (UPS == 2) steps, each adding a
    // share of the pass's penalty terms; the first also reads the next pass ahead (so that no
    // step waits for LDS), the last stores the pass.  UPS == 2 appends the second unit.
    auto drain_step = [&](int ua, int st) {
        constexpr int SPP = UPS == 1 ? 4 : 2;      // steps per pass
        constexpr int WPS = 4 / SPP;               // dwords of the pass per step
        constexpr int PER_UNIT = 2 + 4 * SPP;
        if (st < 0 || st >= UPS * PER_UNIT)
            return;
        const int u = ua + st / PER_UNIT, k = st % PER_UNIT;
        if (k == 0) {
            unit_write(u);
        } else if (k == 1) {
            unit_read(0);
        } else {
            const int ps = (k - 2) / SPP, part = (k - 2) % SPP;
            if (part == 0 && ps < 3)
                unit_read(ps + 1);
#pragma unroll
            for (int w = 0; w < WPS; ++w)
                pen_word((uint32_t)dr[ps & 1][part * WPS + w]);
            if (part == SPP - 1)
                unit_store(u, ps);
        }
    };
    auto drain_units_now = [&](int first_unit) {  // not overlapped: the rest of a tile, at once
#pragma unroll
        for (int u = 0; u < T::UNITS; ++u)
            if (u >= first_unit) {
                unit_write(u);
#pragma unroll
                for (int ps = 0; ps < 4; ++ps) {
                    unit_read(ps);
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        pen_word((uint32_t)dr[ps & 1][w]);
                    unit_store(u, ps);
                }
            }
    };

#ifdef TWEO_DEFER_STAMPS
    int stamp_n = 0;
#endif
    // ---- one stage: 2 slabs x 16 MFMA slots ------------------------------------------------
    // On entry fa[0] and fb[0..3] hold the fragments of slab 0 (row 0 / all columns) of this
    // stage.  DR >= 0: drain units UPS*DR .. UPS*DR + UPS-1 of the previous tile along the way.
    auto stage = [&](auto dr_c) {
        constexpr int DR = decltype(dr_c)::value;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = kk * 16 + i * 4 + j;
                    if (t == 16) {
                        // every wave has read the B half of this stage (its slab-1 fragments were
                        // requested in slots 12..15): the half can be refilled
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                        block_barrier();
                    }
                    if (t == 28) {
                        // every LDS read of this stage has been issued: wait for them and for this
                        // wave's share of the next stage (everything but the eight B pieces of the
                        // stage after next, the youngest loads), then publish
                        asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
                        block_barrier();
                        flip_stage();
                    }
                    mfma(i, j);
                    if (j == 0) {
                        if (i < 3)
                            load_a(fa[(i + 1) & 1], kk, i + 1);
                        else
                            load_a(fa[0], kk ^ 1, 0);  // next slab (after the flip: next stage)
                    }
                    if (i == 3)
                        load_b(fb[j], kk ^ 1, j);
                    // operand stream, at most one piece per slot: A of the next stage (second
                    // half of its pieces) in slots 0..3, B of the stage after next in slots 16..23
                    // (its buffer half was released at slot 16), A of the stage after next (first
                    // half) in slots 28..31 (released at slot 28)
                    if (t < 4) {
                        dma_piece_a(4 + t);
                        if (t == 3)
                            stream_advance(sa, false);
                    } else if (t >= 16 && t < 24) {
                        dma_piece_b(t - 16);
                        if (t == 23)
                            stream_advance(sb, true);
                    } else if (t >= 28) {
                        dma_piece_a(t - 28);
                    }
                    if (DR >= 0)
                        drain_step(UPS * DR, t);
                    __builtin_amdgcn_sched_barrier(0);
                }
    };
    using std::integral_constant;

    // ---- prologue: stage 0 whole, B of stage 1, the first four A pieces of stage 1 ----------
    sa.id = sb.id = slot;
    sa.bufoff = sb.bufoff = 0;
    stream_set(sa, false);
    stream_set(sb, true);
#pragma unroll
    for (int p8 = 0; p8 < 8; ++p8)
        dma_piece_a(p8);
    stream_advance(sa, false);
#pragma unroll
    for (int r = 0; r < 2; ++r) {
#pragma unroll
        for (int p8 = 0; p8 < 8; ++p8)
            dma_piece_b(p8);
        stream_advance(sb, true);
    }
#pragma unroll
    for (int p8 = 0; p8 < 4; ++p8)
        dma_piece_a(p8);
    wait_vmcnt<12>();
    block_barrier();
    load_a(fa[0], 0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        load_b(fb[j], 0, j);

#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            clear_block(i, j);

    // first tile: nothing to drain yet
    int id = slot;
    {
        int tm, tn;
        tile_from_id(id, g.tiles_m, g.tiles_n, tm, tn);
        for (int s = 0; s < kt; ++s)
            stage(integral_constant<int, -1>{});
        convert();
        ptm = tm;
        ptn = tn;
    }
    // every further tile drains its predecessor during its first 8 / UPS stages
    for (id += G; id < total; id += G) {
        int tm, tn;
        tile_from_id(id, g.tiles_m, g.tiles_n, tm, tn);
        stage(integral_constant<int, 0>{});
        stage(integral_constant<int, 1>{});
        stage(integral_constant<int, 2>{});
        stage(integral_constant<int, 3>{});
        if constexpr (UPS == 1) {
            stage(integral_constant<int, 4>{});
            stage(integral_constant<int, 5>{});
            stage(integral_constant<int, 6>{});
            stage(integral_constant<int, 7>{});
        }
        for (int s = T::UNITS / UPS; s < kt; ++s)
            stage(integral_constant<int, -1>{});
        convert();
        ptm = tm;
        ptn = tn;
    }
    drain_units_now(0);
    pen_flush();
    wait_vmcnt<0>();  // the operand stream's last (unused) loads must land before the LDS is released
}

}  // namespace tweo
