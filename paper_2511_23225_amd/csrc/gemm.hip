// 8-bit "NT" GEMM for gfx950: C[M,N] = A[M,K] * B[N,K]^T with both operands
// K-contiguous, FP8 (E4M3, fp32 accumulate) or INT8 (int32 accumulate), fused
// epilogue: per-tensor dequantisation scale, optional residual add, bf16 store
// and the TWEO penalty partial sum (Sec. 3.3) of the stored values.
//
// The forward, data-gradient and weight-gradient products of a per-tensor FP8
// linear layer (Sec. 4.3) are all this one product on suitably transposed
// copies of the quantized operands; the W8A8 linear of Sec. 4.4 is its INT8
// instantiation.
//
// Structure of a workgroup: BM x BN output tile, WM x WN waves, each wave
// owning a (BM/WM) x (BN/WN) sub-tile made of 32x32 MFMA blocks
// (v_mfma_f32_32x32x64_f8f6f4 / v_mfma_i32_32x32x32_i8).  K is walked in
// slabs of 128 bytes, double buffered in LDS.  A 128-byte LDS row is split in
// eight 16-byte chunks whose position is XOR-swizzled with the row number so
// that the 16-byte-per-lane fragment reads of 32 different rows spread over
// all banks.
#include <hip/hip_ext.h>
#include "gemm_common.h"
#include "gemm_defer.h"

namespace tweo {

constexpr int kBK = 128;  // bytes of K per LDS stage

// Physical 16-byte chunk of logical chunk c in LDS row `row`.
__device__ __forceinline__ int swz(int row, int c) { return c ^ ((row ^ (row >> 3)) & 7); }

template <int BM_, int BN_, int WM_, int WN_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
    static constexpr int THREADS = WM * WN * kWave;
    static constexpr int TM = BM / WM, TN = BN / WN;  // per-wave sub-tile
    static constexpr int MT = TM / 32, NT = TN / 32;  // 32x32 MFMA blocks per wave
    static constexpr int STAGE_BYTES = (BM + BN) * kBK;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static constexpr int A_LD = BM * 8 / THREADS;  // 16-byte chunks per thread per stage
    static constexpr int B_LD = BN * 8 / THREADS;
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be made of 32x32 blocks");
    static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "loader split");
};


// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Give
// every XCD a contiguous run of tile ids, and walk tile ids in groups of 8 tile
// rows so that the 32 workgroups resident on one XCD share A and B panels.
__device__ __forceinline__ void tile_of_workgroup(int wg, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int total = tiles_m * tiles_n;
    const int per = total >> 3, rem = total & 7;
    const int xcd = wg & 7, idx = wg >> 3;
    const int id = xcd * per + (xcd < rem ? xcd : rem) + idx;
    constexpr int GROUP = 8;
    const int width = GROUP * tiles_n;
    const int group = id / width, first_m = group * GROUP;
    const int gsz = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
    const int in_group = id - group * width;
    tm = first_m + in_group % gsz;
    tn = in_group / gsz;
}

// Epilogue shared by the GEMM kernels.  An MFMA 32x32 block leaves C[m, n] in
// acc[4q + r] with m = lane%32 and n = 8q + 4*(lane/32) + r, i.e. a lane holds
// four consecutive n of one row.  To write whole 128-byte lines, each wave
// passes one 32-row band of its sub-tile at a time through its own slice of LDS
// (fp32, row stride TN*4+16 bytes: conflict-free for the 16-byte writes and
// reads) and reads it back with TN/8 lanes per row, 8 consecutive n per lane.
// That lane then applies the scale, adds the residual (16-byte load), rounds to
// bf16, stores 16 bytes, and accumulates the penalty term (|a| / (tau+eps))^p of
// the value as stored (Sec. 3.3); the terms are reduced lane -> wave ->
// workgroup into one fp32 partial per workgroup.  The caller must have placed a
// workgroup barrier between the last LDS read of the main loop and this call.
template <typename T>
struct EpiLayout {
    static constexpr int ROW_BYTES = T::TN * 4 + 16;
    static constexpr int WAVE_BYTES = 32 * ROW_BYTES;
    static constexpr int LPR = T::TN / 8;       // lanes per row when reading back
    static constexpr int ROWS_PER_PASS = kWave / LPR;
    static constexpr int PASSES = 32 / ROWS_PER_PASS;
    // bf16 staging (no residual): half the bytes, so two bands fit and band i+1 can be written
    // while band i is still being read back
    static constexpr int ROW2_BYTES = T::TN * 2 + 16;
    static constexpr int BAND2_BYTES = 32 * ROW2_BYTES;
    static_assert(2 * BAND2_BYTES <= WAVE_BYTES + 1024, "bf16 double buffer fits the slice (with slack)");
    static constexpr int SLICE_BYTES = WAVE_BYTES > 2 * BAND2_BYTES ? WAVE_BYTES : 2 * BAND2_BYTES;
    static_assert(SLICE_BYTES * (T::THREADS / kWave) <= T::LDS_BYTES, "epilogue staging fits in LDS");
};

// Specialisations: PMODE 4 (p == 4, the paper's setting), 0 (no penalty) or -1 (p read at run
// time); RES 1 / 0 (residual present / absent) or -1 (tested at run time); INTERIOR true when the
// whole tile lies inside the matrix, so that no store needs a predicate.  The interior
// specialisations are straight-line code per band: a predicate or a run-time test per pass
// would cut the code into one basic block per pass and chain sixteen LDS round trips.
template <typename T, bool INT8, int PMODE, int RES, bool INTERIOR, typename ACC, typename HOOK>
__device__ __forceinline__ void epilogue_impl(const GemmDev &g, ACC (&acc)[T::MT][T::NT],
                                              uint8_t *smem, int tm, int tn, int wm, int wn,
                                              int lane, int wave, int tid, int partial_index,
                                              HOOK &band_hook)
{
    using E = EpiLayout<T>;
    const int l31 = lane & 31, lh = lane >> 5;
    float alpha;
    if constexpr (INT8)
        alpha = g.alpha;
    else
        alpha = (*g.s0) * (*g.s1);
    float pen = 0.0f;
    uint8_t *stage = smem + wave * E::SLICE_BYTES;
    uint8_t *wr = stage + l31 * E::ROW_BYTES + lh * 16;
    const int rd_row = lane / E::LPR, rd_seg = lane % E::LPR;
    const uint8_t *rd = stage + rd_row * E::ROW_BYTES + rd_seg * 32;
    // addressing: a uniform base per (band, pass) plus one 32-bit byte offset per lane
    const int m0 = tm * T::BM + wm * T::TM, n0 = tn * T::BN + wn * T::TN;
    const uint32_t lane_off = ((uint32_t)rd_row * (uint32_t)g.N + (uint32_t)rd_seg * 8u) * 2u;
    const int64_t base_off = ((int64_t)m0 * g.N + n0) * 2;
    uint8_t *out_base = (uint8_t *)g.out + base_off;
    const uint8_t *res_base = (const uint8_t *)g.residual + base_off;
    const int rows_left = g.M - m0 - rd_row;  // row r of the sub-tile is valid for this lane if r < rows_left
    const bool n_ok = n0 + rd_seg * 8 < g.N;
    const bool has_res = RES < 0 ? g.residual != nullptr : RES != 0;
    const bool has_pen = PMODE < 0 ? g.p != 0 : PMODE != 0;
    // dequantisation steps per row / column (INT8, general form only): this lane's eight columns
    // are the same in every pass; alpha is 1 then
    const bool has_vec = INT8 && RES < 0 && g.rs != nullptr;
    float cstep[8] = {1.0f, 1.0f, 1.0f, 1.0f, 1.0f, 1.0f, 1.0f, 1.0f};
    if (has_vec) {
        alpha = 1.0f;
        if (n_ok) {
#pragma unroll
            for (int r = 0; r < 8; ++r)
                cstep[r] = g.cs[(int64_t)(n0 + rd_seg * 8 + r) * g.cs_stride];
        }
    }
    if constexpr (RES == 0 && INTERIOR && PMODE >= 0) {
        // Fast path: round to bf16 in the MFMA layout, stage packed values (half the LDS bytes),
        // two bands in flight.
        uint8_t *wr2 = stage + l31 * E::ROW2_BYTES + lh * 8;
        const uint8_t *rd2 = stage + rd_row * E::ROW2_BYTES + rd_seg * 16;
        auto write_band = [&](int i) {
#pragma unroll
            for (int j = 0; j < T::NT; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint2 pk = make_uint2(pack_bf16x2((float)acc[i][j][4 * q + 0] * alpha,
                                                            (float)acc[i][j][4 * q + 1] * alpha),
                                                pack_bf16x2((float)acc[i][j][4 * q + 2] * alpha,
                                                            (float)acc[i][j][4 * q + 3] * alpha));
                    *(uint2 *)(wr2 + (i & 1) * E::BAND2_BYTES + j * 64 + q * 16) = pk;
                }
        };
        write_band(0);
#pragma unroll
        for (int i = 0; i < T::MT; ++i) {
            band_hook(i);
            if (i + 1 < T::MT)
                write_band(i + 1);
#pragma unroll
            for (int ps = 0; ps < E::PASSES; ++ps) {
                const uint4 packed = *(const uint4 *)(rd2 + (i & 1) * E::BAND2_BYTES +
                                                      ps * E::ROWS_PER_PASS * E::ROW2_BYTES);
                const int64_t row_off = (int64_t)(i * 32 + ps * E::ROWS_PER_PASS) * g.N * 2;
                *(uint4 *)(out_base + row_off + lane_off) = packed;
                if constexpr (PMODE == 4) {
                    const float t[8] = {bf16lo_to_f32(packed.x), bf16hi_to_f32(packed.x),
                                        bf16lo_to_f32(packed.y), bf16hi_to_f32(packed.y),
                                        bf16lo_to_f32(packed.z), bf16hi_to_f32(packed.z),
                                        bf16lo_to_f32(packed.w), bf16hi_to_f32(packed.w)};
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        const float a2 = t[r] * t[r];
                        pen = __builtin_fmaf(a2, a2, pen);
                    }
                }
            }
        }
    } else {
#pragma unroll
    for (int i = 0; i < T::MT; ++i) {
        band_hook(i);  // the caller's work to spread over the bands (e.g. next tile's DMA issue)
#pragma unroll
        for (int j = 0; j < T::NT; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                v4f v;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    v[r] = (float)acc[i][j][4 * q + r] * alpha;
                *(v4f *)(wr + j * 128 + q * 32) = v;
            }
        // the wave reads only what it wrote itself: LDS executes a wave's accesses in order
#pragma unroll
        for (int ps = 0; ps < E::PASSES; ++ps) {
            const v4f lo = *(const v4f *)(rd + ps * E::ROWS_PER_PASS * E::ROW_BYTES);
            const v4f hi = *(const v4f *)(rd + ps * E::ROWS_PER_PASS * E::ROW_BYTES + 16);
            const int row_u = i * 32 + ps * E::ROWS_PER_PASS;  // uniform row of this pass
            if (INTERIOR || (row_u < rows_left && n_ok)) {
                const int64_t row_off = (int64_t)row_u * g.N * 2;
                float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                if (has_vec) {
                    const float rstep = g.rs[(int64_t)(m0 + row_u + rd_row) * g.rs_stride];
#pragma unroll
                    for (int r = 0; r < 8; ++r)
                        v[r] = (v[r] * rstep) * cstep[r];
                }
                if (has_res) {
                    const uint4 rr = *(const uint4 *)(res_base + row_off + lane_off);
                    v[0] += bf16lo_to_f32(rr.x);
                    v[1] += bf16hi_to_f32(rr.x);
                    v[2] += bf16lo_to_f32(rr.y);
                    v[3] += bf16hi_to_f32(rr.y);
                    v[4] += bf16lo_to_f32(rr.z);
                    v[5] += bf16hi_to_f32(rr.z);
                    v[6] += bf16lo_to_f32(rr.w);
                    v[7] += bf16hi_to_f32(rr.w);
                }
                if (has_vec && g.out_i8) {  // INT8 output: one byte per element, no penalty
                    uint32_t lo4 = 0, hi4 = 0;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        lo4 |= round_to_i8(v[r], g.out_inv_step) << (8 * r);
                        hi4 |= round_to_i8(v[4 + r], g.out_inv_step) << (8 * r);
                    }
                    *(uint2 *)((uint8_t *)g.out + (base_off + row_off + (int64_t)lane_off) / 2) = make_uint2(lo4, hi4);
                    continue;
                }
                const uint4 packed = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                                pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
                *(uint4 *)(out_base + row_off + lane_off) = packed;
                if (has_pen) {
                    const float t[8] = {bf16lo_to_f32(packed.x), bf16hi_to_f32(packed.x),
                                        bf16lo_to_f32(packed.y), bf16hi_to_f32(packed.y),
                                        bf16lo_to_f32(packed.z), bf16hi_to_f32(packed.z),
                                        bf16lo_to_f32(packed.w), bf16hi_to_f32(packed.w)};
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        if constexpr (PMODE == 4) {
                            // sum a^4 here, times (1/(tau+eps))^4 once per lane below
                            const float a2 = t[r] * t[r];
                            pen = __builtin_fmaf(a2, a2, pen);
                        } else {
                            const float u = __builtin_fabsf(t[r]) * g.inv_tau;
                            float w = u;
                            for (int e = 1; e < g.p; ++e)
                                w *= u;
                            pen += w;
                        }
                    }
                }
            }
        }
    }
    }
    if (has_pen) {  // uniform over the workgroup
        __shared__ float red[T::THREADS / kWave];
        if constexpr (PMODE == 4) {
            const float it2 = g.inv_tau * g.inv_tau;
            pen *= it2 * it2;
        }
        pen = wave_reduce_sum(pen);
        if (lane == 0)
            red[wave] = pen;
        __syncthreads();
        if (tid == 0) {
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < T::THREADS / kWave; ++w)
                s += red[w];
            g.partials[partial_index] = s;
        }
    }
}

struct NoBandHook {
    __device__ __forceinline__ void operator()(int) const {}
};

template <typename T, bool INT8, typename ACC, typename HOOK>
__device__ __forceinline__ void epilogue(const GemmDev &g, ACC (&acc)[T::MT][T::NT], uint8_t *smem,
                                         int tm, int tn, int wm, int wn, int lane, int wave, int tid,
                                         int partial_index, HOOK &band_hook)
{
    const bool interior = (tm + 1) * T::BM <= g.M && (tn + 1) * T::BN <= g.N;
    const bool res = g.residual != nullptr;
    const bool vec = INT8 && g.rs != nullptr;  // step vectors: the general form below applies them
#define TWEO_EPI(PM, RS, IN) \
    epilogue_impl<T, INT8, PM, RS, IN>(g, acc, smem, tm, tn, wm, wn, lane, wave, tid, partial_index, band_hook)
    if (vec)
        TWEO_EPI(-1, -1, false);
    else if (interior && g.p == 4 && !res)
        TWEO_EPI(4, 0, true);
    else if (interior && g.p == 4)
        TWEO_EPI(4, 1, true);
    else if (interior && g.p == 0 && !res)
        TWEO_EPI(0, 0, true);
    else
        TWEO_EPI(-1, -1, false);
#undef TWEO_EPI
}

// K split: the fp32 sums of one run, straight from the MFMA layout.  Lane (l31, lh) holds row l31
// and columns 8q + 4lh .. +3 of each 32x32 block (16-byte stores; the four q of a block complete
// the row's 128-byte line).
template <typename T, typename ACC>
__device__ __forceinline__ void store_ksplit_run(const GemmDev &g, ACC (&acc)[T::MT][T::NT], int split, int tm,
                                                 int tn, int wm, int wn, int l31, int lh)
{
    float *dst = g.ksplit_out + (int64_t)split * g.M * g.N;
#pragma unroll
    for (int i = 0; i < T::MT; ++i) {
        const int m = tm * T::BM + wm * T::TM + i * 32 + l31;
#pragma unroll
        for (int j = 0; j < T::NT; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = tn * T::BN + wn * T::TN + j * 32 + 8 * q + 4 * lh;
                if (m < g.M && n < g.N)
                    *(v4f *)(dst + (int64_t)m * g.N + n) =
                        v4f{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
            }
    }
}

template <typename T, bool INT8, bool A_E5M2 = false>
__global__ __launch_bounds__(T::THREADS) void gemm_nt_kernel(GemmDev g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int BM = T::BM, BN = T::BN;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int wm = wave / T::WN, wn = wave % T::WN;
    int tm, tn;
    // with a K split the grid is ksplit runs of the tile grid: run `split` takes K stages
    // [split * k_tiles / ksplit, (split + 1) * k_tiles / ksplit)
    const int n_tiles = g.tiles_m * g.tiles_n;
    const int split = g.ksplit > 1 ? (int)blockIdx.x / n_tiles : 0;
    tile_of_workgroup((int)blockIdx.x - split * n_tiles, g.tiles_m, g.tiles_n, tm, tn);

    // ---- global -> register -> LDS staging --------------------------------
    // chunk id = tid + i*THREADS : row = id/8, chunk-in-row = id%8 (same for all i)
    const int ld_row0 = tid >> 3, ld_ch = tid & 7;
    constexpr int ROW_STEP = T::THREADS / 8;
    const uint8_t *Abase = g.A + (int64_t)tm * BM * g.K + ld_ch * 16;
    const uint8_t *Bbase = g.B + (int64_t)tn * BN * g.K + ld_ch * 16;
    const int a_rows = g.M - tm * BM, b_rows = g.N - tn * BN;  // valid rows in this tile (>0)
    uint32_t a_off[T::A_LD], b_off[T::B_LD];
    int a_lds[T::A_LD], b_lds[T::B_LD];
#pragma unroll
    for (int i = 0; i < T::A_LD; ++i) {
        int row = ld_row0 + i * ROW_STEP;
        int grow = row < a_rows ? row : a_rows - 1;  // clamp: rows past M are never stored
        a_off[i] = (uint32_t)grow * (uint32_t)g.K;
        a_lds[i] = row * kBK + swz(row, ld_ch) * 16;
    }
#pragma unroll
    for (int i = 0; i < T::B_LD; ++i) {
        int row = ld_row0 + i * ROW_STEP;
        int grow = row < b_rows ? row : b_rows - 1;
        b_off[i] = (uint32_t)grow * (uint32_t)g.K;
        b_lds[i] = BM * kBK + row * kBK + swz(row, ld_ch) * 16;
    }
    v4i a_reg[T::A_LD], b_reg[T::B_LD];
    auto load_global = [&](int k0) {
        const bool k_ok = k0 + ld_ch * 16 < g.K;  // K % 16 == 0: a chunk is all in or all out
#pragma unroll
        for (int i = 0; i < T::A_LD; ++i)
            a_reg[i] = k_ok ? *(const v4i *)(Abase + a_off[i] + k0) : v4i{0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < T::B_LD; ++i)
            b_reg[i] = k_ok ? *(const v4i *)(Bbase + b_off[i] + k0) : v4i{0, 0, 0, 0};
    };
    auto store_lds = [&](int stage) {
        uint8_t *s = smem + stage * T::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < T::A_LD; ++i)
            *(v4i *)(s + a_lds[i]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < T::B_LD; ++i)
            *(v4i *)(s + b_lds[i]) = b_reg[i];
    };

    // ---- accumulators -------------------------------------------------------
    using acc_t = typename std::conditional<INT8, v16i, v16f>::type;
    acc_t acc[T::MT][T::NT];
#pragma unroll
    for (int i = 0; i < T::MT; ++i)
#pragma unroll
        for (int j = 0; j < T::NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[i][j][v] = 0;

    // fragment rows of this lane inside the stage
    const int l31 = lane & 31, lh = lane >> 5;
    const int a_row0 = wm * T::TM + l31;  // + mt*32
    const int b_row0 = wn * T::TN + l31;  // + nt*32

    auto compute_stage = [&](int stage) {
        const uint8_t *sA = smem + stage * T::STAGE_BYTES;
        const uint8_t *sB = sA + BM * kBK;
        if constexpr (!INT8) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {  // two K=64 slabs
                v8i fa[T::MT], fb[T::NT];
                const int c0 = kk * 4 + lh * 2;
#pragma unroll
                for (int i = 0; i < T::MT; ++i) {
                    int row = a_row0 + i * 32;
                    v4i x0 = *(const v4i *)(sA + row * kBK + swz(row, c0) * 16);
                    v4i x1 = *(const v4i *)(sA + row * kBK + swz(row, c0 + 1) * 16);
                    fa[i] = v8i{x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
                }
#pragma unroll
                for (int j = 0; j < T::NT; ++j) {
                    int row = b_row0 + j * 32;
                    v4i x0 = *(const v4i *)(sB + row * kBK + swz(row, c0) * 16);
                    v4i x1 = *(const v4i *)(sB + row * kBK + swz(row, c0 + 1) * 16);
                    fb[j] = v8i{x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
                }
#pragma unroll
                for (int i = 0; i < T::MT; ++i)
#pragma unroll
                    for (int j = 0; j < T::NT; ++j)
                        // first operand -> register-distributed index (n), second -> lane index (m)
                        // source formats: the first (B) always E4M3, the second (A) E4M3 or E5M2
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                            fb[j], fa[i], acc[i][j], 0, A_E5M2 ? 1 : 0, 0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {  // four K=32 slabs
                v4i fa[T::MT], fb[T::NT];
                const int c0 = kk * 2 + lh;
#pragma unroll
                for (int i = 0; i < T::MT; ++i) {
                    int row = a_row0 + i * 32;
                    fa[i] = *(const v4i *)(sA + row * kBK + swz(row, c0) * 16);
                }
#pragma unroll
                for (int j = 0; j < T::NT; ++j) {
                    int row = b_row0 + j * 32;
                    fb[j] = *(const v4i *)(sB + row * kBK + swz(row, c0) * 16);
                }
#pragma unroll
                for (int i = 0; i < T::MT; ++i)
#pragma unroll
                    for (int j = 0; j < T::NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[j], fa[i], acc[i][j],
                                                                          0, 0, 0);
            }
        }
    };

    // ---- main loop ----------------------------------------------------------
    const int k_tiles = (g.K + kBK - 1) / kBK;
    int kt_begin = 0, kt_end = k_tiles;
    if (g.ksplit > 1) {
        kt_begin = (int)((int64_t)split * k_tiles / g.ksplit);
        kt_end = (int)((int64_t)(split + 1) * k_tiles / g.ksplit);
    }
    load_global(kt_begin * kBK);
    store_lds(0);
    __syncthreads();
    for (int kt = kt_begin; kt < kt_end; ++kt) {
        const bool more = kt + 1 < kt_end;
        if (more)
            load_global((kt + 1) * kBK);
        compute_stage((kt - kt_begin) & 1);
        if (more)
            store_lds((kt - kt_begin + 1) & 1);
        __syncthreads();
    }

    if constexpr (!INT8) {
        if (g.ksplit > 1) {
            store_ksplit_run<T>(g, acc, split, tm, tn, wm, wn, l31, lh);
            return;
        }
    }
    // the loop ends with a barrier: every wave is done reading the stages
    NoBandHook no_hook;
    epilogue<T, INT8>(g, acc, smem, tm, tn, wm, wn, lane, wave, tid, blockIdx.x, no_hook);
}

// ---------------------------------------------------------------------------
// Pipelined kernel: global -> LDS by direct DMA loads (global_load_lds_dwordx4,
// no staging registers), NS stages of 64 bytes of K each, one workgroup barrier
// per stage, MFMA operand fragments double-buffered in registers so that the
// LDS reads of stage s+1 run under the MFMAs of stage s.  Needs K % 64 == 0.
//
// LDS layout of a stage: BM rows of A then BN rows of B, 64 bytes per row, the
// four 16-byte chunks of a row XOR-swizzled with (row/4)%4: 16 consecutive rows
// reading the same logical chunk then cover all 64 banks exactly once.  A DMA
// instruction of one wave writes 1024 contiguous LDS bytes (lane*16) = 16 rows;
// the swizzle is applied by choosing which global chunk each lane fetches.
template <int BM_, int BN_, int WM_, int WN_, int NS_, int WPE_ = 1>
struct TileD {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, NS = NS_;
    static constexpr int WPE = WPE_;  // waves per SIMD the register budget must allow
    static constexpr int NWAVES = WM * WN, THREADS = NWAVES * kWave;
    static constexpr int TM = BM / WM, TN = BN / WN;
    static constexpr int MT = TM / 32, NT = TN / 32;
    static constexpr int BK = 64;
    static constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK, STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = NS * STAGE_BYTES;
    static constexpr int A_DMA = BM / (16 * NWAVES), B_DMA = BN / (16 * NWAVES);  // per wave per stage
    static constexpr int LOADS = A_DMA + B_DMA;
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be made of 32x32 blocks");
    static_assert(BM % (16 * NWAVES) == 0 && BN % (16 * NWAVES) == 0, "DMA split");
    static_assert(NS >= 3 && LOADS * (NS - 2) < 64, "vmcnt range");
};


template <typename T, bool INT8>
__global__ __launch_bounds__(T::THREADS, T::WPE) void gemm_nt_dma_kernel(GemmDev g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = wave / T::WN, wn = wave % T::WN;
    int tm, tn;
    // with a K split the grid is ksplit runs of the tile grid: run `split` takes K stages
    // [split * stages / ksplit, (split + 1) * stages / ksplit)
    const int n_tiles = g.tiles_m * g.tiles_n;
    const int split = g.ksplit > 1 ? (int)blockIdx.x / n_tiles : 0;
    tile_of_workgroup((int)blockIdx.x - split * n_tiles, g.tiles_m, g.tiles_n, tm, tn);
    int kt = g.K / T::BK, kt_begin = 0;
    if (g.ksplit > 1) {
        kt_begin = (int)((int64_t)split * kt / g.ksplit);
        kt = (int)((int64_t)(split + 1) * kt / g.ksplit) - kt_begin;
    }

    // ---- DMA addressing -----------------------------------------------------
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const uint8_t *Ag = g.A + (int64_t)tm * T::BM * g.K + (int64_t)kt_begin * T::BK;
    const uint8_t *Bg = g.B + (int64_t)tn * T::BN * g.K + (int64_t)kt_begin * T::BK;
    const int a_rows = g.M - tm * T::BM, b_rows = g.N - tn * T::BN;
    uint32_t a_voff[T::A_DMA], b_voff[T::B_DMA];
#pragma unroll
    for (int i = 0; i < T::A_DMA; ++i) {
        int row = (i * T::NWAVES + wave) * 16 + (lane >> 2);
        int c = (lane & 3) ^ ((row >> 2) & 3);
        int grow = row < a_rows ? row : a_rows - 1;  // rows past M are loaded twice, never stored
        a_voff[i] = (uint32_t)grow * (uint32_t)g.K + c * 16;
    }
#pragma unroll
    for (int i = 0; i < T::B_DMA; ++i) {
        int row = (i * T::NWAVES + wave) * 16 + (lane >> 2);
        int c = (lane & 3) ^ ((row >> 2) & 3);
        int grow = row < b_rows ? row : b_rows - 1;
        b_voff[i] = (uint32_t)grow * (uint32_t)g.K + c * 16;
    }
    auto issue_stage = [&](int s) {
        const uint32_t dst = lds_base + (s % T::NS) * T::STAGE_BYTES + wave * 1024;
        const uint8_t *ap = Ag + (int64_t)s * T::BK, *bp = Bg + (int64_t)s * T::BK;
#pragma unroll
        for (int i = 0; i < T::A_DMA; ++i)
            dma_load16(dst + i * T::NWAVES * 1024, ap, a_voff[i]);
#pragma unroll
        for (int i = 0; i < T::B_DMA; ++i)
            dma_load16(dst + T::A_BYTES + i * T::NWAVES * 1024, bp, b_voff[i]);
    };

    // ---- fragments ------------------------------------------------------------
    const int l31 = lane & 31, lh = lane >> 5;
    const int sw = (l31 >> 2) & 3;
    // logical chunks of this lane: FP8 takes 32 contiguous bytes (chunks 2h, 2h+1) for one
    // K=64 MFMA; INT8 takes chunk h for the first K=32 MFMA and chunk 2+h for the second.
    const int c0 = INT8 ? lh : 2 * lh, c1 = INT8 ? 2 + lh : 2 * lh + 1;
    const int a_frag0 = (wm * T::TM + l31) * T::BK, b_frag0 = T::A_BYTES + (wn * T::TN + l31) * T::BK;
    const int off0 = (c0 ^ sw) * 16, off1 = (c1 ^ sw) * 16;
    struct Frag {
        v4i a0[T::MT], a1[T::MT], b0[T::NT], b1[T::NT];
    };
    auto load_frags = [&](Frag &f, int s) {
        const uint8_t *st = smem + (s % T::NS) * T::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < T::MT; ++i) {
            f.a0[i] = *(const v4i *)(st + a_frag0 + i * 32 * T::BK + off0);
            f.a1[i] = *(const v4i *)(st + a_frag0 + i * 32 * T::BK + off1);
        }
#pragma unroll
        for (int j = 0; j < T::NT; ++j) {
            f.b0[j] = *(const v4i *)(st + b_frag0 + j * 32 * T::BK + off0);
            f.b1[j] = *(const v4i *)(st + b_frag0 + j * 32 * T::BK + off1);
        }
    };
    using acc_t = typename std::conditional<INT8, v16i, v16f>::type;
    acc_t acc[T::MT][T::NT];
#pragma unroll
    for (int i = 0; i < T::MT; ++i)
#pragma unroll
        for (int j = 0; j < T::NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[i][j][v] = 0;
    auto mfma_stage = [&](const Frag &f) {
#pragma unroll
        for (int i = 0; i < T::MT; ++i)
#pragma unroll
            for (int j = 0; j < T::NT; ++j) {
                if constexpr (INT8) {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.b0[j], f.a0[i], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.b1[j], f.a1[i], acc[i][j], 0, 0, 0);
                } else {
                    v8i fa = {f.a0[i][0], f.a0[i][1], f.a0[i][2], f.a0[i][3],
                              f.a1[i][0], f.a1[i][1], f.a1[i][2], f.a1[i][3]};
                    v8i fb = {f.b0[j][0], f.b0[j][1], f.b0[j][2], f.b0[j][3],
                              f.b1[j][0], f.b1[j][1], f.b1[j][2], f.b1[j][3]};
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb, fa, acc[i][j], 0, 0,
                                                                                0, 0, 0, 0);
                }
            }
    };

    // ---- pipeline ---------------------------------------------------------------
    // Invariant at the top of iteration s: stages <= s+NS-2 have been issued.
#pragma unroll
    for (int s = 0; s < T::NS - 1; ++s)
        if (s < kt)
            issue_stage(s);
    if (kt >= T::NS - 1)
        wait_vmcnt<T::LOADS *(T::NS - 2)>();
    else
        wait_vmcnt<0>();
    block_barrier();
    Frag fr[2];
    load_frags(fr[0], 0);
    // Steady state: stage ss with ss + NS - 1 < kt.  Two stages per trip so that the two
    // fragment buffers have fixed names; the body is one basic block (no conditions), which
    // lets the scheduler run the LDS reads of stage ss+1 under the MFMAs of stage ss.
    auto steady_step = [&](int ss, const Frag &cur, Frag &nxt) {
        // stage ss+1 must have landed (for every wave) before its fragments are read; the
        // barrier also frees the buffer of stage ss-1 for the DMA issued right after it
        wait_vmcnt<T::LOADS *(T::NS - 3)>();
        block_barrier();
        issue_stage(ss + T::NS - 1);
        load_frags(nxt, ss + 1);
        mfma_stage(cur);
        // ask the scheduler for: MFMA, a few LDS reads, MFMA, ... so the reads of the next
        // stage are in flight while this stage's MFMAs occupy the matrix pipe
        constexpr int N_MFMA = T::MT * T::NT * (INT8 ? 2 : 1), N_DS = 2 * (T::MT + T::NT);
        constexpr int DS_PER = (N_DS + N_MFMA - 2) / (N_MFMA - 1);
#pragma unroll
        for (int k = 0; k < N_MFMA; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);       // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, DS_PER, 0);  // DS reads
        }
    };
    auto tail_step = [&](int ss, const Frag &cur, Frag &nxt) {
        if (ss + 1 < kt) {
            wait_vmcnt<0>();
            block_barrier();
            if (ss + T::NS - 1 < kt)
                issue_stage(ss + T::NS - 1);
            load_frags(nxt, ss + 1);
        }
        mfma_stage(cur);
    };
    int s = 0;
    const int steady_end = kt - (T::NS - 1);
    for (; s + 1 < steady_end; s += 2) {
        steady_step(s, fr[0], fr[1]);
        steady_step(s + 1, fr[1], fr[0]);
    }
    for (; s < kt; s += 2) {
        tail_step(s, fr[0], fr[1]);
        if (s + 1 < kt)
            tail_step(s + 1, fr[1], fr[0]);
    }
    if constexpr (!INT8) {
        if (g.ksplit > 1) {
            store_ksplit_run<T>(g, acc, split, tm, tn, wm, wn, l31, lh);
            return;
        }
    }
    block_barrier();  // every wave is done reading the stages before they are reused
    NoBandHook no_hook;
    epilogue<T, INT8>(g, acc, smem, tm, tn, wm, wn, lane, wave, tid, blockIdx.x, no_hook);
}

// ---------------------------------------------------------------------------
// Persistent streaming kernel (K % 128 == 0): the large-shape workhorse.
//
// What measurement on gfx950 dictated:
//  * the L2 -> CU path moves ~23 TB/s (whole chip) when every wave-level load
//    covers whole 128-byte lines, but only ~15 TB/s in 64-byte pieces, and a
//    256x256 tile at MFMA peak needs 19.5 TB/s.  So a stage is 128 bytes of K
//    per row (one full line per row per DMA instruction: 8 rows x 128 B);
//  * 64 KB in flight per CU is enough to reach that rate, so two stages of
//    (BM+BN) x 128 B are used for the 256x256 tile (128 KB of the 160 KB LDS);
//  * with one workgroup per CU, prologue, epilogue and the burst of output
//    writes of a tile are exposed.  Workgroups are therefore persistent: before
//    the epilogue of tile t the DMA loads of the first stage(s) of tile t+1 are
//    already issued, and the stores of tile t drain under the MFMAs of t+1.
//
// A stage holds two K=64 MFMA slabs.  Fragments are double-buffered in
// registers across the stage barrier: the last slab of stage s-1 is multiplied
// after the barrier of stage s, under the LDS reads of the first slab of s.
// LDS rows are 128 bytes; the eight 16-byte chunks of a row are XOR-swizzled
// with (row/2)%8, which makes the 16-byte fragment reads of 16 consecutive rows
// cover all 64 banks once and does not depend on the 32-row block index.
template <int BM_, int BN_, int WM_, int WN_, int NS_, int WPE_>
struct TileS {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, NS = NS_, WPE = WPE_;
    static constexpr int NWAVES = WM * WN, THREADS = NWAVES * kWave;
    static constexpr int TM = BM / WM, TN = BN / WN;
    static constexpr int MT = TM / 32, NT = TN / 32;
    static constexpr int BK = 128;
    static constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK, STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int A_DMA = BM / (8 * NWAVES), B_DMA = BN / (8 * NWAVES);  // per wave per stage
    static constexpr int LOADS = A_DMA + B_DMA;
    static constexpr int EPI_FP32 = 32 * (TN * 4 + 16), EPI_BF16 = 2 * 32 * (TN * 2 + 16);
    static constexpr int EPI_BYTES = NWAVES * (EPI_FP32 > EPI_BF16 ? EPI_FP32 : EPI_BF16);
    // stages 0..NS-2 of the next tile are prefetched under the epilogue, which stages its
    // output in the LDS behind them
    static constexpr int EPI_OFFSET = (NS - 1) * STAGE_BYTES;
    static constexpr int LDS_BYTES =
        NS * STAGE_BYTES > EPI_OFFSET + EPI_BYTES ? NS * STAGE_BYTES : EPI_OFFSET + EPI_BYTES;
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be made of 32x32 blocks");
    static_assert(BM % (8 * NWAVES) == 0 && BN % (8 * NWAVES) == 0, "DMA split");
    static_assert(NS >= 2 && LOADS * (NS - 1) < 64, "vmcnt range");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS capacity");
};


//
// SK ("stream-K"): when the tile count is not a multiple of the workgroup count, the last,
// partial round would leave CUs idle (176 or 192 tiles of a weight gradient on 256 CUs: a
// quarter to a third of the machine).  With SK the whole rounds are handed out as before and
// the K loops of the remaining tiles are cut into one contiguous range of stages per workgroup
// (cut points snapped away from tile ends).  A workgroup that multiplied only part of a tile's
// K range writes its fp32 (int32) accumulators to a slot of the workspace and counts itself in
// on the tile's counter; whoever arrives last adds all slots of the tile in K order - a fixed
// order, whoever that is - and runs the ordinary epilogue.  Nobody waits for anybody.
// Measured on MI355X this is slower than leaving the CUs idle (every tile of the split round is
// finished by a fixup at the very end of the kernel: a burst of device-scope slot traffic with
// nothing left to hide it under; 192x256 tiles fix the common tile counts instead), so it is
// off unless tweo_set_stream_k(1) asks for it; the parity tests keep it honest.
template <typename T, bool INT8, bool SK>
__global__ __launch_bounds__(T::THREADS, T::WPE) void gemm_nt_stream_kernel(GemmDev g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = wave / T::WN, wn = wave % T::WN;
    const int total = g.tiles_m * g.tiles_n;
    // Persistent schedule: round r hands tile ids [r*G, (r+1)*G) to the G workgroups; inside a
    // round each XCD (workgroup index mod 8) gets a contiguous run of ids, i.e. neighbouring
    // tiles, so that the 32 CUs behind one L2 share A and B panels.
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, per_xcd = G >> 3, rem_xcd = G & 7;
    const int slot = xcd * per_xcd + (xcd < rem_xcd ? xcd : rem_xcd) + (blockIdx.x >> 3);

    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const int dma_row = lane >> 3, dma_p = lane & 7;
    const uint8_t *Ag, *Bg;
    uint32_t a_voff[T::A_DMA], b_voff[T::B_DMA];
    auto set_tile = [&](int tm, int tn) {
        Ag = g.A + (int64_t)tm * T::BM * g.K;
        Bg = g.B + (int64_t)tn * T::BN * g.K;
        const int a_rows = g.M - tm * T::BM, b_rows = g.N - tn * T::BN;
#pragma unroll
        for (int i = 0; i < T::A_DMA; ++i) {
            const int row = (i * T::NWAVES + wave) * 8 + dma_row;
            const int c = dma_p ^ ((row >> 1) & 7);
            const int grow = row < a_rows ? row : a_rows - 1;  // rows past M: loaded twice, never stored
            a_voff[i] = (uint32_t)grow * (uint32_t)g.K + c * 16;
        }
#pragma unroll
        for (int i = 0; i < T::B_DMA; ++i) {
            const int row = (i * T::NWAVES + wave) * 8 + dma_row;
            const int c = dma_p ^ ((row >> 1) & 7);
            const int grow = row < b_rows ? row : b_rows - 1;
            b_voff[i] = (uint32_t)grow * (uint32_t)g.K + c * 16;
        }
    };
    auto issue_stage = [&](int s) {
        const uint32_t dst = lds_base + (s % T::NS) * T::STAGE_BYTES + wave * 1024;
        const uint8_t *ap = Ag + (int64_t)s * T::BK, *bp = Bg + (int64_t)s * T::BK;
#pragma unroll
        for (int i = 0; i < T::A_DMA; ++i)
            dma_load16(dst + i * T::NWAVES * 1024, ap, a_voff[i]);
#pragma unroll
        for (int i = 0; i < T::B_DMA; ++i)
            dma_load16(dst + T::A_BYTES + i * T::NWAVES * 1024, bp, b_voff[i]);
    };

    // fragment addressing: lane (l31, lh) reads row l31 of each 32-row block; logical chunks of
    // slab kk: FP8 4kk+2lh, 4kk+2lh+1 (32 contiguous bytes for one K=64 MFMA);
    // INT8 4kk+lh and 4kk+2+lh (one chunk for each of the two K=32 MFMAs)
    const int l31 = lane & 31, lh = lane >> 5;
    const int sw = (l31 >> 1) & 7;
    int frag_off[2][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int c0 = INT8 ? 4 * kk + lh : 4 * kk + 2 * lh;
        const int c1 = INT8 ? 4 * kk + 2 + lh : 4 * kk + 2 * lh + 1;
        frag_off[kk][0] = (c0 ^ sw) * 16;
        frag_off[kk][1] = (c1 ^ sw) * 16;
    }
    const int a_frag0 = (wm * T::TM + l31) * T::BK, b_frag0 = T::A_BYTES + (wn * T::TN + l31) * T::BK;
    struct Frag {
        v4i a0[T::MT], a1[T::MT], b0[T::NT], b1[T::NT];
    };
    auto load_frags = [&](Frag &f, int s, int kk) {
        const uint8_t *st = smem + (s % T::NS) * T::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < T::MT; ++i) {
            f.a0[i] = *(const v4i *)(st + a_frag0 + i * 32 * T::BK + frag_off[kk][0]);
            f.a1[i] = *(const v4i *)(st + a_frag0 + i * 32 * T::BK + frag_off[kk][1]);
        }
#pragma unroll
        for (int j = 0; j < T::NT; ++j) {
            f.b0[j] = *(const v4i *)(st + b_frag0 + j * 32 * T::BK + frag_off[kk][0]);
            f.b1[j] = *(const v4i *)(st + b_frag0 + j * 32 * T::BK + frag_off[kk][1]);
        }
    };
    using acc_t = typename std::conditional<INT8, v16i, v16f>::type;
    acc_t acc[T::MT][T::NT];
    auto mfma_slab = [&](const Frag &f) {
#pragma unroll
        for (int i = 0; i < T::MT; ++i)
#pragma unroll
            for (int j = 0; j < T::NT; ++j) {
                if constexpr (INT8) {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.b0[j], f.a0[i], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.b1[j], f.a1[i], acc[i][j], 0, 0, 0);
                } else {
                    v8i fa = {f.a0[i][0], f.a0[i][1], f.a0[i][2], f.a0[i][3],
                              f.a1[i][0], f.a1[i][1], f.a1[i][2], f.a1[i][3]};
                    v8i fb = {f.b0[j][0], f.b0[j][1], f.b0[j][2], f.b0[j][3],
                              f.b1[j][0], f.b1[j][1], f.b1[j][2], f.b1[j][3]};
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb, fa, acc[i][j], 0, 0,
                                                                                0, 0, 0, 0);
                }
            }
    };

    // Steady-state slab: MFMA unit k (one 32x32 block), then one piece of the next slab's
    // fragments, then one piece of the DMA of a later stage, with a scheduling fence after each
    // unit.  Spreading the DMA instructions over the MFMAs keeps a wave from sitting in the
    // vector-memory issue queue (a 64 KB stage is 64 KB/clk-limited address work) while the
    // matrix pipe runs dry.
    auto issue_piece = [&](int s, int idx) {
        const uint32_t dst = lds_base + (s % T::NS) * T::STAGE_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < T::A_DMA; ++i)
            if (idx == i)
                dma_load16(dst + i * T::NWAVES * 1024, Ag + (int64_t)s * T::BK, a_voff[i]);
#pragma unroll
        for (int i = 0; i < T::B_DMA; ++i)
            if (idx == T::A_DMA + i)
                dma_load16(dst + T::A_BYTES + i * T::NWAVES * 1024, Bg + (int64_t)s * T::BK, b_voff[i]);
    };
    auto slab_step = [&](const Frag &cur, Frag &nxt, int s_ld, int kk_ld, int dma_stage) {
        constexpr int UNITS = T::MT * T::NT;
        constexpr int DMA_PER = (T::LOADS + UNITS - 1) / UNITS;
        const uint8_t *st = smem + (s_ld % T::NS) * T::STAGE_BYTES;
#pragma unroll
        for (int k = 0; k < UNITS; ++k) {
            const int i = k / T::NT, j = k % T::NT;
            if constexpr (INT8) {
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur.b0[j], cur.a0[i], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur.b1[j], cur.a1[i], acc[i][j], 0, 0, 0);
            } else {
                v8i fa = {cur.a0[i][0], cur.a0[i][1], cur.a0[i][2], cur.a0[i][3],
                          cur.a1[i][0], cur.a1[i][1], cur.a1[i][2], cur.a1[i][3]};
                v8i fb = {cur.b0[j][0], cur.b0[j][1], cur.b0[j][2], cur.b0[j][3],
                          cur.b1[j][0], cur.b1[j][1], cur.b1[j][2], cur.b1[j][3]};
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb, fa, acc[i][j], 0, 0, 0, 0,
                                                                            0, 0);
            }
            if (k < T::MT) {
                nxt.a0[k] = *(const v4i *)(st + a_frag0 + k * 32 * T::BK + frag_off[kk_ld][0]);
                nxt.a1[k] = *(const v4i *)(st + a_frag0 + k * 32 * T::BK + frag_off[kk_ld][1]);
            } else if (k < T::MT + T::NT) {
                nxt.b0[k - T::MT] = *(const v4i *)(st + b_frag0 + (k - T::MT) * 32 * T::BK + frag_off[kk_ld][0]);
                nxt.b1[k - T::MT] = *(const v4i *)(st + b_frag0 + (k - T::MT) * 32 * T::BK + frag_off[kk_ld][1]);
            }
            if (dma_stage >= 0) {
#pragma unroll
                for (int d = 0; d < DMA_PER; ++d)
                    if (k * DMA_PER + d < T::LOADS)
                        issue_piece(dma_stage, k * DMA_PER + d);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        static_assert(T::MT + T::NT <= UNITS, "fragment pieces fit in the MFMA units of a slab");
    };

    const int kt_full = g.K / T::BK;
    Frag fr[2];

    // ---- work units of this workgroup: whole tiles, then (SK) the segments of its stage range
    struct Unit {
        int tm, tn, s0, kt, id, seg;  // kt: stages in the unit; id: tile id; seg: ordinal in the range
    };
    const int sk_rounds = SK ? g.sk_full_rounds : 0;
    const int sk_first = sk_rounds * G;               // first tile id of the remainder
    const int sk_tiles = SK ? total - sk_first : 0;   // < G
    // start of workgroup w's range in the remainder's stage space [0, sk_tiles * kt_full)
    auto sk_bound = [&](int w) -> int64_t {
        constexpr int SNAP = 4;
        int64_t x = (int64_t)w * sk_tiles * kt_full / G;
        const int o = (int)(x % kt_full);
        if (o < SNAP)
            x -= o;
        else if (o > kt_full - SNAP)
            x += kt_full - o;
        return x;
    };
    int64_t sk_x0 = 0, sk_x1 = 0;
    if constexpr (SK) {
        sk_x0 = sk_bound(slot);
        sk_x1 = sk_bound(slot + 1);
    }
    auto get_unit = [&](int u, Unit &U) -> bool {
        if (!SK || u < sk_rounds) {
            const int id = slot + u * G;
            if (id >= (SK ? sk_first : total))
                return false;
            tile_from_id(id, g.tiles_m, g.tiles_n, U.tm, U.tn);
            U.s0 = 0;
            U.kt = kt_full;
            U.id = id;
            U.seg = 0;
            return true;
        }
        int64_t pos = sk_x0;
        for (int c = 0;; ++c) {
            if (pos >= sk_x1)
                return false;
            const int rt = (int)(pos / kt_full), s0 = (int)(pos % kt_full);
            const int64_t left = sk_x1 - pos;
            const int len = left < kt_full - s0 ? (int)left : kt_full - s0;
            if (c == u - sk_rounds) {
                U.id = sk_first + rt;
                tile_from_id(U.id, g.tiles_m, g.tiles_n, U.tm, U.tn);
                U.s0 = s0;
                U.kt = len;
                U.seg = c;
                return true;
            }
            pos += len;
        }
    };
    auto set_unit = [&](const Unit &U) {
        set_tile(U.tm, U.tn);
        Ag += (int64_t)U.s0 * T::BK;
        Bg += (int64_t)U.s0 * T::BK;
    };

    Unit cur, nxt;
    int u = 0;
    bool have = get_unit(0, cur);
    if (have) {
        set_unit(cur);
#pragma unroll
        for (int s = 0; s < T::NS - 1; ++s)
            if (s < cur.kt)
                issue_stage(s);
    }
    while (have) {
#pragma unroll
        for (int i = 0; i < T::MT; ++i)
#pragma unroll
            for (int j = 0; j < T::NT; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    acc[i][j][v] = 0;

        // the next unit: scalar divisions, done here so that they are off the critical path at
        // the unit boundary
        const bool have_next = get_unit(u + 1, nxt);
        const int kt = cur.kt;

        // ---- stage 0: nothing to multiply yet.  vmcnt(0) also covers the previous tile's stores.
        wait_vmcnt<0>();
        block_barrier();
        if (T::NS - 1 < kt)
            issue_stage(T::NS - 1);
        load_frags(fr[0], 0, 0);
        load_frags(fr[1], 0, 1);
        mfma_slab(fr[0]);
        // ---- steady stages: s + NS - 1 < kt
        int s = 1;
        for (; s + T::NS - 1 < kt; ++s) {
            // stage s has landed for every wave; the barrier also frees the buffer of stage s-1
            wait_vmcnt<T::LOADS *(T::NS - 2)>();
            block_barrier();
            slab_step(fr[1], fr[0], s, 0, s + T::NS - 1);
            slab_step(fr[0], fr[1], s, 1, -1);
        }
        // ---- tail stages: nothing left to issue
        for (; s < kt; ++s) {
            wait_vmcnt<0>();
            block_barrier();
            load_frags(fr[0], s, 0);
            mfma_slab(fr[1]);
            load_frags(fr[1], s, 1);
            mfma_slab(fr[0]);
        }
        mfma_slab(fr[1]);

        // ---- unit boundary: every wave is done reading the stages; start the next unit's loads,
        //      then write this tile out (its stores drain under the next unit's MFMAs)
        block_barrier();
        if (have_next)
            set_unit(nxt);
        // the next unit's first stage(s) are issued piecewise, one share per epilogue band, so
        // that no wave queues up behind 64 KB of address work before it can start its epilogue
        auto prefetch_hook = [&](int band) {
            if (have_next) {
                constexpr int PER_BAND = (T::LOADS + T::MT - 1) / T::MT;
#pragma unroll
                for (int s2 = 0; s2 < T::NS - 1; ++s2)
                    if (s2 < nxt.kt) {
#pragma unroll
                        for (int d = 0; d < PER_BAND; ++d)
                            if (band * PER_BAND + d < T::LOADS)
                                issue_piece(s2, band * PER_BAND + d);
                    }
            }
        };
        bool whole = true;
        if constexpr (SK)
            whole = cur.s0 == 0 && cur.kt == kt_full;
        if (whole) {
            epilogue<T, INT8>(g, acc, smem + T::EPI_OFFSET, cur.tm, cur.tn, wm, wn, lane, wave, tid, cur.id,
                              prefetch_hook);
        } else {
            __shared__ int sk_arrival;
            using word_t = typename std::conditional<INT8, int, float>::type;
            constexpr int SLOT_WORDS = T::BM * T::BN;
#pragma unroll
            for (int b = 0; b < T::MT; ++b)
                prefetch_hook(b);
            // This workgroup's slot: 2 per workgroup (first / later segment of its range); pairs
            // of accumulator words, layout [wave][block][pair][lane], every store 512 B contiguous.
            // The slots are written and read with device-scope (cache-bypassing) accesses: the
            // workgroups of a tile may sit behind different L2s, and a fence that writes back and
            // invalidates a whole L2 would throw away the operand panels its 32 CUs share.
            typedef uint32_t u4 __attribute__((ext_vector_type(4)));
            constexpr int kDeviceScope = 16;  // cache policy bit sc1: performed at device scope
            constexpr uint32_t SLOT_BYTES = (uint32_t)SLOT_WORDS * 4;
            auto slot_rsrc = [&](int w, int later) {
                return __builtin_amdgcn_make_buffer_rsrc(
                    (uint8_t *)g.sk_partials + (size_t)(2 * w + later) * SLOT_BYTES, 0, (int)SLOT_BYTES, 0x00020000);
            };
            const uint32_t lane_off = ((uint32_t)wave * T::MT * T::NT * 4 * kWave + lane) * 16u;
            {
                const auto mine = slot_rsrc(slot, cur.seg > 0 ? 1 : 0);
#pragma unroll
                for (int i = 0; i < T::MT; ++i)
#pragma unroll
                    for (int j = 0; j < T::NT; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const u4 v = {__builtin_bit_cast(uint32_t, (word_t)acc[i][j][4 * q]),
                                          __builtin_bit_cast(uint32_t, (word_t)acc[i][j][4 * q + 1]),
                                          __builtin_bit_cast(uint32_t, (word_t)acc[i][j][4 * q + 2]),
                                          __builtin_bit_cast(uint32_t, (word_t)acc[i][j][4 * q + 3])};
                            __builtin_amdgcn_raw_buffer_store_b128(v, mine, lane_off + ((i * T::NT + j) * 4 + q) * kWave * 16,
                                                                   0, kDeviceScope);
                        }
            }
            // pieces of this tile, in K order: the workgroups whose ranges meet its stage interval
            const int rt = cur.id - sk_first;
            const int64_t lo = (int64_t)rt * kt_full, hi = lo + kt_full;
            int w_a = (int)(lo * G / ((int64_t)sk_tiles * kt_full));
            if (w_a > G - 1)
                w_a = G - 1;
            while (w_a > 0 && sk_bound(w_a) > lo)
                --w_a;
            while (w_a + 1 < G && sk_bound(w_a + 1) <= lo)
                ++w_a;
            int pieces = 0;
            for (int w = w_a; w < G && sk_bound(w) < hi; ++w)
                if (sk_bound(w + 1) > sk_bound(w))
                    ++pieces;
            // every store of the slot has been acknowledged before the arrival is counted
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            wait_vmcnt<0>();
            __syncthreads();
            if (tid == 0)
                sk_arrival = (int)__hip_atomic_fetch_add(g.sk_counters + rt, 1u, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            const bool last = sk_arrival == pieces - 1;
            if (last) {
#pragma unroll
                for (int i = 0; i < T::MT; ++i)
#pragma unroll
                    for (int j = 0; j < T::NT; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            acc[i][j][v] = 0;
                for (int w = w_a; w < G && sk_bound(w) < hi; ++w) {
                    if (sk_bound(w + 1) <= sk_bound(w))
                        continue;
                    const auto src = slot_rsrc(w, sk_bound(w) >= lo ? 0 : 1);
#pragma unroll
                    for (int i = 0; i < T::MT; ++i) {
                        u4 v[T::NT][4];  // a band's worth of loads in flight
#pragma unroll
                        for (int j = 0; j < T::NT; ++j)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                v[j][q] = __builtin_amdgcn_raw_buffer_load_b128(
                                    src, lane_off + ((i * T::NT + j) * 4 + q) * kWave * 16, 0, kDeviceScope);
#pragma unroll
                        for (int j = 0; j < T::NT; ++j)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
#pragma unroll
                                for (int r = 0; r < 4; ++r)
                                    acc[i][j][4 * q + r] += __builtin_bit_cast(word_t, v[j][q][r]);
                    }
                }
                NoBandHook no_hook;
                epilogue<T, INT8>(g, acc, smem + T::EPI_OFFSET, cur.tm, cur.tn, wm, wn, lane, wave, tid, cur.id,
                                  no_hook);
            }
        }
        cur = nxt;
        have = have_next;
        ++u;
    }
}

// ---------------------------------------------------------------------------
// W8A8 linear for small M (decode-time batches, M <= 128): the product is bound by streaming the
// N x K weight bytes from HBM once.  One workgroup per CU owns up to NB blocks of 16 weight rows
// (block ids b, b + grid, ...); its 8 waves split K; products come from v_mfma_i32_16x16x64_i8
// (operand row = lane % 16, 16 bytes at k = 16 * (lane / 16)); the partial int32 tiles of the
// waves are added through LDS - exact, so the result is the same bits as any other summation
// order.  y = bf16(fp32(acc) * alpha) (Sec. 4.4), or with VEC y = bf16((fp32(acc) * rs[m]) * cs[n]):
// dequantisation steps per token and per output channel.
struct StepVectors {
    const float *rs, *cs;
    int rs_stride, cs_stride;
    int out_i8;  // Y holds int8 = clamp(rne(y * out_inv_step), +-127) instead of bf16
    float out_inv_step;
};

// How the operands get to the MFMAs decides everything here.  Measured on MI355X: a load in the
// MFMA operand layout (a 16-lane group touches 16 different rows, 16 bytes of each) moves 16 bytes
// per clock and CU through the texture unit, about 25 GB/s per CU, and with every workgroup
// reading all of X from the L2 the time of such kernels was (weights + CUs x X) / 6.5 TB/s for every
// shape and M (11008 -> 4096 at M = 64: 32 us).  A direct-to-LDS load in which 16 neighbouring
// lanes read 256 contiguous bytes moves 64 bytes per clock.  So both operands are staged through a
// ring of LDS stages and
// every byte, weights included, arrives by such loads: a stage is KCH = 64 * KSTEPS bytes of K for
// the M rows of X and the workgroup's 16 * NB weight rows, S stages form a ring, S - 1 of them are
// in flight while one is multiplied, one barrier per stage.  The 16-byte chunks of a row are
// stored XOR-swizzled with the row's index in its block of 16 (the loading lane picks the global
// chunk accordingly), so that the fragment reads of 16 rows at one k are conflict free.  Wave w
// multiplies k step w % KSTEPS of every stage, for the M blocks of part w / KSTEPS; the partial
// tiles meet in LDS at the end.  Stages past the end of K re-load the last one into slots nobody
// reads any more, so that the count of loads in flight stays what the waits assume.
template <int MB, int NB, int KSTEPS, int S, bool VEC>
__global__ __launch_bounds__(512) void w8a8_skinny_ring_kernel(const int8_t *__restrict__ X,
                                                               const int8_t *__restrict__ W, int M, int N, int K,
                                                               float alpha, StepVectors sv, uint16_t *__restrict__ Y)
{
    constexpr int WAVES = 8, STEP = 64, KCH = KSTEPS * STEP, PARTS = WAVES / KSTEPS, MBW = MB / PARTS;
    constexpr int ROWS_X = MB * 16, ROWS = ROWS_X + NB * 16, STAGE = ROWS * KCH;
    constexpr int RPI = 1024 / KCH, NI = ROWS / RPI, PPW = (NI + WAVES - 1) / WAVES, CPR = KCH / 16;
    // the waves' partial tiles meet in the ring's memory, RB blocks of weight rows at a time
    constexpr int RB_FIT = (S * STAGE) / (WAVES * MBW * 1024), RB = RB_FIT < NB ? RB_FIT : NB, T = RB * MBW;
    static_assert(MB % PARTS == 0 && 1024 % KCH == 0 && ROWS % RPI == 0, "shapes divide");
    static_assert(S * STAGE <= 160 * 1024 && RB >= 1, "LDS capacity");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int r16 = lane & 15, kc = lane >> 4;
    const int step = wave % KSTEPS, part = wave / KSTEPS;
    const int steps = K / STEP, blocks = (N + 15) / 16, grid = gridDim.x;
    const int chunks = (K + KCH - 1) / KCH;
    const bool ragged = K % KCH != 0;
    // workgroups walk the chunks in rotated orders (they all read the same X)
    const int rot = (int)((blockIdx.x >> 3) % (unsigned)chunks);
    auto chunk_at = [&](int t) {
        const int c = t < chunks ? t : chunks - 1;
        const int r = c + rot;
        return r < chunks ? r : r - chunks;
    };
    // fragment reads: row r16 of a block, chunk 4 * step + kc of the stage, swizzled
    const uint32_t frag_col = (uint32_t)(((step * 4 + kc) ^ r16) * 16);
    for (int first = blockIdx.x; first < blocks; first += NB * grid) {
        // this wave's DMA instructions of a stage: instruction i covers the stage's rows i * RPI ..,
        // lane l the LDS slot (row l / CPR, chunk l % CPR), which holds the global chunk slot ^ row
        const uint8_t *src[PPW];
        uint32_t voff[PPW], voff_last[PPW], dst[PPW];
#pragma unroll
        for (int j = 0; j < PPW; ++j) {
            int i = j * WAVES + wave;
            i = i < NI ? i : NI - 1;
            const int rr = i * RPI + lane / CPR, R = rr & 15, c = (lane % CPR) ^ R;
            uint32_t rowoff;
            if (i * RPI < ROWS_X) {  // uniform: an instruction lies in X or in one weight block
                const int m = rr < M ? rr : M - 1;
                src[j] = (const uint8_t *)X;
                rowoff = (uint32_t)m * (uint32_t)K;
            } else {
                const int a = (i * RPI - ROWS_X) / 16;
                int blk = first + a * grid;
                blk = blk < blocks ? blk : blocks - 1;  // block slots past the end: duplicates, never stored
                const int n = blk * 16 + R < N ? R : N - 1 - blk * 16;
                src[j] = (const uint8_t *)W + (int64_t)blk * 16 * K;
                rowoff = (uint32_t)n * (uint32_t)K;
            }
            voff[j] = rowoff + (uint32_t)c * 16u;
            // the last chunk of a K that ends inside it: chunks past K read the row's first bytes
            // (they only ever meet zeroed X fragments); this offset is absolute in K
            const int k_last = (chunks - 1) * KCH + c * 16;
            voff_last[j] = rowoff + (uint32_t)(k_last + 16 <= K ? k_last : c * 16 % STEP);
            dst[j] = (uint32_t)i * 1024u;
        }
        auto dma_stage = [&](int cc, int slot) {
            const bool last = ragged && cc == chunks - 1;
#pragma unroll
            for (int j = 0; j < PPW; ++j)
                dma_load16(lds_base + slot * STAGE + dst[j], last ? src[j] : src[j] + (int64_t)cc * KCH,
                           last ? voff_last[j] : voff[j]);
        };
        v4i acc[NB][MBW];
#pragma unroll
        for (int a = 0; a < NB; ++a)
#pragma unroll
            for (int b = 0; b < MBW; ++b)
                acc[a][b] = v4i{0, 0, 0, 0};
        auto multiply = [&](int cc, int slot) {
            const uint8_t *st = smem + slot * STAGE + frag_col;
            const bool ok = cc * KSTEPS + step < steps;
            v4i wfr[NB], xfr[MBW];
#pragma unroll
            for (int a = 0; a < NB; ++a)
                wfr[a] = *(const v4i *)(st + (ROWS_X + a * 16 + r16) * KCH);
#pragma unroll
            for (int b = 0; b < MBW; ++b) {
                const v4i v = *(const v4i *)(st + ((part * MBW + b) * 16 + r16) * KCH);
                xfr[b] = ok ? v : v4i{0, 0, 0, 0};
            }
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int b = 0; b < MBW; ++b)
                    // first operand -> register index (n), second -> lane%16 (m)
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wfr[a], xfr[b], acc[a][b], 0, 0, 0);
        };
        block_barrier();  // the ring is free (previous pass: reduction)
#pragma unroll
        for (int t = 0; t < S - 1; ++t)
            dma_stage(chunk_at(t), t);
        int slot = 0, fill = S - 1;  // slot of stage c; slot the next stage goes to
        for (int c = 0; c < chunks; ++c) {
            wait_vmcnt<(S - 2) * PPW>();  // this wave's loads of stage c have landed ...
            block_barrier();              // ... everybody's have, and the slot of stage c - 1 is free
            dma_stage(chunk_at(c + S - 1), fill);
            multiply(chunk_at(c), slot);
            slot = slot + 1 == S ? 0 : slot + 1;
            fill = fill + 1 == S ? 0 : fill + 1;
        }
        wait_vmcnt<0>();  // the loads past the end have landed: the ring can be reused
        // acc[v] of lane l is C[n = 4*(l/16) + v, m = l%16] of its 16x16 block
        v4i(*red)[T][kWave] = (v4i(*)[T][kWave])smem;
#pragma unroll
        for (int a0 = 0; a0 < NB; a0 += RB) {
            block_barrier();  // the ring, or the sums of the blocks before, have been read
#pragma unroll
            for (int a = a0; a < a0 + RB && a < NB; ++a)
#pragma unroll
                for (int b = 0; b < MBW; ++b)
                    red[wave][(a - a0) * MBW + b][lane] = acc[a][b];
            block_barrier();
            for (int t = tid; t < RB * MB * kWave; t += WAVES * kWave) {
                const int a = a0 + t / (MB * kWave), b = (t / kWave) % MB, l = t % kWave;
                const int blk = first + a * grid;
                if (a >= NB || blk >= blocks)
                    continue;
                const int w0 = (b / MBW) * KSTEPS, tile = (a - a0) * MBW + b % MBW;
                v4i sum = red[w0][tile][l];
#pragma unroll
                for (int w = 1; w < KSTEPS; ++w)
                    sum += red[w0 + w][tile][l];
                const int m = b * 16 + (l & 15), n = blk * 16 + 4 * (l >> 4);
                if (m < M && n < N) {
                    float y[4];
                    if constexpr (VEC) {
                        const float rstep = sv.rs[(int64_t)m * sv.rs_stride];
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            y[v] = ((float)sum[v] * rstep) * sv.cs[(int64_t)(n + v) * sv.cs_stride];
                        if (sv.out_i8) {
                            *(uint32_t *)((uint8_t *)Y + (int64_t)m * N + n) =
                                round_to_i8(y[0], sv.out_inv_step) | (round_to_i8(y[1], sv.out_inv_step) << 8) |
                                (round_to_i8(y[2], sv.out_inv_step) << 16) | (round_to_i8(y[3], sv.out_inv_step) << 24);
                            continue;
                        }
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            y[v] = (float)sum[v] * alpha;
                    }
                    *(uint2 *)(Y + (int64_t)m * N + n) = make_uint2(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));
                }
            }
        }
    }
}

// Second half of a K split: out = bf16((*s0 * *s1) * (((p_0 + p_1) + p_2) + ...)), the runs added
// in index order (the result does not depend on which workgroup finished first).
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partials, int splits,
                                                            int64_t mn, const float *__restrict__ s0,
                                                            const float *__restrict__ s1, uint16_t *__restrict__ out)
{
    const float alpha = (*s0) * (*s1);
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i >= mn)
        return;
    v4f lo = *(const v4f *)(partials + i), hi = *(const v4f *)(partials + i + 4);
    for (int s = 1; s < splits; ++s) {
        lo += *(const v4f *)(partials + (int64_t)s * mn + i);
        hi += *(const v4f *)(partials + (int64_t)s * mn + i + 4);
    }
    *(uint4 *)(out + i) = make_uint4(pack_bf16x2(lo[0] * alpha, lo[1] * alpha), pack_bf16x2(lo[2] * alpha, lo[3] * alpha),
                                     pack_bf16x2(hi[0] * alpha, hi[1] * alpha), pack_bf16x2(hi[2] * alpha, hi[3] * alpha));
}

// Second half of a K split on the deferred-epilogue kernel's tiles: the runs sit in the
// workspace in the order the GEMM's lanes held them ([unit = split * tiles + tile][wave][block]
// [quarter][lane] float4: rows lane % 32 of the block, columns 8 * quarter + 4 * (lane / 32) .. +3).
// A wave of this kernel takes one pair of neighbouring blocks of one tile (64 columns x 32 rows),
// adds the runs in index order, scales, rounds and regroups the lanes' values into whole 128-byte
// lines of the output as the GEMM's own write-out does.
// INT8: the runs are int32 sums (added exactly, then y = bf16(fp32(sum) * alpha_i8), Sec. 4.4 Eq. 4).
template <bool INT8>
__global__ __launch_bounds__(256) void splitk_reduce_defer_kernel(const float4 *__restrict__ partials, int splits,
                                                                  int tiles_m, int tiles_n, int N,
                                                                  const float *__restrict__ s0,
                                                                  const float *__restrict__ s1, float alpha_i8,
                                                                  uint16_t *__restrict__ out)
{
    using T = DeferTile<4>;
    const float alpha = INT8 ? alpha_i8 : (*s0) * (*s1);
    const int lane = threadIdx.x & (kWave - 1), l31 = lane & 31, lh = lane >> 5;
    const int task = blockIdx.x * 4 + (threadIdx.x >> 6);  // (tile, wave, band i, block pair jp)
    const int n_tiles = tiles_m * tiles_n;
    const int tile = task >> 5, wave = (task >> 3) & 3, i = (task >> 1) & 3, jp = task & 1;
    if (tile >= n_tiles)
        return;
    const int wm = wave >> 1, wn = wave & 1;
    typedef typename std::conditional<INT8, v4i, v4f>::type sum_t;
    sum_t sum[2][4];
    const int64_t unit_stride = (int64_t)T::NWAVES * T::NB * 4 * kWave;
    const float4 *src = partials + ((int64_t)tile * T::NWAVES + wave) * (T::NB * 4 * kWave) +
                        (int64_t)((i * 4 + 2 * jp) * 4) * kWave + lane;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v = src[(b * 4 + q) * kWave];
            sum[b][q] = __builtin_bit_cast(sum_t, v);
        }
    for (int sp = 1; sp < splits; ++sp) {
        src += (int64_t)n_tiles * unit_stride;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = src[(b * 4 + q) * kWave];
                sum[b][q] += __builtin_bit_cast(sum_t, v);
            }
    }
    uint32_t A[8], B[8];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            A[2 * q + h] = pack_bf16x2((float)sum[0][q][2 * h] * alpha, (float)sum[0][q][2 * h + 1] * alpha);
            B[2 * q + h] = pack_bf16x2((float)sum[1][q][2 * h] * alpha, (float)sum[1][q][2 * h + 1] * alpha);
        }
    block_pair_to_lines(A, B);
    int tm, tn;
    tile_from_id(tile, tiles_m, tiles_n, tm, tn);
    const int64_t row0 = (int64_t)tm * T::BM + wm * 128 + i * 32 + (l31 & ~3);
    const int64_t col0 = (int64_t)tn * T::BN + wn * 128 + jp * 64 + lh * 32 + (l31 & 3) * 8;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        *(uint4 *)(out + (row0 + u) * N + col0) = make_uint4(A[2 * u], A[2 * u + 1], B[2 * u], B[2 * u + 1]);
}

// ---------------------------------------------------------------------------
// host side

typedef Tile<256, 256, 2, 2> T256x256;
typedef Tile<128, 128, 2, 2> T128x128;
typedef Tile<64, 64, 1, 1> T64x64;
typedef TileD<256, 256, 2, 4, 4, 2> D256x256w8;
typedef TileD<128, 128, 2, 2, 4, 2> D128x128w4;
typedef TileS<256, 256, 2, 4, 2, 2> S256x256w8;  // persistent, 8 waves, one workgroup per CU
typedef TileS<128, 128, 2, 2, 2, 2> S128x128w4;  // two workgroups per CU
typedef TileS<192, 256, 2, 4, 2, 2> S192x256w8;  // for tile counts that 256x256 quantises badly

// Measurement hook: pairs of events that the next GEMM kernel launches record at their own
// start and end (a queue, consumed one pair per launch).  Unlike events recorded on the stream
// around a call, these do not drain the stream in front of the kernel.
constexpr int kMaxProfilePairs = 8;
static hipEvent_t g_prof_events[2 * kMaxProfilePairs];
static int g_prof_count = 0, g_prof_next = 0;
bool set_profile_events(void *const *events, int pairs)
{
    if (pairs < 0 || pairs > kMaxProfilePairs)
        return false;
    for (int i = 0; i < 2 * pairs; ++i)
        g_prof_events[i] = (hipEvent_t)events[i];
    g_prof_count = pairs;
    g_prof_next = 0;
    return true;
}
bool take_profile_events(hipEvent_t *e0, hipEvent_t *e1)
{
    if (g_prof_next >= g_prof_count)
        return false;
    *e0 = g_prof_events[2 * g_prof_next];
    *e1 = g_prof_events[2 * g_prof_next + 1];
    ++g_prof_next;
    return true;
}
template <typename KERNEL, typename... ARGS>
static void launch_gemm_kernel(KERNEL kernel, dim3 grid, dim3 block, size_t lds, hipStream_t s, ARGS... args)
{
    hipEvent_t e0, e1;
    if (take_profile_events(&e0, &e1)) {
        hipExtLaunchKernelGGL(kernel, grid, block, lds, s, e0, e1, 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
    }
}

int num_cus_public();
static int g_tile_override = 0;
static bool g_stream_k_off = true;  // measured slower than the plain schedule on MI355X: opt-in
void set_gemm_tile_override(int variant) { g_tile_override = variant; }
void set_stream_k(bool on) { g_stream_k_off = !on; }
bool stream_k_enabled() { return !g_stream_k_off; }

// stream-K workspace: arrival counters (one per remainder tile, fewer than workgroups), then two
// accumulator slots of one tile per workgroup
constexpr size_t kStreamKCounterBytes = 4096;
constexpr int kStreamKMaxWorkgroups = 1024;
size_t stream_k_workspace_bytes()
{
    return kStreamKCounterBytes + (size_t)2 * num_cus_public() * 256 * 256 * 4;
}

// Kernel variants (the numbers are what tweo_set_gemm_tile takes; retired ones are refused).
// 1, 3, 4: register-staged kernel (any K % 16 == 0), tiles 256x256, 128x128, 64x64.  6, 8:
// DMA-pipelined kernel on 64-byte stages (K % 64 == 0), 256x256 with 8 waves and 128x128.  11, 13,
// 14: persistent streaming kernel (K % 128 == 0): 256x256, 128x128, 192x256.  15: deferred-epilogue
// persistent kernel (256x256, four waves; M, N % 256 == 0, K % 128 == 0, K >= 512).  16: the same
// kernel on 192x256 tiles (any M, K >= 2048).  17: the INT8 weight-streaming kernel (M <= 128).
constexpr int kNumVariants = 17;
static const int kVariantBM[kNumVariants + 1] = {0, 256, 256, 128, 64, 256, 256, 256, 128, 256, 128, 256, 256, 128, 192, 256, 192, 64};
static const int kVariantBN[kNumVariants + 1] = {0, 256, 128, 128, 64, 256, 256, 128, 128, 128, 256, 256, 128, 128, 256, 256, 256, 64};
int gemm_num_variants() { return kNumVariants; }
bool gemm_variant_exists(int v)
{
    return v >= 0 && v <= kNumVariants && v != 2 && v != 5 && v != 7 && v != 9 && v != 10 && v != 12;
}

static int num_cus();
int num_cus_public() { return num_cus(); }
static int num_cus()
{
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
    }
    return n;
}

constexpr int kMaxDeferWorkgroups = 1024;
static int defer_workgroups(int64_t M, int64_t N, int bm = 256)
{
    const int64_t tiles = ((M + bm - 1) / bm) * (N / 256);
    const int64_t cap = num_cus() < kMaxDeferWorkgroups ? num_cus() : kMaxDeferWorkgroups;
    return (int)(tiles < cap ? tiles : cap);
}

static int pick_variant(int64_t M, int64_t N, int64_t K)
{
    auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
    int v = g_tile_override >= 17 ? 4 : g_tile_override;
    if (v == 0) {
        if (M * N <= 128 * 128 * 16) {
            v = 4;
        } else {
            // rounds of tiles over the machine x cost of a tile; per-workgroup speeds are measured
            // ratios: the persistent 256x256 kernel owns a CU, the 128x128 one shares it in pairs
            const double cus = num_cus();
            auto cost = [&](int bm, int bn, double slots, double speed) {
                const double rounds = (double)((tiles(bm, bn) + (int64_t)slots - 1) / (int64_t)slots);
                return rounds * bm * bn / speed;
            };
            const double c11 = cost(256, 256, cus, 1.0);
            const double c13 = cost(128, 128, 2 * cus, 0.425);
            const double c14 = cost(192, 256, cus, 0.97);
            // The deferred-epilogue kernel (one wave per SIMD, operand halves refilled behind
            // their own barriers) where the shape allows it: ahead of the 8-wave kernel by 15 %
            // when a tile's write-out has 15 stages to hide under, by nothing at 6 stages.
            const int64_t kt = K / 128;
            const bool e15 = M % 256 == 0 && N % 256 == 0 && K % 128 == 0 && K >= 512 && 2 * tiles(256, 256) >= (int64_t)cus;
            const bool e16 = N % 256 == 0 && K % 128 == 0 && K >= 2048;
            const double gain = kt >= 16 ? 1.15 : (kt >= 8 ? 1.08 : 1.0);
            const double c15 = e15 ? cost(256, 256, cus, gain) : 1e300;
            const double c16 = e16 ? cost(192, 256, cus, 0.97 * gain) : 1e300;
            v = 11;
            double best = c11;
            if (c14 < best) {
                v = 14;
                best = c14;
            }
            if (c15 < best) {
                v = 15;
                best = c15;
            }
            if (c16 < best) {
                v = 16;
                best = c16;
            }
            if (c13 < best)
                v = 13;
            if (v == 11 && e15)
                v = 15;
            if (v == 14 && e16)
                v = 16;
            // few K stages per tile: the big tiles' fixed cost per tile (fill, write-out) weighs
            // more than the model's rounds say (8192x2304, K = 768: 26 us against 31 us measured)
            if (v == 14 && K < 1024 && c13 < 1.2 * c14)
                v = 13;
            // at most one 128x128 tile per CU under a long contraction: the non-persistent
            // kernel with its four-stage ring is 10-15 % ahead (weight gradients of narrow layers);
            // with more tiles than CUs it falls behind (INT8, 12288 wide over 4096 at M = 384 / 512:
            // 39 / 47 us against 32 / 37)
            if (v == 13 && K >= 4096 && K % 64 == 0 && tiles(128, 128) <= (int64_t)cus)
                v = 8;
        }
    }
    if (v >= 11 && K % 128 != 0)  // the persistent kernels need whole 128-byte stages
        v = v == 13 ? 8 : 6;
    if (v >= 5 && K % 64 != 0)
        v = v == 6 ? 1 : 3;
    return v;
}

// The deferred-epilogue kernel covers whole 256x256 tiles, K in whole stages with enough of
// them to drain a tile under, no residual, p in {0, 4}.
static bool defer_ok(const GemmArgs &a)
{
    return a.M % 256 == 0 && a.N % 256 == 0 && a.K % 128 == 0 && a.K >= 512 && a.residual == nullptr &&
           a.row_step == nullptr && (a.p == 0 || a.p == 4) && a.N <= ((int64_t)1 << 22);
}

static bool defer192_ok(const GemmArgs &a)
{
    return a.N % 256 == 0 && a.K % 128 == 0 && a.K >= 2048 && a.residual == nullptr &&
           a.row_step == nullptr && (a.p == 0 || a.p == 4) && a.N <= ((int64_t)1 << 22);
}

static int resolve_variant(const GemmArgs &a)
{
    int v = pick_variant(a.M, a.N, a.K);
    if (v == 15 && !defer_ok(a))
        v = 11;
    if (v == 16 && !defer192_ok(a))
        v = 14;
    return v;
}

int fp8_gemm_partials(const GemmArgs &a)
{
    const int v = resolve_variant(a);
    if (v == 15 || v == 16)  // one partial per wave of each workgroup (never more than per 64x64 block)
        return defer_workgroups(a.M, a.N, kVariantBM[v]) * DeferTile<4>::PARTIALS_PER_WG;
    return (int)(((a.M + kVariantBM[v] - 1) / kVariantBM[v]) * ((a.N + kVariantBN[v] - 1) / kVariantBN[v]));
}

template <typename T, bool INT8, bool DMA, bool A_E5M2 = false>
static hipError_t launch_tile(const GemmArgs &a, hipStream_t s)
{
    static bool attr_done = false;  // per instantiation
    const void *kern;
    if constexpr (DMA)
        kern = (const void *)gemm_nt_dma_kernel<T, INT8>;
    else
        kern = (const void *)gemm_nt_kernel<T, INT8, A_E5M2>;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           T::LDS_BYTES);
        if (e != hipSuccess)
            return e;
        attr_done = true;
    }
    GemmDev g;
    g.A = a.A;
    g.B = a.B;
    g.M = (int)a.M;
    g.N = (int)a.N;
    g.K = (int)a.K;
    g.s0 = a.s0;
    g.s1 = a.s1;
    g.alpha = a.alpha;
    g.residual = (const uint16_t *)a.residual;
    g.out = (uint16_t *)a.out;
    g.inv_tau = a.inv_tau;
    g.p = a.p;
    g.partials = a.partials;
    g.rs = a.row_step;
    g.cs = a.col_step;
    g.rs_stride = a.row_step_stride;
    g.cs_stride = a.col_step_stride;
    g.out_i8 = a.out_i8 ? 1 : 0;
    g.out_inv_step = a.out_inv_step;
    g.ksplit = 1;
    g.ksplit_out = nullptr;
    g.tiles_m = (int)((a.M + T::BM - 1) / T::BM);
    g.tiles_n = (int)((a.N + T::BN - 1) / T::BN);
    const dim3 grid((unsigned)(g.tiles_m * g.tiles_n)), block(T::THREADS);
    if constexpr (DMA)
        launch_gemm_kernel(gemm_nt_dma_kernel<T, INT8>, grid, block, T::LDS_BYTES, s, g);
    else
        launch_gemm_kernel(gemm_nt_kernel<T, INT8, A_E5M2>, grid, block, T::LDS_BYTES, s, g);
    return hipGetLastError();
}

// Stream-K pays when a tile count leaves a noticeable part of the last round idle and each
// workgroup's share of the remainder is long enough to amortise a fixup.
static bool stream_k_plan(int64_t total_tiles, int64_t kt, int grid, const GemmArgs &a, size_t slot_bytes,
                          int &full_rounds)
{
    if (g_stream_k_off || total_tiles <= 0 || grid <= 0)
        return false;
    full_rounds = (int)(total_tiles / grid);
    const int64_t rem = total_tiles % grid;
    if (rem == 0 || kt < 16 || rem * kt / grid < 16)
        return false;
    const int64_t rounds = full_rounds + 1;
    if ((double)(rounds * grid - total_tiles) / (double)(rounds * grid) < 0.04)
        return false;
    const size_t need = kStreamKCounterBytes + (size_t)2 * grid * slot_bytes;
    return a.sk_workspace != nullptr && a.sk_workspace_bytes >= need &&
           ((uintptr_t)a.sk_workspace & 255u) == 0;
}

template <typename T, bool INT8, int WG_PER_CU, bool SK>
static hipError_t launch_stream_inst(const GemmArgs &a, hipStream_t s, int grid, int full_rounds)
{
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_nt_stream_kernel<T, INT8, SK>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess)
            return e;
        attr_done = true;
    }
    GemmDev g;
    g.A = a.A;
    g.B = a.B;
    g.M = (int)a.M;
    g.N = (int)a.N;
    g.K = (int)a.K;
    g.s0 = a.s0;
    g.s1 = a.s1;
    g.alpha = a.alpha;
    g.residual = (const uint16_t *)a.residual;
    g.out = (uint16_t *)a.out;
    g.inv_tau = a.inv_tau;
    g.p = a.p;
    g.partials = a.partials;
    g.rs = a.row_step;
    g.cs = a.col_step;
    g.rs_stride = a.row_step_stride;
    g.cs_stride = a.col_step_stride;
    g.out_i8 = a.out_i8 ? 1 : 0;
    g.out_inv_step = a.out_inv_step;
    g.ksplit = 1;
    g.ksplit_out = nullptr;
    g.tiles_m = (int)((a.M + T::BM - 1) / T::BM);
    g.tiles_n = (int)((a.N + T::BN - 1) / T::BN);
    g.sk_full_rounds = full_rounds;
    g.sk_counters = (uint32_t *)a.sk_workspace;
    g.sk_partials = (uint8_t *)a.sk_workspace + kStreamKCounterBytes;
    if constexpr (SK) {
        hipError_t e = launch_fill_u32(g.sk_counters, (int)(kStreamKCounterBytes / 4), 0u, s);
        if (e != hipSuccess)
            return e;
    }
    launch_gemm_kernel(gemm_nt_stream_kernel<T, INT8, SK>, dim3((unsigned)grid), dim3(T::THREADS), T::LDS_BYTES, s, g);
    return hipGetLastError();
}

template <typename T, bool INT8, int WG_PER_CU>
static hipError_t launch_stream(const GemmArgs &a, hipStream_t s)
{
    const int64_t total = ((a.M + T::BM - 1) / T::BM) * ((a.N + T::BN - 1) / T::BN);
    int grid = num_cus() * WG_PER_CU;
    if (grid > total)
        grid = (int)total;
    if constexpr (WG_PER_CU == 1) {
        // stream-K always runs one workgroup on every CU (with fewer tiles than CUs the split
        // remainder is the whole job)
        int full_rounds = 0;
        const int cus = num_cus();
        if (cus <= kStreamKMaxWorkgroups &&
            stream_k_plan(total, a.K / T::BK, cus, a, (size_t)T::BM * T::BN * 4, full_rounds))
            return launch_stream_inst<T, INT8, WG_PER_CU, true>(a, s, cus, full_rounds);
    }
    return launch_stream_inst<T, INT8, WG_PER_CU, false>(a, s, grid, 0);
}

template <bool INT8, int PMODE, int D, int MT, bool A_E5M2 = false>
static hipError_t launch_defer_inst(const GemmArgs &a, hipStream_t s)
{
    using T = DeferTile<MT>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_nt_defer_kernel<INT8, PMODE, D, MT, A_E5M2>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess)
            return e;
        attr_done = true;
    }
    GemmDev g;
    g.A = a.A;
    g.B = a.B;
    g.M = (int)a.M;
    g.N = (int)a.N;
    g.K = (int)a.K;
    g.s0 = a.s0;
    g.s1 = a.s1;
    g.alpha = a.alpha;
    g.residual = nullptr;
    g.out = (uint16_t *)a.out;
    g.inv_tau = a.inv_tau;
    g.p = a.p;
    g.partials = a.partials;
    g.rs = a.row_step;
    g.cs = a.col_step;
    g.rs_stride = a.row_step_stride;
    g.cs_stride = a.col_step_stride;
    g.out_i8 = a.out_i8 ? 1 : 0;
    g.out_inv_step = a.out_inv_step;
    g.ksplit = 1;
    g.ksplit_out = nullptr;
    g.tiles_m = (int)((a.M + T::BM - 1) / T::BM);
    g.tiles_n = (int)(a.N / T::BN);
    const int grid = defer_workgroups(a.M, a.N, T::BM);
    launch_gemm_kernel(gemm_nt_defer_kernel<INT8, PMODE, D, MT, A_E5M2>, dim3((unsigned)grid), dim3(T::THREADS), T::LDS_BYTES, s, g);
    return hipGetLastError();
}

template <bool INT8>
static hipError_t launch_defer(const GemmArgs &a, hipStream_t s)
{
    // a tile is written out over the first 15, 7, 5 or 3 stages of the next one (never its last)
    const int64_t kt = a.K / 128;
    if (a.p == 4) {
        if (kt >= 16)
            return launch_defer_inst<INT8, 4, 15, 4>(a, s);
        if (kt >= 8)
            return launch_defer_inst<INT8, 4, 7, 4>(a, s);
        return kt >= 6 ? launch_defer_inst<INT8, 4, 5, 4>(a, s) : launch_defer_inst<INT8, 4, 3, 4>(a, s);
    }
    if (kt >= 16)
        return launch_defer_inst<INT8, 0, 15, 4>(a, s);
    if (kt >= 8)
        return launch_defer_inst<INT8, 0, 7, 4>(a, s);
    return kt >= 6 ? launch_defer_inst<INT8, 0, 5, 4>(a, s) : launch_defer_inst<INT8, 0, 3, 4>(a, s);
}

// 192x256 tiles: long contractions only (K >= 2048)
template <bool INT8>
static hipError_t launch_defer192(const GemmArgs &a, hipStream_t s)
{
    return a.p == 4 ? launch_defer_inst<INT8, 4, 15, 3>(a, s) : launch_defer_inst<INT8, 0, 15, 3>(a, s);
}

template <bool INT8>
static hipError_t launch_gemm(const GemmArgs &a, hipStream_t s)
{
    switch (resolve_variant(a)) {
    case 1: return launch_tile<T256x256, INT8, false>(a, s);
    case 3: return launch_tile<T128x128, INT8, false>(a, s);
    case 4: return launch_tile<T64x64, INT8, false>(a, s);
    case 6: return launch_tile<D256x256w8, INT8, true>(a, s);
    case 8: return launch_tile<D128x128w4, INT8, true>(a, s);
    case 11: return launch_stream<S256x256w8, INT8, 1>(a, s);
    case 13: return launch_stream<S128x128w4, INT8, 2>(a, s);
    case 14: return launch_stream<S192x256w8, INT8, 1>(a, s);
    case 15: return launch_defer<INT8>(a, s);
    default: return launch_defer192<INT8>(a, s);
    }
}

// K split for outputs with far fewer tiles than CUs and a very long contraction (weight gradients
// of narrow layers: 2304x768 over 50432 tokens is 27 tiles): `splits` workgroups per 256x256
// tile, each at least 16 stages long, fp32 runs to scratch, one reduce launch.  1 = no split.
// Measured: 349 -> 117 us for that shape, 104 -> 94 us for 2048x2048 over 16384 (64 tiles, the
// limit taken); at a contraction of 8192 the scratch traffic and the second launch eat the gain
// (40 -> 46 us), hence the 16384 floor.
// The same on the deferred-epilogue kernel (whole 256x256 tiles, K in whole 128-byte stages), one
// unit per CU at most and at least 16 stages per unit (with 8 the fp32 runs' traffic grows faster
// than the units shrink).  Measured in the blocks' steps: 2304x768 over 50432 tokens 117 -> 88 us,
// 3072x768 143 -> 111 us, 2048x2048 over 16384 91 -> 71 us; over 8192 tokens 2304x768 49 -> 35 us,
// 768x768 48 -> 30 us, 3072x768 51 -> 39 us; a contraction of 4096 loses (14 -> 20 us), and so do
// 64 tiles over 8192 (40 -> 46 us).  From 80 stages on, up to half as many tiles as CUs are split
// (INT8, 4096 wide over 11008: 64 tiles 67 -> 60 us, 80 tiles 106 -> 68 us): the INT8 flavour of the
// same kernel leaves int32 runs, which the reduce kernel adds exactly.
constexpr int kKsplitDeferMinStages = 16, kKsplitDeferMinKt = 64;
static int defer_ksplit(int64_t M, int64_t N, int64_t K)
{
    if (g_tile_override != 0 || M % 256 != 0 || N % 256 != 0 || K % 128 != 0 || N > ((int64_t)1 << 22))
        return 1;
    const int64_t tiles = (M / 256) * (N / 256), kt = K / 128, cus = num_cus();
    if (kt < kKsplitDeferMinKt || tiles * (kt >= 80 ? 2 : 6) > cus)
        return 1;
    int64_t splits = cus / tiles;
    if (splits > kt / kKsplitDeferMinStages)
        splits = kt / kKsplitDeferMinStages;
    if (splits > 32)
        splits = 32;
    return splits >= 2 ? (int)splits : 1;
}

int fp8_gemm_ksplit(int64_t M, int64_t N, int64_t K)
{
    if (g_tile_override != 0)
        return 1;
    const int ds = defer_ksplit(M, N, K);
    if (ds > 1)
        return ds;
    const int64_t tiles = ((M + 255) / 256) * ((N + 255) / 256), k_tiles = (K + kBK - 1) / kBK;
    const int64_t cus = num_cus();
    if (tiles * 4 > cus || k_tiles < 128)
        return 1;
    int64_t splits = cus / tiles;
    if (splits > k_tiles / 16)
        splits = k_tiles / 16;
    if (splits > 32)
        splits = 32;
    return splits >= 2 ? (int)splits : 1;
}

size_t fp8_gemm_ksplit_bytes(int64_t M, int64_t N, int64_t K)
{
    const int splits = fp8_gemm_ksplit(M, N, K);
    return splits > 1 ? (size_t)splits * (size_t)M * (size_t)N * sizeof(float) : 0;
}

// DMA: the direct-to-LDS kernel on 64-byte stages (K % 64 == 0, E4M3 operands), else the
// register-staged one.
template <bool A_E5M2, bool DMA>
static hipError_t launch_ksplit(const GemmArgs &a, hipStream_t s, int splits)
{
    using T = typename std::conditional<DMA, D256x256w8, T256x256>::type;
    static_assert(!(DMA && A_E5M2), "the direct-to-LDS kernel takes E4M3 operands only");
    const void *kern;
    if constexpr (DMA)
        kern = (const void *)gemm_nt_dma_kernel<T, false>;
    else
        kern = (const void *)gemm_nt_kernel<T, false, A_E5M2>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess)
            return e;
        attr_done = true;
    }
    GemmDev g{};
    g.A = a.A;
    g.B = a.B;
    g.M = (int)a.M;
    g.N = (int)a.N;
    g.K = (int)a.K;
    g.s0 = a.s0;
    g.s1 = a.s1;
    g.out = (uint16_t *)a.out;
    g.tiles_m = (int)((a.M + T::BM - 1) / T::BM);
    g.tiles_n = (int)((a.N + T::BN - 1) / T::BN);
    g.ksplit = splits;
    g.ksplit_out = (float *)a.sk_workspace;
    const dim3 grid((unsigned)(g.tiles_m * g.tiles_n * splits)), block(T::THREADS);
    const int64_t mn = a.M * a.N;
    const dim3 rgrid((unsigned)((mn / 8 + 255) / 256));
    // a profiled launch brackets both kernels: start event on the first, end event on the second
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (g_prof_next < g_prof_count) {
        e0 = g_prof_events[2 * g_prof_next];
        e1 = g_prof_events[2 * g_prof_next + 1];
        ++g_prof_next;
    }
    auto launch_first = [&](auto kernel) {
        if (e0 != nullptr)
            hipExtLaunchKernelGGL(kernel, grid, block, T::LDS_BYTES, s, e0, nullptr, 0, g);
        else
            hipLaunchKernelGGL(kernel, grid, block, T::LDS_BYTES, s, g);
    };
    if constexpr (DMA)
        launch_first(gemm_nt_dma_kernel<T, false>);
    else
        launch_first(gemm_nt_kernel<T, false, A_E5M2>);
    if (e1 != nullptr)
        hipExtLaunchKernelGGL(splitk_reduce_kernel, rgrid, dim3(256), 0, s, nullptr, e1, 0,
                              (const float *)g.ksplit_out, splits, mn, a.s0, a.s1, (uint16_t *)a.out);
    else
        hipLaunchKernelGGL(splitk_reduce_kernel, rgrid, dim3(256), 0, s, (const float *)g.ksplit_out, splits, mn, a.s0,
                           a.s1, (uint16_t *)a.out);
    return hipGetLastError();
}

template <bool A_E5M2, bool INT8 = false>
static hipError_t launch_ksplit_defer(const GemmArgs &a, hipStream_t s, int splits)
{
    using T = DeferTile<4>;
    const void *kern = (const void *)gemm_nt_defer_kernel<INT8, 0, 3, 4, A_E5M2, true, true>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess)
            return e;
        attr_done = true;
    }
    GemmDev g{};
    g.A = a.A;
    g.B = a.B;
    g.M = (int)a.M;
    g.N = (int)a.N;
    g.K = (int)a.K;
    g.s0 = a.s0;
    g.s1 = a.s1;
    g.out = (uint16_t *)a.out;
    g.tiles_m = (int)(a.M / T::BM);
    g.tiles_n = (int)(a.N / T::BN);
    g.ksplit = splits;
    g.ksplit_out = (float *)a.sk_workspace;
    const int n_tiles = g.tiles_m * g.tiles_n;
    const dim3 grid((unsigned)(n_tiles * splits)), block(T::THREADS), rgrid((unsigned)(n_tiles * 8));
    hipEvent_t e0 = nullptr, e1 = nullptr;  // a profiled launch brackets both kernels
    take_profile_events(&e0, &e1);
    if (e0 != nullptr)
        hipExtLaunchKernelGGL((gemm_nt_defer_kernel<INT8, 0, 3, 4, A_E5M2, true, true>), grid, block, T::LDS_BYTES, s, e0,
                              nullptr, 0, g);
    else
        hipLaunchKernelGGL((gemm_nt_defer_kernel<INT8, 0, 3, 4, A_E5M2, true, true>), grid, block, T::LDS_BYTES, s, g);
    if (e1 != nullptr)
        hipExtLaunchKernelGGL(splitk_reduce_defer_kernel<INT8>, rgrid, dim3(256), 0, s, nullptr, e1, 0,
                              (const float4 *)g.ksplit_out, splits, g.tiles_m, g.tiles_n, g.N, a.s0, a.s1, a.alpha,
                              (uint16_t *)a.out);
    else
        hipLaunchKernelGGL(splitk_reduce_defer_kernel<INT8>, rgrid, dim3(256), 0, s, (const float4 *)g.ksplit_out, splits,
                           g.tiles_m, g.tiles_n, g.N, a.s0, a.s1, a.alpha, (uint16_t *)a.out);
    return hipGetLastError();
}

// E5M2 A operand (gradient GEMMs of the HYBRID recipe; no penalty, no residual): the deferred
// kernel where it applies, else the register-staged kernel.
static hipError_t launch_fp8_gemm_e5m2(const GemmArgs &a, hipStream_t s)
{
    if (a.p != 0 || a.residual != nullptr)
        return hipErrorInvalidValue;
    const int v = resolve_variant(a);
    if (v == 15) {
        const int64_t kt = a.K / 128;
        if (kt >= 16)
            return launch_defer_inst<false, 0, 15, 4, true>(a, s);
        if (kt >= 8)
            return launch_defer_inst<false, 0, 7, 4, true>(a, s);
        return kt >= 6 ? launch_defer_inst<false, 0, 5, 4, true>(a, s) : launch_defer_inst<false, 0, 3, 4, true>(a, s);
    }
    if (v == 16)
        return launch_defer_inst<false, 0, 15, 3, true>(a, s);
    if (a.M * a.N <= 128 * 128 * 16)
        return launch_tile<T64x64, false, false, true>(a, s);
    if (a.M * a.N <= 1024 * 1024)
        return launch_tile<T128x128, false, false, true>(a, s);
    return launch_tile<T256x256, false, false, true>(a, s);
}

hipError_t launch_fp8_gemm(const GemmArgs &a, hipStream_t s)
{
    if (a.p == 0 && a.residual == nullptr) {
        const int splits = fp8_gemm_ksplit(a.M, a.N, a.K);
        if (splits > 1 && a.sk_workspace != nullptr && ((uintptr_t)a.sk_workspace & 15u) == 0 &&
            a.sk_workspace_bytes >= (size_t)splits * (size_t)a.M * (size_t)a.N * sizeof(float))
        {
            if (defer_ksplit(a.M, a.N, a.K) > 1)
                return a.a_e5m2 ? launch_ksplit_defer<true>(a, s, splits) : launch_ksplit_defer<false>(a, s, splits);
            if (a.a_e5m2)
                return launch_ksplit<true, false>(a, s, splits);
            return a.K % 64 == 0 ? launch_ksplit<false, true>(a, s, splits) : launch_ksplit<false, false>(a, s, splits);
        }
    }
    return a.a_e5m2 ? launch_fp8_gemm_e5m2(a, s) : launch_gemm<false>(a, s);
}
template <int MB, int NB, int KSTEPS, int S>
static hipError_t launch_skinny_ring(const GemmArgs &a, hipStream_t s)
{
    constexpr int LDS = S * (MB * 16 + NB * 16) * KSTEPS * 64;
    static bool attr_done[2] = {false, false};
    const int vec = a.row_step != nullptr ? 1 : 0;
    const void *kern = vec ? (const void *)w8a8_skinny_ring_kernel<MB, NB, KSTEPS, S, true>
                           : (const void *)w8a8_skinny_ring_kernel<MB, NB, KSTEPS, S, false>;
    if (!attr_done[vec]) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess)
            return e;
        attr_done[vec] = true;
    }
    const int blocks = (int)((a.N + 15) / 16);
    int grid = num_cus();
    if (grid > blocks)
        grid = blocks;
    const StepVectors sv{a.row_step, a.col_step, a.row_step_stride, a.col_step_stride, a.out_i8 ? 1 : 0, a.out_inv_step};
    if (vec)
        launch_gemm_kernel(w8a8_skinny_ring_kernel<MB, NB, KSTEPS, S, true>, dim3((unsigned)grid), dim3(512), LDS, s,
                           (const int8_t *)a.A, (const int8_t *)a.B, (int)a.M, (int)a.N, (int)a.K, a.alpha, sv,
                           (uint16_t *)a.out);
    else
        launch_gemm_kernel(w8a8_skinny_ring_kernel<MB, NB, KSTEPS, S, false>, dim3((unsigned)grid), dim3(512), LDS, s,
                           (const int8_t *)a.A, (const int8_t *)a.B, (int)a.M, (int)a.N, (int)a.K, a.alpha, sv,
                           (uint16_t *)a.out);
    return hipGetLastError();
}

// stage shapes: M <= 16: 512 bytes of K a stage (eight k steps, one per wave); above: 256 bytes (four
// k steps x two parts of the M blocks; 512 where a workgroup has one block of weight rows); ring depth
// what 160 KB of LDS allow (the depth hardly matters: two stages measured like five)
constexpr int64_t kSkinnyMaxM = 128;  // rows of X the weight-streaming kernel takes
static hipError_t launch_skinny_ring_any(const GemmArgs &a, hipStream_t s)
{
    const int64_t blocks = (a.N + 15) / 16, cus = num_cus();
    const int64_t per = (blocks + cus - 1) / cus;
    if (a.M <= 16) {
        if (per <= 1)
            return launch_skinny_ring<1, 1, 8, 6>(a, s);
        if (per == 2)
            return launch_skinny_ring<1, 2, 8, 5>(a, s);
        if (per == 3)
            return launch_skinny_ring<1, 3, 8, 4>(a, s);
        return launch_skinny_ring<1, 4, 8, 3>(a, s);
    }
    if (a.M <= 32) {
        if (per <= 1)
            return launch_skinny_ring<2, 1, 4, 8>(a, s);
        if (per == 2)
            return launch_skinny_ring<2, 2, 4, 8>(a, s);
        if (per == 3)
            return launch_skinny_ring<2, 3, 4, 6>(a, s);
        return launch_skinny_ring<2, 4, 4, 6>(a, s);
    }
    if (a.M <= 64) {
        if (per <= 1)  // 512-byte stages: half as many barriers (11008 -> 4096 at M = 64: 18.0 -> 16.7 us)
            return launch_skinny_ring<4, 1, 8, 3>(a, s);
        if (per == 2)
            return launch_skinny_ring<4, 2, 4, 6>(a, s);
        if (per == 3)
            return launch_skinny_ring<4, 3, 4, 5>(a, s);
        return launch_skinny_ring<4, 4, 4, 4>(a, s);
    }
    if (a.M > 128)  // up to 256 rows for one block of weight rows per workgroup (see launch_i8_gemm)
        return a.M <= 192 ? launch_skinny_ring<12, 1, 4, 3>(a, s) : launch_skinny_ring<16, 1, 4, 2>(a, s);
    // 64 < M <= 128: eight blocks of 16 rows of X beside the weight rows, 256-byte stages
    if (per <= 1)
        return launch_skinny_ring<8, 1, 4, 4>(a, s);
    if (per == 2)
        return launch_skinny_ring<8, 2, 4, 4>(a, s);
    if (per == 3)
        return launch_skinny_ring<8, 3, 4, 3>(a, s);
    return launch_skinny_ring<8, 4, 4, 3>(a, s);
}

hipError_t launch_i8_gemm(const GemmArgs &a, hipStream_t s)
{
    // small M: the weight-streaming kernel (forced tiled variants keep the tiled kernels, for
    // tests; 17 forces this one).  Measured cold at the 7B shapes, kernel time in us for M = 1 /
    // 16 / 32 / 64 / 128: 4096 -> 12288: 10.7 / 11.3 / 13.0 / 15.6 / 19.6, 11008 -> 4096: 10.2 / 10.8 /
    // 14.1 / 16.8 / 27.0 (a plain read of the 45-50 MB of weights by one kernel takes 10.2-11.1; the
    // tiled kernels at M = 128: 27 and 66).
    if ((g_tile_override == 0 || g_tile_override == 17) && a.M <= kSkinnyMaxM && a.K % 64 == 0 && a.N % 4 == 0)
        return launch_skinny_ring_any(a, s);
    // up to 256 rows into a projection of at most one block of 16 weight rows per CU under a long
    // contraction (11008 -> 4096: 16 tiles of 256x256): still the weight stream, unless the K split
    // below applies (M = 256 with a workspace)
    if ((g_tile_override == 0 || g_tile_override == 17) && a.M <= 256 && a.K % 64 == 0 && a.N % 4 == 0 &&
        a.K >= 8192 && (a.N + 15) / 16 <= num_cus() &&
        !(a.row_step == nullptr && !a.out_i8 && defer_ksplit(a.M, a.N, a.K) > 1 && a.sk_workspace != nullptr &&
          a.sk_workspace_bytes >= (size_t)defer_ksplit(a.M, a.N, a.K) * (size_t)a.M * (size_t)a.N * sizeof(int32_t)))
        return launch_skinny_ring_any(a, s);
    // few whole 256x256 tiles under a long contraction (prefill chunks of a few hundred tokens into
    // a narrow projection): the K split of the deferred-epilogue kernel, int32 runs added exactly
    if (a.row_step == nullptr && !a.out_i8) {
        const int splits = defer_ksplit(a.M, a.N, a.K);
        if (splits > 1 && a.sk_workspace != nullptr && ((uintptr_t)a.sk_workspace & 15u) == 0 &&
            a.sk_workspace_bytes >= (size_t)splits * (size_t)a.M * (size_t)a.N * sizeof(int32_t))
            return launch_ksplit_defer<false, true>(a, s, splits);
    }
    return launch_gemm<true>(a, s);
}

}  // namespace tweo
