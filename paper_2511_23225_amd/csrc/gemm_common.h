// Pieces shared by the 8-bit GEMM kernels (gfx950).
#pragma once
#include <type_traits>
#include "kernels.h"
#include "device_utils.h"

namespace tweo {

// C[M,N] = A[M,K] * B[N,K]^T, both operands K-contiguous; see GemmArgs for the fields.
struct GemmDev {
    const uint8_t *A, *B;
    int M, N, K;
    const float *s0, *s1;
    float alpha;
    const uint16_t *residual;
    uint16_t *out;
    float inv_tau;
    int p;
    float *partials;
    int tiles_m, tiles_n;
    // stream-K only: whole rounds of tiles before the split remainder, fp32/int32 accumulator
    // slots (2 per workgroup, one tile each) and one arrival counter per remainder tile (zeroed)
    int sk_full_rounds;
    void *sk_partials;
    uint32_t *sk_counters;
    // INT8 only, both or neither: dequantisation steps per output row / column (stride 1) or per
    // tensor (stride 0); then y = bf16((fp32(acc) * rs[m*rs_stride]) * cs[n*cs_stride])
    const float *rs, *cs;
    int rs_stride, cs_stride;
    // with step vectors only: out holds int8 [M,N] = clamp(rne(y * out_inv_step), +-127) instead of bf16
    int out_i8;
    float out_inv_step;
    // K split (register-staged FP8 kernel only): ksplit > 1 workgroups share a tile, workgroup
    // `split` multiplies its run of K stages and stores the fp32 sums to
    // ksplit_out[split][M][N]; a second kernel adds the runs in order and rounds
    int ksplit;
    float *ksplit_out;
};

// raster of tile ids: groups of 8 tile rows, column-major inside a group
__device__ __forceinline__ void tile_from_id(int id, int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int GROUP = 8;
    const int width = GROUP * tiles_n;
    const int group = id / width, first_m = group * GROUP;
    const int gsz = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
    const int in_group = id - group * width;
    tm = first_m + in_group % gsz;
    tn = in_group / gsz;
}

// One 16-byte-per-lane DMA load: LDS[m0 + lane*16 ..] = global[base + voff ..].
__device__ __forceinline__ void dma_load16(uint32_t lds_addr, const uint8_t *base, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory", "m0");
}

// 4x4 transposition of p0..p3 over the four lanes of a quad: afterwards register u of lane a holds
// what register a of lane u held.  Two rounds of pairwise exchanges (partner lane ^ 1 on register
// pairs (0,1), (2,3); partner lane ^ 2 on pairs (0,2), (1,3)): a lane whose bit is clear takes the
// partner's lower register into its upper one, a lane whose bit is set the partner's upper
// register into its lower one.  Each exchange is one v_cndmask_b32 whose first source comes
// through the DPP quad permutation (vcc ? src1 : permuted src0); the compiler does not fuse the
// two, hence asm.  A DPP source must have been written two wait states earlier: the order below
// keeps every result two instructions away from its use, and the leading s_nop covers the inputs.
struct QuadMasks {
    uint64_t odd, even, upper, lower;  // lanes with lane & 1 set / clear, lane & 2 set / clear
};
__device__ __forceinline__ QuadMasks quad_masks()
{
    return QuadMasks{0xAAAAAAAAAAAAAAAAull, 0x5555555555555555ull, 0xCCCCCCCCCCCCCCCCull, 0x3333333333333333ull};
}
__device__ __forceinline__ void quad_transpose(uint32_t &p0, uint32_t &p1, uint32_t &p2, uint32_t &p3, const QuadMasks &m)
{
    uint32_t n0, n1, n2, n3, r0, r1, r2, r3;
    asm volatile("s_nop 1\n\t"
                 "s_mov_b64 vcc, %[odd]\n\t"
                 "v_cndmask_b32_dpp %[n1], %[p0], %[p1], vcc quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
                 "v_cndmask_b32_dpp %[n3], %[p2], %[p3], vcc quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
                 "s_mov_b64 vcc, %[even]\n\t"
                 "v_cndmask_b32_dpp %[n0], %[p1], %[p0], vcc quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
                 "v_cndmask_b32_dpp %[n2], %[p3], %[p2], vcc quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
                 "s_mov_b64 vcc, %[upper]\n\t"
                 "v_cndmask_b32_dpp %[r3], %[n1], %[n3], vcc quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
                 "v_cndmask_b32_dpp %[r2], %[n0], %[n2], vcc quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
                 "s_mov_b64 vcc, %[lower]\n\t"
                 "v_cndmask_b32_dpp %[r1], %[n3], %[n1], vcc quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
                 "v_cndmask_b32_dpp %[r0], %[n2], %[n0], vcc quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf"
                 : [n0] "=&v"(n0), [n1] "=&v"(n1), [n2] "=&v"(n2), [n3] "=&v"(n3), [r0] "=&v"(r0), [r1] "=&v"(r1),
                   [r2] "=&v"(r2), [r3] "=&v"(r3)
                 : [p0] "v"(p0), [p1] "v"(p1), [p2] "v"(p2), [p3] "v"(p3), [odd] "s"(m.odd), [even] "s"(m.even),
                   [upper] "s"(m.upper), [lower] "s"(m.lower)
                 : "vcc");
    p0 = r0;
    p1 = r1;
    p2 = r2;
    p3 = r3;
}

// Two neighbouring 32x32 blocks of an MFMA result, packed to bf16 pairs (word 2q+h of lane
// (row, lh): columns 8q + 4lh + 2h, +1 of the block), regrouped for whole-line stores: on return
// {A[2u], A[2u+1], B[2u], B[2u+1]} of lane (row, lh) are columns 32lh + 8(row % 4) .. +7 of the
// block pair's 64 columns in row 4 * (row / 4) + u.
__device__ __forceinline__ void block_pair_to_lines(uint32_t (&A)[8], uint32_t (&B)[8])
{
    const QuadMasks m = quad_masks();
#pragma unroll
    for (int w = 0; w < 8; ++w)  // block 2c+1 of the lower half-wave <-> block 2c of the upper one
        asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(A[w]), "+v"(B[w]));
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        quad_transpose(A[d], A[2 + d], A[4 + d], A[6 + d], m);
        quad_transpose(B[d], B[2 + d], B[4 + d], B[6 + d], m);
    }
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

__device__ __forceinline__ void block_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

}  // namespace tweo
