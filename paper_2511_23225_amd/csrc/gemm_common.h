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
