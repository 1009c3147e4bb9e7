// HBM-bound passes of the per-tensor FP8 / INT8 recipes: amax reduction, E4M3
// quantize-cast (with a transposed copy), static INT8 quantize, and the small
// fill / finish kernels around them.  gfx950 only.
#include <hip/hip_ext.h>
#include <atomic>
#include <chrono>
#include "kernels.h"
#include "device_utils.h"

namespace tweo {

// ---------------------------------------------------------------------------
// fill: clears device scalars without a memset node (safe under graph capture).
__global__ void fill_u32_kernel(uint32_t *p, int n, uint32_t v)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        p[i] = v;
}

hipError_t launch_fill_u32(uint32_t *p, int n, uint32_t v, hipStream_t s)
{
    hipLaunchKernelGGL(fill_u32_kernel, dim3((n + 63) / 64), dim3(64), 0, s, p, n, v);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// amax (Sec. 4.3 / Eq. 4): max over the whole tensor of the 15-bit magnitude
// patterns.  2 B/element of HBM reads, nothing else: 16-byte loads, packed 16-bit max, wave shuffle + LDS tree, then one integer
// atomicMax per workgroup on the fp32 bit pattern (positive floats order like
// unsigned integers, so the result is exact and order independent).
// One workgroup of 1024 threads per CU at most: the atomics of concurrently
// finishing workgroups serialise on the one address (measured ~12 ns each; with
// 2048 small workgroups they tripled the time of a 67 MB tensor, with 256 large
// ones the pass runs at the speed of a plain read).
constexpr int kAmaxThreads = 1024;

__device__ __forceinline__ uint32_t pk_absmax(uint32_t m, uint32_t d)
{
    u16x2 a = __builtin_bit_cast(u16x2, m);
    u16x2 b = __builtin_bit_cast(u16x2, d & 0x7FFF7FFFu);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, b));
}

__device__ __forceinline__ uint32_t pk_absmax4(uint32_t m, uint4 v)
{
    m = pk_absmax(m, v.x);
    m = pk_absmax(m, v.y);
    m = pk_absmax(m, v.z);
    return pk_absmax(m, v.w);
}

template <int P>
__device__ __forceinline__ float inject_one(float dy, float a, float inv_tau, float coef, int p)
{
    const float u = __builtin_fabsf(a) * inv_tau;
    float w = 1.0f;
    if constexpr (P == 4) {
        w = u * u * u;
    } else {
        // p is at most 8: a fixed trip count keeps the callers' loops unrollable
#pragma unroll
        for (int e = 1; e < 8; ++e)
            w = e < p ? w * u : w;
    }
    const float t = coef * w;
    // sign(a) = 0 for a = 0; a NaN activation poisons the gradient, as it should
    return dy + (a > 0.0f ? t : (a < 0.0f ? -t : (a == 0.0f ? 0.0f : a)));
}

// The injection as a prologue of the gradient's amax and cast passes: the gradient is formed
// (and rounded to bf16, as the stand-alone kernel stores it) on the way in.
struct InjectArgs {
    const uint16_t *act;  // the penalised activation, same shape as the gradient
    float inv_tau, coef;
    int p;
};

template <int P>  // 4: the paper's power, straight-line; 0: inj.p, any power up to 8
__device__ __forceinline__ uint4 inject_vec(uint4 d, uint4 a, const InjectArgs &inj)
{
    const uint32_t dd[4] = {d.x, d.y, d.z, d.w}, aa[4] = {a.x, a.y, a.z, a.w};
    uint32_t r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        r[k] = pack_bf16x2(inject_one<P>(bf16lo_to_f32(dd[k]), bf16lo_to_f32(aa[k]), inj.inv_tau, inj.coef, inj.p),
                           inject_one<P>(bf16hi_to_f32(dd[k]), bf16hi_to_f32(aa[k]), inj.inv_tau, inj.coef, inj.p));
    return make_uint4(r[0], r[1], r[2], r[3]);
}

// Each workgroup owns one contiguous chunk of the tensor and walks it with
// eight 16-byte loads in flight per lane (measured: ~30 % more bandwidth than a
// grid-stride walk, whose concurrent streams are megabytes apart).
constexpr int kAmaxUnroll = 8;
constexpr int kAmaxMaxPartials = kAmaxPartialsMax;  // workgroups of one amax launch (one per CU)

// PARTIAL: workgroup b stores its maximum to out[b] (no atomic, nothing to clear beforehand);
// the consumer takes the maximum over the workgroups (quantize kernels below).
template <bool PARTIAL = false>
__device__ __forceinline__ void amax_body(const uint4 *__restrict__ x, int64_t n_vec, int64_t per_block,
                                          int block, const uint16_t *__restrict__ tail, int n_tail,
                                          uint32_t *out)
{
    __shared__ uint32_t red[kAmaxThreads / kWave];
    const int64_t b0 = (int64_t)block * per_block;
    const int64_t b1 = b0 + per_block < n_vec ? b0 + per_block : n_vec;
    int64_t i = b0 + threadIdx.x;
    uint32_t m = 0;
    for (; i + (kAmaxUnroll - 1) * kAmaxThreads < b1; i += kAmaxUnroll * kAmaxThreads) {
        uint4 v[kAmaxUnroll];
#pragma unroll
        for (int u = 0; u < kAmaxUnroll; ++u)
            v[u] = x[i + u * kAmaxThreads];
#pragma unroll
        for (int u = 0; u < kAmaxUnroll; ++u)
            m = pk_absmax4(m, v[u]);
    }
    for (; i < b1; i += kAmaxThreads)
        m = pk_absmax4(m, x[i]);
    if (block == 0 && (int)threadIdx.x < n_tail)
        m = pk_absmax(m, tail[threadIdx.x]);
    uint32_t r = (m & 0xFFFFu) > (m >> 16) ? (m & 0xFFFFu) : (m >> 16);
    r = wave_reduce_max_u32(r);
    if ((threadIdx.x & (kWave - 1)) == 0)
        red[threadIdx.x / kWave] = r;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kAmaxThreads / kWave; ++w)
            r = red[w] > r ? red[w] : r;
        // bf16 magnitude widened to the fp32 pattern.  The result only grows, so a workgroup
        // whose maximum is already covered skips the atomic (they serialise on one address).
        const uint32_t mine = r << 16;
        if constexpr (PARTIAL) {
            out[block] = mine;
        } else {
            if (mine > __atomic_load_n(out, __ATOMIC_RELAXED))
                atomicMax(out, mine);
        }
    }
}

template <bool PARTIAL>
__global__ __launch_bounds__(kAmaxThreads) void amax_kernel(const uint4 *__restrict__ x,
                                                            int64_t n_vec, int64_t per_block,
                                                            const uint16_t *__restrict__ tail,
                                                            int n_tail, uint32_t *out)
{
    amax_body<PARTIAL>(x, n_vec, per_block, (int)blockIdx.x, tail, n_tail, out);
}

// Two tensors in one launch (the activation and the weight of a linear layer): workgroups
// [0, blocks0) reduce the first, the rest the second.  Element counts are multiples of 8.
template <bool PARTIAL>
__global__ __launch_bounds__(kAmaxThreads) void amax2_kernel(const uint4 *__restrict__ x0, int64_t n_vec0,
                                                             int64_t per_block0, int blocks0, uint32_t *out0,
                                                             const uint4 *__restrict__ x1, int64_t n_vec1,
                                                             int64_t per_block1, uint32_t *out1)
{
    if ((int)blockIdx.x < blocks0)
        amax_body<PARTIAL>(x0, n_vec0, per_block0, (int)blockIdx.x, nullptr, 0, out0);
    else
        amax_body<PARTIAL>(x1, n_vec1, per_block1, (int)blockIdx.x - blocks0, nullptr, 0, out1);
}

// amax of the gradient with the penalty gradient added on the way in (one maximum per workgroup)
template <int P>
__global__ __launch_bounds__(kAmaxThreads) void amax_inject_kernel(const uint4 *__restrict__ dy, InjectArgs inj,
                                                                   int64_t n_vec, int64_t per_block,
                                                                   uint32_t *__restrict__ partials)
{
    __shared__ uint32_t red[kAmaxThreads / kWave];
    const uint4 *act = (const uint4 *)inj.act;
    const int64_t b0 = (int64_t)blockIdx.x * per_block;
    const int64_t b1 = b0 + per_block < n_vec ? b0 + per_block : n_vec;
    uint32_t m = 0;
    constexpr int UNROLL = 4;  // eight 16-byte loads in flight per lane, as in the plain amax
    int64_t i = b0 + threadIdx.x;
    for (; i + (UNROLL - 1) * kAmaxThreads < b1; i += UNROLL * kAmaxThreads) {
        uint4 d[UNROLL], a[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            d[u] = dy[i + u * kAmaxThreads];
            a[u] = act[i + u * kAmaxThreads];
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            m = pk_absmax4(m, inject_vec<P>(d[u], a[u], inj));
    }
    for (; i < b1; i += kAmaxThreads)
        m = pk_absmax4(m, inject_vec<P>(dy[i], act[i], inj));
    uint32_t r = (m & 0xFFFFu) > (m >> 16) ? (m & 0xFFFFu) : (m >> 16);
    r = wave_reduce_max_u32(r);
    if ((threadIdx.x & (kWave - 1)) == 0)
        red[threadIdx.x / kWave] = r;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kAmaxThreads / kWave; ++w)
            r = red[w] > r ? red[w] : r;
        partials[blockIdx.x] = r << 16;
    }
}

static int amax_cus()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            cus = v;
        else
            cus = 256;
        if (cus > kAmaxMaxPartials)
            cus = kAmaxMaxPartials;
    }
    return cus;
}

static hipError_t launch_amax2_impl(const void *x0_bf16, int64_t n0, float *amax0_zeroed, const void *x1_bf16,
                                    int64_t n1, float *amax1_zeroed, bool partial, int *blocks0, int *blocks1,
                                    hipStream_t s)
{
    // the workgroups of one wave over the CUs are shared out in proportion to the tensor sizes
    const int cus = amax_cus();
    const int64_t v0 = n0 / 8, v1 = n1 / 8;
    const int64_t chunk = kAmaxUnroll * kAmaxThreads;
    int64_t b1 = (int64_t)((double)cus * (double)v1 / (double)(v0 + v1) + 0.5);
    if (b1 < 1)
        b1 = 1;
    if (b1 > cus - 1)
        b1 = cus - 1;
    int64_t b0 = cus - b1;
    if (b0 > (v0 + chunk - 1) / chunk)
        b0 = (v0 + chunk - 1) / chunk;
    if (b1 > (v1 + chunk - 1) / chunk)
        b1 = (v1 + chunk - 1) / chunk;
    if (partial)
        hipLaunchKernelGGL(amax2_kernel<true>, dim3((unsigned)(b0 + b1)), dim3(kAmaxThreads), 0, s,
                           (const uint4 *)x0_bf16, v0, (v0 + b0 - 1) / b0, (int)b0, (uint32_t *)amax0_zeroed,
                           (const uint4 *)x1_bf16, v1, (v1 + b1 - 1) / b1, (uint32_t *)amax1_zeroed);
    else
        hipLaunchKernelGGL(amax2_kernel<false>, dim3((unsigned)(b0 + b1)), dim3(kAmaxThreads), 0, s,
                           (const uint4 *)x0_bf16, v0, (v0 + b0 - 1) / b0, (int)b0, (uint32_t *)amax0_zeroed,
                           (const uint4 *)x1_bf16, v1, (v1 + b1 - 1) / b1, (uint32_t *)amax1_zeroed);
    if (blocks0)
        *blocks0 = (int)b0;
    if (blocks1)
        *blocks1 = (int)b1;
    return hipGetLastError();
}

hipError_t launch_amax2(const void *x0_bf16, int64_t n0, float *amax0_zeroed, const void *x1_bf16, int64_t n1,
                        float *amax1_zeroed, hipStream_t s)
{
    return launch_amax2_impl(x0_bf16, n0, amax0_zeroed, x1_bf16, n1, amax1_zeroed, false, nullptr, nullptr, s);
}

// One maximum per workgroup into partials0[0 .. *blocks0) and partials1[0 .. *blocks1) (each at most
// kAmaxMaxPartials): nothing to clear, no atomics.
hipError_t launch_amax2_partials(const void *x0_bf16, int64_t n0, uint32_t *partials0, int *blocks0,
                                 const void *x1_bf16, int64_t n1, uint32_t *partials1, int *blocks1, hipStream_t s)
{
    return launch_amax2_impl(x0_bf16, n0, (float *)partials0, x1_bf16, n1, (float *)partials1, true, blocks0,
                             blocks1, s);
}

static hipError_t launch_amax_impl(const void *x_bf16, int64_t n, float *amax_zeroed, bool partial, int *blocks_out,
                                   hipStream_t s)
{
    const int64_t n_vec = n / 8;
    const int n_tail = (int)(n % 8);
    // chunks of at least 128 KB (one unrolled trip), at most one workgroup per CU
    const int cus = amax_cus();
    int64_t blocks = n_vec / (kAmaxUnroll * kAmaxThreads);
    if (blocks < 1)
        blocks = 1;
    if (blocks > cus)
        blocks = cus;
    const int64_t per_block = (n_vec + blocks - 1) / blocks;
    if (partial)
        hipLaunchKernelGGL(amax_kernel<true>, dim3((unsigned)blocks), dim3(kAmaxThreads), 0, s,
                           (const uint4 *)x_bf16, n_vec, per_block, (const uint16_t *)x_bf16 + n_vec * 8, n_tail,
                           (uint32_t *)amax_zeroed);
    else {
        // the stand-alone reduction is also a measurement kernel (a pure read of n elements): it
        // takes an armed pair of profile events like the GEMM kernels do
        hipEvent_t e0, e1;
        if (take_profile_events(&e0, &e1))
            hipExtLaunchKernelGGL(amax_kernel<false>, dim3((unsigned)blocks), dim3(kAmaxThreads), 0, s, e0, e1, 0,
                                  (const uint4 *)x_bf16, n_vec, per_block, (const uint16_t *)x_bf16 + n_vec * 8, n_tail,
                                  (uint32_t *)amax_zeroed);
        else
            hipLaunchKernelGGL(amax_kernel<false>, dim3((unsigned)blocks), dim3(kAmaxThreads), 0, s,
                               (const uint4 *)x_bf16, n_vec, per_block, (const uint16_t *)x_bf16 + n_vec * 8, n_tail,
                               (uint32_t *)amax_zeroed);
    }
    if (blocks_out)
        *blocks_out = (int)blocks;
    return hipGetLastError();
}

hipError_t launch_amax(const void *x_bf16, int64_t n, float *amax_zeroed, hipStream_t s)
{
    return launch_amax_impl(x_bf16, n, amax_zeroed, false, nullptr, s);
}

hipError_t launch_amax_partials(const void *x_bf16, int64_t n, uint32_t *partials, int *blocks, hipStream_t s)
{
    return launch_amax_impl(x_bf16, n, (float *)partials, true, blocks, s);
}

// ---------------------------------------------------------------------------
// E4M3 quantize-cast (Sec. 4.3): q = e4m3(fp32(x) * scale), scale = 448/amax
// derived on the device from the amax scalar.  Rounding is the hardware's
// round-to-nearest-even conversion; saturation at +-448 (Sec. 1) is applied in
// front of it so that the result does not depend on the conversion's overflow
// behaviour, and NaN is routed around the clamp.
//
// Each lane owns an 8x8 block of elements: eight 16-byte loads (one per row),
// eight 8-byte stores of q, and - after an in-register 8x8 byte transpose with
// v_perm_b32 - eight 8-byte stores of qT.  A wave is 8x8 lanes = 64x64
// elements, so loads are 128 B contiguous per row and both outputs are written
// in 64 B contiguous pieces.  No LDS, no barriers.
// 3 B/element of HBM traffic without qT, 4 B/element with it.
constexpr int kQuantThreads = 256;
constexpr int kQuantTileRows = 64;
constexpr int kQuantTileCols = 256;

__device__ __forceinline__ float sat_e4m3(float v)
{
    float c = __builtin_amdgcn_fmed3f(v, -448.0f, 448.0f);
    return v != v ? v : c;
}

__device__ __forceinline__ uint32_t cvt4_e4m3(float a, float b, float c, float d)
{
    int r = __builtin_amdgcn_cvt_pk_fp8_f32(sat_e4m3(a), sat_e4m3(b), 0, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(sat_e4m3(c), sat_e4m3(d), r, true);
    return (uint32_t)r;
}

// E5M2, the gradient format of the HYBRID recipe (Sec. 4.3): same cast with the range +-57344.
__device__ __forceinline__ float sat_e5m2(float v)
{
    float c = __builtin_amdgcn_fmed3f(v, -57344.0f, 57344.0f);
    return v != v ? v : c;
}

__device__ __forceinline__ uint32_t cvt4_e5m2(float a, float b, float c, float d)
{
    int r = __builtin_amdgcn_cvt_pk_bf8_f32(sat_e5m2(a), sat_e5m2(b), 0, false);
    r = __builtin_amdgcn_cvt_pk_bf8_f32(sat_e5m2(c), sat_e5m2(d), r, true);
    return (uint32_t)r;
}

template <bool E5M2>
__device__ __forceinline__ uint32_t cvt4_f8(float a, float b, float c, float d)
{
    if constexpr (E5M2)
        return cvt4_e5m2(a, b, c, d);
    else
        return cvt4_e4m3(a, b, c, d);
}

template <bool E5M2>
__device__ __forceinline__ float scale_f8(float amax)
{
    return scale_from_amax_range(amax, E5M2 ? 57344.0f : 448.0f);
}

// rows a,b,c,d (one dword = 4 bytes each) -> columns t0..t3 of the 4x4 byte matrix
__device__ __forceinline__ void transpose4x4_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d,
                                                   uint32_t &t0, uint32_t &t1, uint32_t &t2,
                                                   uint32_t &t3)
{
    uint32_t p0 = __builtin_amdgcn_perm(b, a, 0x05010400u);  // a0 b0 a1 b1
    uint32_t p1 = __builtin_amdgcn_perm(b, a, 0x07030602u);  // a2 b2 a3 b3
    uint32_t p2 = __builtin_amdgcn_perm(d, c, 0x05010400u);  // c0 d0 c1 d1
    uint32_t p3 = __builtin_amdgcn_perm(d, c, 0x07030602u);  // c2 d2 c3 d3
    t0 = __builtin_amdgcn_perm(p2, p0, 0x05040100u);         // a0 b0 c0 d0
    t1 = __builtin_amdgcn_perm(p2, p0, 0x07060302u);         // a1 b1 c1 d1
    t2 = __builtin_amdgcn_perm(p3, p1, 0x05040100u);         // a2 b2 c2 d2
    t3 = __builtin_amdgcn_perm(p3, p1, 0x07060302u);         // a3 b3 c3 d3
}

// Delayed scaling (Sec. 4.3: the recipe the paper trained with) hands the cast a scale that was
// fixed before this tensor was seen and wants this tensor's amax back for the history: DELAYED
// kernels read the scale itself from `amax`, and add the maximum magnitude pattern of what they
// load to *amax_acc (one atomicMax per workgroup, skipped when already covered).
__device__ __forceinline__ void quant_amax_commit(uint32_t m, uint32_t *amax_acc, bool atomic = true)
{
    __shared__ uint32_t red[kQuantThreads / kWave];
    uint32_t r = (m & 0xFFFFu) > (m >> 16) ? (m & 0xFFFFu) : (m >> 16);
    r = wave_reduce_max_u32(r);
    if ((threadIdx.x & (kWave - 1)) == 0)
        red[threadIdx.x / kWave] = r;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kQuantThreads / kWave; ++w)
            r = red[w] > r ? red[w] : r;
        const uint32_t mine = r << 16;
        if (!atomic)
            *amax_acc = mine;  // a slot of this workgroup's own
        else if (mine > __atomic_load_n(amax_acc, __ATOMIC_RELAXED))
            atomicMax(amax_acc, mine);
    }
}

template <bool WITH_T, bool DELAYED, bool E5M2 = false>
__global__ __launch_bounds__(kQuantThreads) void quantize_e4m3_kernel(
    const uint16_t *__restrict__ x, int64_t rows, int64_t cols, int64_t tiles_x,
    const float *__restrict__ amax, uint8_t *__restrict__ q, uint8_t *__restrict__ qT,
    float *scale_out, float *scale_inv_out, uint32_t *amax_acc)
{
    const float scale = DELAYED ? *amax : scale_f8<E5M2>(*amax);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (scale_out)
            *scale_out = scale;
        if (scale_inv_out)
            *scale_inv_out = 1.0f / scale;
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t by = blockIdx.x / tiles_x, bx = blockIdx.x % tiles_x;
    const int64_t r0 = by * kQuantTileRows + (lane >> 3) * 8;
    const int64_t c0 = bx * kQuantTileCols + wave * 64 + (lane & 7) * 8;
    // lanes outside the tensor load nothing and store nothing, but every lane reaches the one
    // workgroup barrier of the amax commit
    const bool active = c0 < cols && r0 < rows;
    uint4 in[8];
    uint32_t mx = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        in[i] = make_uint4(0, 0, 0, 0);
        if (active && r0 + i < rows)
            in[i] = *(const uint4 *)(x + (r0 + i) * cols + c0);
        if constexpr (DELAYED)
            mx = pk_absmax4(mx, in[i]);
    }
    if constexpr (DELAYED)
        if (amax_acc != nullptr)  // uniform over the grid
            quant_amax_commit(mx, amax_acc);
    if (!active)
        return;
    uint32_t lo[8], hi[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        lo[i] = cvt4_f8<E5M2>(bf16lo_to_f32(in[i].x) * scale, bf16hi_to_f32(in[i].x) * scale,
                          bf16lo_to_f32(in[i].y) * scale, bf16hi_to_f32(in[i].y) * scale);
        hi[i] = cvt4_f8<E5M2>(bf16lo_to_f32(in[i].z) * scale, bf16hi_to_f32(in[i].z) * scale,
                          bf16lo_to_f32(in[i].w) * scale, bf16hi_to_f32(in[i].w) * scale);
        if (r0 + i < rows)
            *(uint2 *)(q + (r0 + i) * cols + c0) = make_uint2(lo[i], hi[i]);
    }
    if (WITH_T) {
        // T[j] = column j of the 8x8 block = bytes (row0..row7)
        uint32_t ta[8], tb[8];  // ta: rows 0-3, tb: rows 4-7
        transpose4x4_bytes(lo[0], lo[1], lo[2], lo[3], ta[0], ta[1], ta[2], ta[3]);
        transpose4x4_bytes(hi[0], hi[1], hi[2], hi[3], ta[4], ta[5], ta[6], ta[7]);
        transpose4x4_bytes(lo[4], lo[5], lo[6], lo[7], tb[0], tb[1], tb[2], tb[3]);
        transpose4x4_bytes(hi[4], hi[5], hi[6], hi[7], tb[4], tb[5], tb[6], tb[7]);
        const bool full = (r0 + 8 <= rows) && ((rows & 7) == 0);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint8_t *dst = qT + (c0 + j) * rows + r0;
            if (full) {
                *(uint2 *)dst = make_uint2(ta[j], tb[j]);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (r0 + i < rows)
                        dst[i] = (uint8_t)((i < 4 ? ta[j] >> (8 * i) : tb[j] >> (8 * (i - 4))) & 0xFF);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// LayerNorm in front of the cast (Sec. 4.3: the LayerNorm components run under FP8 with the linear
// layers, i.e. the normalised activation is what the next linear's per-tensor cast consumes).
// Textbook row-wise normalisation, biased variance; the value is rounded ONCE to bf16 (the stored
// activation) and that bf16 value is what amax and the FP8 rounding see.  The arithmetic is fp64:
// its instructions issue at the rate of fp32 ones on this chip and the passes are bound by memory,
// so the stored bits do not depend on the summation order to any extent a test could see.
struct LnArgs {
    const double *stats;           // per row: mean, 1 / sqrt(var + eps)
    const uint16_t *gamma, *beta;  // bf16 [cols]; beta may be nullptr
};

// fp64 -> fp32 such that rounding the result to bf16 (round to nearest even) is the single correct
// rounding of the fp64 value: the 29 mantissa bits that fp32 cannot hold are cut off and, if any
// was set, the last bit that fp32 does hold is set ("round to odd"); the conversion is then exact,
// and a value rounded to odd at 24 bits rounds to 8 bits like the original.  (Below the smallest
// normal fp32, 1.2e-38, the conversion itself rounds again; a normalised activation is either an
// exact zero or many orders of magnitude above that.)
__device__ __forceinline__ float f64_to_f32_for_bf16(double v)
{
    uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)b, cut = lo & 0x1FFFFFFFu;
    const uint32_t lo2 = (lo & 0xE0000000u) | ((cut + 0x1FFFFFFFu) & 0x20000000u);
    b = (b & 0xFFFFFFFF00000000ull) | lo2;
    return (float)__builtin_bit_cast(double, b);
}

// eight elements of a row: y = (x - mean) * (rstd * gamma) + beta in fp64 (one rounding more or
// less than the textbook order of operations: 1e-16 relative, far below anything a bf16 rounding
// sees), as packed bf16 pairs.  g64 / b64: the eight columns' parameters, widened by the caller.
__device__ __forceinline__ uint4 ln_vec(uint4 x, double mean, double rstd, const double (&g64)[8], const double (&b64)[8],
                                        bool has_beta)
{
    const uint32_t xx[4] = {x.x, x.y, x.z, x.w};
    uint32_t r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const double d0 = (double)bf16lo_to_f32(xx[k]) - mean, d1 = (double)bf16hi_to_f32(xx[k]) - mean;
        const double a0 = rstd * g64[2 * k], a1 = rstd * g64[2 * k + 1];
        // without a beta nothing is added, so that a zero keeps the sign the product gives it
        const double y0 = has_beta ? __builtin_fma(d0, a0, b64[2 * k]) : d0 * a0;
        const double y1 = has_beta ? __builtin_fma(d1, a1, b64[2 * k + 1]) : d1 * a1;
        r[k] = pack_bf16x2(f64_to_f32_for_bf16(y0), f64_to_f32_for_bf16(y1));
    }
    return make_uint4(r[0], r[1], r[2], r[3]);
}

__device__ __forceinline__ void widen8(uint4 v, double (&out)[8])
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        out[2 * k] = (double)bf16lo_to_f32(w[k]);
        out[2 * k + 1] = (double)bf16hi_to_f32(w[k]);
    }
}

// h = bf16(x + r) on eight elements: the fp32 sum of two bf16 values rounded to bf16 equals the
// exact sum rounded once (the fp32 sum is exact unless the smaller term lies below the bf16
// rounding position of the larger one by more than fp32 can hold, and then it decides nothing)
__device__ __forceinline__ uint4 add_bf16x8(uint4 a, uint4 b)
{
    const uint32_t aa[4] = {a.x, a.y, a.z, a.w}, bb[4] = {b.x, b.y, b.z, b.w};
    uint32_t r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        r[k] = pack_bf16x2(bf16lo_to_f32(aa[k]) + bf16lo_to_f32(bb[k]), bf16hi_to_f32(aa[k]) + bf16hi_to_f32(bb[k]));
    return make_uint4(r[0], r[1], r[2], r[3]);
}

__device__ __forceinline__ double sum8_f64(uint4 v)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
        s += (double)bf16lo_to_f32(w[k]) + (double)bf16hi_to_f32(w[k]);
    return s;
}

__device__ __forceinline__ double sumsq8_f64(uint4 v, double mean)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const double d0 = (double)bf16lo_to_f32(w[k]) - mean, d1 = (double)bf16hi_to_f32(w[k]) - mean;
        s += d0 * d0 + d1 * d1;
    }
    return s;
}

// Row statistics: one wave per row, the first kLnCached 16-byte pieces of every lane stay in
// registers between the mean and the variance, so rows of up to 4096 elements are read from memory
// once (2 B/element).  RESIDUAL: the row is h = bf16(x + r), stored to h_out on the way.
constexpr int kLnThreads = 256;
constexpr int kLnCached = 8;

template <bool RESIDUAL>
__global__ __launch_bounds__(kLnThreads) void ln_stats_kernel(const uint4 *x, const uint4 *res, uint4 *h_out,
                                                              int64_t rows, int vec_per_row, double eps,
                                                              double *__restrict__ stats)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    constexpr int WAVES = kLnThreads / kWave;
    const double n = (double)vec_per_row * 8.0;
    for (int64_t row = (int64_t)blockIdx.x * WAVES + wave; row < rows; row += (int64_t)gridDim.x * WAVES) {
        const uint4 *xr = x + row * vec_per_row;
        const uint4 *rr = RESIDUAL ? res + row * vec_per_row : nullptr;
        uint4 *hr = RESIDUAL ? h_out + row * vec_per_row : nullptr;
        uint4 c[kLnCached];
        double s = 0.0;
#pragma unroll
        for (int u = 0; u < kLnCached; ++u) {
            const int i = lane + u * kWave;
            c[u] = make_uint4(0u, 0u, 0u, 0u);
            if (i < vec_per_row) {
                c[u] = xr[i];
                if constexpr (RESIDUAL) {
                    c[u] = add_bf16x8(c[u], rr[i]);
                    hr[i] = c[u];
                }
                s += sum8_f64(c[u]);
            }
        }
        for (int i = lane + kLnCached * kWave; i < vec_per_row; i += kWave) {
            uint4 v = xr[i];
            if constexpr (RESIDUAL) {
                v = add_bf16x8(v, rr[i]);
                hr[i] = v;
            }
            s += sum8_f64(v);
        }
        const double mean = wave_reduce_sum(s) / n;
        double ss = 0.0;
#pragma unroll
        for (int u = 0; u < kLnCached; ++u)
            if (lane + u * kWave < vec_per_row)
                ss += sumsq8_f64(c[u], mean);
        // h_out may be x or the residual itself (an in-place update of the stream): what this lane
        // stored above is read back, not formed again
        for (int i = lane + kLnCached * kWave; i < vec_per_row; i += kWave)
            ss += sumsq8_f64(RESIDUAL ? hr[i] : xr[i], mean);
        const double var = wave_reduce_sum(ss) / n;
        if (lane == 0) {
            stats[2 * row] = mean;
            stats[2 * row + 1] = 1.0 / __builtin_sqrt(var + eps);
        }
    }
}

// Same cast for shapes with rows % 16 == 0 and cols % 16 == 0: a lane owns a
// 16x16 block (two 16-byte loads per row), so q is written in 16-byte pieces
// that 8 neighbouring lanes join into whole 128-byte lines, and - after sixteen
// 4x4 byte transposes - qT likewise.  A wave covers 128x128 elements, a
// workgroup 256x256.
constexpr int kQuantBigTile = 256;

// INJECT: 0 = plain cast; 4 / 1 = the penalty gradient is added on the way in (p = 4 / any p)
// LN: the tensor that is cast is the LayerNorm of x (statistics precomputed per row).  AMAX_ONLY
// (with DELAYED's bounded grid and tile loop): nothing is stored, workgroup b leaves the maximum
// magnitude pattern of what it would have cast in amax_acc[b].
// T_LATER: the transposed codes are not read before a later call (a forward cast's, which wait for
// the backward pass): streaming stores.
template <bool WITH_T, bool DELAYED, bool E5M2 = false, int INJECT = 0, bool LN = false, bool AMAX_ONLY = false,
          bool T_LATER = false>
__device__ __forceinline__ void quantize_e4m3_16x16_body(
    const uint16_t *__restrict__ x, int64_t rows, int64_t cols, int64_t tiles_x,
    const float *__restrict__ amax, uint8_t *__restrict__ q, uint8_t *__restrict__ qT,
    float *scale_out, float *scale_inv_out, uint32_t *amax_acc, int64_t block, int64_t n_blocks,
    const uint32_t *__restrict__ amax_partials = nullptr, int n_partials = 0, float *amax_store = nullptr,
    InjectArgs inj = InjectArgs{}, LnArgs ln = LnArgs{}, uint16_t *__restrict__ y_out = nullptr)
{
    static_assert(!AMAX_ONLY || DELAYED, "the amax-only pass walks the tiles with a bounded grid");
    float amax_v = 0.0f;
    if constexpr (AMAX_ONLY) {
        // no scale needed
    } else if (amax_partials != nullptr) {  // uniform: the maxima of the amax launch's workgroups
        __shared__ uint32_t pred[kQuantThreads / kWave];
        uint32_t m = 0;
        for (int i = threadIdx.x; i < n_partials; i += kQuantThreads) {
            const uint32_t v = amax_partials[i];
            m = v > m ? v : m;
        }
        m = wave_reduce_max_u32(m);
        if ((threadIdx.x & (kWave - 1)) == 0)
            pred[threadIdx.x / kWave] = m;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < kQuantThreads / kWave; ++w)
            m = pred[w] > m ? pred[w] : m;
        amax_v = __uint_as_float(m);
        if (block == 0 && threadIdx.x == 0)
            *amax_store = amax_v;
    } else {
        amax_v = *amax;
    }
    const float scale = DELAYED ? amax_v : scale_f8<E5M2>(amax_v);
    if (!AMAX_ONLY && block == 0 && threadIdx.x == 0) {
        if (scale_out)
            *scale_out = scale;
        if (scale_inv_out)
            *scale_inv_out = 1.0f / scale;
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    uint32_t mx = 0;
    // DELAYED: a bounded grid walks the tiles (its one atomic per workgroup is then a few hundred
    // per tensor, not thousands); otherwise one tile per workgroup
    const int64_t n_tiles = DELAYED ? tiles_x * ((rows + kQuantBigTile - 1) / kQuantBigTile) : block + 1;
    for (int64_t tile = block; tile < n_tiles; tile += n_blocks) {
    const int64_t by = tile / tiles_x, bx = tile % tiles_x;
    const int64_t r0 = by * kQuantBigTile + (wave >> 1) * 128 + (lane >> 3) * 16;
    const int64_t c0 = bx * kQuantBigTile + (wave & 1) * 128 + (lane & 7) * 16;
    if (c0 >= cols || r0 >= rows)  // whole 16x16 blocks: in or out
        continue;
    uint32_t qd[16][4];
    uint4 lg[2], lb[2];  // LN: gamma and beta of the lane's 16 columns
    if constexpr (LN) {
        lg[0] = ((const uint4 *)(ln.gamma + c0))[0];
        lg[1] = ((const uint4 *)(ln.gamma + c0))[1];
        lb[0] = lb[1] = make_uint4(0u, 0u, 0u, 0u);
        if (ln.beta != nullptr) {
            lb[0] = ((const uint4 *)(ln.beta + c0))[0];
            lb[1] = ((const uint4 *)(ln.beta + c0))[1];
        }
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        uint4 in[8][2];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint4 *src = (const uint4 *)(x + (r0 + half * 8 + i) * cols + c0);
            in[i][0] = src[0];
            in[i][1] = src[1];
            if constexpr (INJECT != 0) {
                const uint4 *asrc = (const uint4 *)(inj.act + (r0 + half * 8 + i) * cols + c0);
                in[i][0] = inject_vec<(INJECT == 4 ? 4 : 0)>(in[i][0], asrc[0], inj);
                in[i][1] = inject_vec<(INJECT == 4 ? 4 : 0)>(in[i][1], asrc[1], inj);
            }
            if constexpr (DELAYED && !LN)
                mx = pk_absmax4(pk_absmax4(mx, in[i][0]), in[i][1]);
        }
        if constexpr (LN) {
            // normalise what was loaded, eight columns at a time (their widened parameters live
            // only that long)
#pragma unroll
            for (int w = 0; w < 2; ++w) {
                double g64[8], b64[8];
                widen8(lg[w], g64);
                widen8(lb[w], b64);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const double2 st = *(const double2 *)(ln.stats + 2 * (r0 + half * 8 + i));
                    in[i][w] = ln_vec(in[i][w], st.x, st.y, g64, b64, ln.beta != nullptr);
                    if constexpr (DELAYED)
                        mx = pk_absmax4(mx, in[i][w]);
                }
            }
            if (!AMAX_ONLY && y_out != nullptr) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    uint4 *dst = (uint4 *)(y_out + (r0 + half * 8 + i) * cols + c0);
                    dst[0] = in[i][0];
                    dst[1] = in[i][1];
                }
            }
        }
        if constexpr (AMAX_ONLY)
            continue;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = half * 8 + i;
#pragma unroll
            for (int w = 0; w < 2; ++w) {
                const uint4 v = in[i][w];
                qd[r][2 * w] = cvt4_f8<E5M2>(bf16lo_to_f32(v.x) * scale, bf16hi_to_f32(v.x) * scale,
                                         bf16lo_to_f32(v.y) * scale, bf16hi_to_f32(v.y) * scale);
                qd[r][2 * w + 1] = cvt4_f8<E5M2>(bf16lo_to_f32(v.z) * scale, bf16hi_to_f32(v.z) * scale,
                                             bf16lo_to_f32(v.w) * scale, bf16hi_to_f32(v.w) * scale);
            }
            *(uint4 *)(q + (r0 + r) * cols + c0) = make_uint4(qd[r][0], qd[r][1], qd[r][2], qd[r][3]);
        }
    }
    if (WITH_T && !AMAX_ONLY) {
#pragma unroll
        for (int C = 0; C < 4; ++C) {
            uint32_t t[4][4];  // t[R][k]: column 4C+k, rows 4R..4R+3
#pragma unroll
            for (int R = 0; R < 4; ++R)
                transpose4x4_bytes(qd[4 * R][C], qd[4 * R + 1][C], qd[4 * R + 2][C], qd[4 * R + 3][C],
                                   t[R][0], t[R][1], t[R][2], t[R][3]);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                typedef uint32_t v4u __attribute__((ext_vector_type(4)));
                v4u *dst = (v4u *)(qT + (c0 + 4 * C + k) * rows + r0);
                const v4u v = {t[0][k], t[1][k], t[2][k], t[3][k]};
                if constexpr (T_LATER)
                    __builtin_nontemporal_store(v, dst);
                else
                    *dst = v;
            }
        }
    }
    }
    // every lane reaches the one workgroup barrier of the amax commit (amax_acc is uniform over
    // the grid; nullptr = the caller already has this tensor's amax)
    if constexpr (AMAX_ONLY)
        quant_amax_commit(mx, amax_acc + block, false);
    else if constexpr (DELAYED)
        if (amax_acc != nullptr)
            quant_amax_commit(mx, amax_acc);
}

// LayerNorm + cast (DELAYED: the scale is read from *amax, the tensor's amax goes to *amax_acc), or
// the amax-only pass over the normalised tensor (one maximum per workgroup into amax_acc[])
template <bool WITH_T, bool DELAYED, bool AMAX_ONLY>
__global__ __launch_bounds__(kQuantThreads) void quantize_ln_16x16_kernel(
    const uint16_t *__restrict__ x, LnArgs ln, int64_t rows, int64_t cols, int64_t tiles_x,
    const float *__restrict__ amax, uint8_t *__restrict__ q, uint8_t *__restrict__ qT, uint16_t *__restrict__ y_out,
    float *scale_out, float *scale_inv_out, uint32_t *amax_acc, const uint32_t *__restrict__ amax_partials,
    int n_partials, float *amax_store)
{
    quantize_e4m3_16x16_body<WITH_T, DELAYED, false, 0, true, AMAX_ONLY>(
        x, rows, cols, tiles_x, amax, q, qT, scale_out, scale_inv_out, amax_acc, blockIdx.x, gridDim.x, amax_partials,
        n_partials, amax_store, InjectArgs{}, ln, y_out);
}

template <bool WITH_T, bool DELAYED, bool E5M2 = false>
__global__ __launch_bounds__(kQuantThreads) void quantize_e4m3_16x16_kernel(
    const uint16_t *__restrict__ x, int64_t rows, int64_t cols, int64_t tiles_x,
    const float *__restrict__ amax, uint8_t *__restrict__ q, uint8_t *__restrict__ qT,
    float *scale_out, float *scale_inv_out, uint32_t *amax_acc, const uint32_t *__restrict__ amax_partials,
    int n_partials, float *amax_store)
{
    quantize_e4m3_16x16_body<WITH_T, DELAYED, E5M2>(x, rows, cols, tiles_x, amax, q, qT, scale_out, scale_inv_out,
                                              amax_acc, blockIdx.x, gridDim.x, amax_partials, n_partials,
                                              amax_store);
}

template <bool E5M2, int INJECT>
__global__ __launch_bounds__(kQuantThreads) void quantize_inject_16x16_kernel(
    const uint16_t *__restrict__ dy, InjectArgs inj, int64_t rows, int64_t cols, int64_t tiles_x,
    uint8_t *__restrict__ q, uint8_t *__restrict__ qT, float *scale_out, float *scale_inv_out,
    const uint32_t *__restrict__ amax_partials, int n_partials, float *amax_store)
{
    quantize_e4m3_16x16_body<true, false, E5M2, INJECT>(dy, rows, cols, tiles_x, amax_store, q, qT, scale_out,
                                                      scale_inv_out, nullptr, blockIdx.x, gridDim.x, amax_partials,
                                                      n_partials, amax_store, inj);
}

// Two tensors in one launch (activation and weight of a linear layer, each with its transposed
// copy): workgroups [0, blocks0) cast the first, the rest the second.
struct QuantTensor {
    const uint16_t *x;
    int64_t rows, cols, tiles_x;
    const float *amax;
    uint8_t *q, *qT;
    float *scale_out, *scale_inv_out;
    const uint32_t *amax_partials;  // or nullptr: then *amax is the maximum
    int n_partials;
    float *amax_store;
};

__global__ __launch_bounds__(kQuantThreads) void quantize2_e4m3_16x16_kernel(QuantTensor t0, int64_t blocks0,
                                                                             QuantTensor t1)
{
    const bool first = (int64_t)blockIdx.x < blocks0;
    const QuantTensor &t = first ? t0 : t1;
    quantize_e4m3_16x16_body<true, false, false, 0, false, false, true>(t.x, t.rows, t.cols, t.tiles_x, t.amax, t.q, t.qT, t.scale_out,
                                          t.scale_inv_out, nullptr,
                                          first ? (int64_t)blockIdx.x : (int64_t)blockIdx.x - blocks0, 1,
                                          t.amax_partials, t.n_partials, t.amax_store);
}

hipError_t launch_quantize2_e4m3(const void *x0_bf16, int64_t rows0, int64_t cols0, float *amax0, uint8_t *q0,
                                 uint8_t *q0T, float *scale0, float *scale0_inv, const void *x1_bf16,
                                 int64_t rows1, int64_t cols1, float *amax1, uint8_t *q1, uint8_t *q1T,
                                 float *scale1, float *scale1_inv, hipStream_t s, const uint32_t *partials0,
                                 int n_partials0, const uint32_t *partials1, int n_partials1)
{
    auto tiles = [](int64_t v) { return (v + kQuantBigTile - 1) / kQuantBigTile; };
    QuantTensor t0{(const uint16_t *)x0_bf16, rows0, cols0, tiles(cols0), amax0, q0, q0T, scale0, scale0_inv,
                   partials0, n_partials0, amax0};
    QuantTensor t1{(const uint16_t *)x1_bf16, rows1, cols1, tiles(cols1), amax1, q1, q1T, scale1, scale1_inv,
                   partials1, n_partials1, amax1};
    const int64_t b0 = tiles(rows0) * tiles(cols0), b1 = tiles(rows1) * tiles(cols1);
    hipLaunchKernelGGL(quantize2_e4m3_16x16_kernel, dim3((unsigned)(b0 + b1)), dim3(kQuantThreads), 0, s, t0, b0, t1);
    return hipGetLastError();
}

template <bool DELAYED, bool E5M2 = false>
static hipError_t launch_quantize_e4m3_impl(const void *x_bf16, int64_t rows, int64_t cols, const float *amax,
                                            uint8_t *q, uint8_t *qT, float *scale_out, float *scale_inv_out,
                                            uint32_t *amax_acc, hipStream_t s,
                                            const uint32_t *amax_partials = nullptr, int n_partials = 0,
                                            float *amax_store = nullptr)
{
    const dim3 block(kQuantThreads);
    if (amax_partials != nullptr && (rows % 16 != 0 || cols % 16 != 0))
        return hipErrorInvalidValue;  // only the whole-block kernel reduces partial maxima
    if (rows % 16 == 0 && cols % 16 == 0) {
        const int64_t tiles_x = (cols + kQuantBigTile - 1) / kQuantBigTile;
        const int64_t tiles_y = (rows + kQuantBigTile - 1) / kQuantBigTile;
        int64_t n_wg = tiles_x * tiles_y;
        if (DELAYED && n_wg > 1024)
            n_wg = 1024;
        const dim3 grid((unsigned)n_wg);
        if (qT)
            hipLaunchKernelGGL((quantize_e4m3_16x16_kernel<true, DELAYED, E5M2>), grid, block, 0, s,
                               (const uint16_t *)x_bf16, rows, cols, tiles_x, amax, q, qT, scale_out,
                               scale_inv_out, amax_acc, amax_partials, n_partials, amax_store);
        else
            hipLaunchKernelGGL((quantize_e4m3_16x16_kernel<false, DELAYED, E5M2>), grid, block, 0, s,
                               (const uint16_t *)x_bf16, rows, cols, tiles_x, amax, q, qT, scale_out,
                               scale_inv_out, amax_acc, amax_partials, n_partials, amax_store);
        return hipGetLastError();
    }
    const int64_t tiles_x = (cols + kQuantTileCols - 1) / kQuantTileCols;
    const int64_t tiles_y = (rows + kQuantTileRows - 1) / kQuantTileRows;
    const dim3 grid((unsigned)(tiles_x * tiles_y));
    if (qT)
        hipLaunchKernelGGL((quantize_e4m3_kernel<true, DELAYED, E5M2>), grid, block, 0, s, (const uint16_t *)x_bf16,
                           rows, cols, tiles_x, amax, q, qT, scale_out, scale_inv_out, amax_acc);
    else
        hipLaunchKernelGGL((quantize_e4m3_kernel<false, DELAYED, E5M2>), grid, block, 0, s, (const uint16_t *)x_bf16,
                           rows, cols, tiles_x, amax, q, qT, scale_out, scale_inv_out, amax_acc);
    return hipGetLastError();
}

hipError_t launch_quantize_e4m3(const void *x_bf16, int64_t rows, int64_t cols, const float *amax,
                                uint8_t *q, uint8_t *qT, float *scale_out, float *scale_inv_out,
                                hipStream_t s)
{
    return launch_quantize_e4m3_impl<false>(x_bf16, rows, cols, amax, q, qT, scale_out, scale_inv_out,
                                            nullptr, s);
}

hipError_t launch_quantize_e5m2(const void *x_bf16, int64_t rows, int64_t cols, const float *amax,
                                uint8_t *q, uint8_t *qT, float *scale_out, float *scale_inv_out,
                                hipStream_t s)
{
    return launch_quantize_e4m3_impl<false, true>(x_bf16, rows, cols, amax, q, qT, scale_out,
                                                  scale_inv_out, nullptr, s);
}

// The cast fed by launch_amax_partials: the maximum over `n_partials` workgroup maxima is taken
// by every workgroup of the cast itself and stored to *amax_out.  rows, cols multiples of 16.
hipError_t launch_quantize_f8_from_partials(const void *x_bf16, int64_t rows, int64_t cols,
                                            const uint32_t *amax_partials, int n_partials, bool e5m2,
                                            float *amax_out, uint8_t *q, uint8_t *qT, float *scale_out,
                                            float *scale_inv_out, hipStream_t s)
{
    if (e5m2)
        return launch_quantize_e4m3_impl<false, true>(x_bf16, rows, cols, amax_out, q, qT, scale_out, scale_inv_out,
                                                      nullptr, s, amax_partials, n_partials, amax_out);
    return launch_quantize_e4m3_impl<false, false>(x_bf16, rows, cols, amax_out, q, qT, scale_out, scale_inv_out,
                                                   nullptr, s, amax_partials, n_partials, amax_out);
}

// amax and cast of dy' = bf16(dy + coef * sign(a) * (|a| * inv_tau)^(p-1)) without storing dy':
// the amax launch leaves workgroup maxima, the cast launch reduces them (rows, cols multiples of 16).
hipError_t launch_amax_quantize_inject(const void *dy_bf16, const void *a_bf16, int64_t rows, int64_t cols,
                                       float inv_tau, float coef, int p, bool e5m2, uint32_t *partials,
                                       float *amax_out, uint8_t *q, uint8_t *qT, float *scale_out,
                                       float *scale_inv_out, hipStream_t s)
{
    const InjectArgs inj{(const uint16_t *)a_bf16, inv_tau, coef, p};
    const int64_t n_vec = rows * cols / 8;
    int64_t blocks = n_vec / (kAmaxUnroll * kAmaxThreads);
    if (blocks < 1)
        blocks = 1;
    if (blocks > amax_cus())
        blocks = amax_cus();
    if (p == 4)
        hipLaunchKernelGGL(amax_inject_kernel<4>, dim3((unsigned)blocks), dim3(kAmaxThreads), 0, s,
                           (const uint4 *)dy_bf16, inj, n_vec, (n_vec + blocks - 1) / blocks, partials);
    else
        hipLaunchKernelGGL(amax_inject_kernel<0>, dim3((unsigned)blocks), dim3(kAmaxThreads), 0, s,
                           (const uint4 *)dy_bf16, inj, n_vec, (n_vec + blocks - 1) / blocks, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    const int64_t tiles_x = (cols + kQuantBigTile - 1) / kQuantBigTile, tiles_y = (rows + kQuantBigTile - 1) / kQuantBigTile;
    const dim3 grid((unsigned)(tiles_x * tiles_y)), block(kQuantThreads);
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, block, 0, s, (const uint16_t *)dy_bf16, inj, rows, cols, tiles_x, q, qT,
                           scale_out, scale_inv_out, (const uint32_t *)partials, (int)blocks, amax_out);
    };
    if (e5m2) {
        if (p == 4)
            launch(quantize_inject_16x16_kernel<true, 4>);
        else
            launch(quantize_inject_16x16_kernel<true, 1>);
    } else {
        if (p == 4)
            launch(quantize_inject_16x16_kernel<false, 4>);
        else
            launch(quantize_inject_16x16_kernel<false, 1>);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// amax and cast in ONE launch (current scaling, Sec. 4.3), the tensor held on chip in between.
// Two passes over a tensor move 6 bytes per element (2 read for the amax, 2 read again and 2
// written by the cast), and the second read costs nearly what the first did even when the
// memory-side cache serves it.  Here one workgroup per CU (8 waves, up to 256 registers a lane)
// reads its share of the tensor(s) once, keeps the last two 16x16 blocks of every lane on chip
// (the last one and the lower half of the one before it in registers, the upper half of that one
// in LDS: 512 KB per CU, 128 MB over the chip - a 16384x2048 activation with its weight fits whole,
// a 16384x6144 gradient to two thirds), publishes its maxima, waits until every workgroup has, and
// casts: what it kept straight from registers and LDS, the rest after reading it again, newest
// first.  Reads and writes also fall into separate phases.
//
// The wait is a barrier over the grid, so every workgroup must be resident: the grid is at most one
// workgroup per CU and the kernel needs a CU's registers whole.  Two such launches running at the
// same time on one device (two streams) could each hold a part of the CUs and wait for the rest:
// callers that overlap bf16 entry points on one device switch this path off
// (set_fused_cast(false)).  The wait is bounded: a workgroup that gives up counts itself in
// g_fused_cast_timeouts, publishes a NaN amax (the scalars the caller reads are then NaN, not
// plausibly wrong) and finishes.
//
// Barrier without read-modify-write atomics, fences or cleared memory: workgroup b writes slot b of
// `slots` (16 bytes each, in the caller's workspace) as two 64-bit words, each one of its maxima
// under a 32-bit tag derived from the call's 64-bit token, both tags new in every call; lane i of
// every workgroup polls slot i until both words carry this call's tags.  A word is stored and loaded whole, at device scope, past the
// XCD-private L2, and carries its own validity, so no release or acquire is needed - either would
// write back or invalidate a whole L2 (measured: 15 us per barrier).  Tokens come from a
// process-wide counter, so whatever an earlier call (or nobody) left in the slots is never
// mistaken for this call's.
__device__ uint32_t g_fused_cast_timeouts;

struct FusedTensor {
    const uint16_t *x;
    int64_t rows, cols, tiles_x;  // tiles_x: 256-column tiles per row of tiles
    uint8_t *q, *qT;
    float *amax_store, *scale_out, *scale_inv_out;
};

constexpr int kFusedThreads = 512, kFusedWaves = kFusedThreads / kWave;
constexpr int kFusedSpinLimit = 1 << 18;  // polls of ~0.25 us each
constexpr int kFusedLdsBytes = 8 * 2 * kFusedThreads * 16;  // eight rows of 32 bytes per lane

struct FusedSlot {
    uint64_t w0, w1;  // token half << 32 | magnitude pattern << 16 (as the amax partials elsewhere)
};

// The grid-wide exchange of the two maxima (packed pairs of bf16 magnitude patterns per lane in, the
// tensors' fp32 amax patterns out): see the comment above for the scheme.  WAVES = waves per
// workgroup; the grid has at most WAVES * 64 workgroups (lane i polls slot i).  Every lane of the
// workgroup calls it.
template <int WAVES>
__device__ __forceinline__ void fused_grid_max(uint32_t mx0, uint32_t mx1, FusedSlot *slots, uint64_t token,
                                               uint32_t &all0, uint32_t &all1)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int G = gridDim.x;
    // BOTH words carry a tag that changes with every call (the token's low half, and the high half of
    // its product with an odd constant): a reader that finds this call's first word next to the
    // second word of the call before must not take that one for new.  (Tags that shared the token's
    // high half - the same in every call of a process - let exactly that happen: rarely, a
    // workgroup cast the second tensor with the maximum of an earlier call.)
    const uint64_t tag0 = token & 0xFFFFFFFFull, tag1 = (token * 0x9E3779B97F4A7C15ull) >> 32;
    __shared__ uint32_t red[2][WAVES];
    __shared__ uint32_t all[2];
    auto fold = [](uint32_t m) { return (m & 0xFFFFu) > (m >> 16) ? (m & 0xFFFFu) : (m >> 16); };
    {
        const uint32_t a = wave_reduce_max_u32(fold(mx0)), b = wave_reduce_max_u32(fold(mx1));
        if (lane == 0) {
            red[0][wave] = a;
            red[1][wave] = b;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t a = red[0][0], b = red[1][0];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) {
            a = red[0][w] > a ? red[0][w] : a;
            b = red[1][w] > b ? red[1][w] : b;
        }
        FusedSlot *mine = slots + blockIdx.x;
        __hip_atomic_store(&mine->w0, (tag0 << 32) | (uint64_t)(a << 16), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&mine->w1, (tag1 << 32) | (uint64_t)(b << 16), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    uint32_t a = 0, b = 0;
    if ((int)threadIdx.x < G) {
        const FusedSlot *theirs = slots + threadIdx.x;
        int spins = 0;
        uint64_t w0, w1;
        for (;;) {
            w0 = __hip_atomic_load(&theirs->w0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            w1 = __hip_atomic_load(&theirs->w1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (((w0 >> 32) == tag0 && (w1 >> 32) == tag1) || ++spins > kFusedSpinLimit)
                break;
            __builtin_amdgcn_s_sleep(8);
        }
        if (spins > kFusedSpinLimit) {
            atomicAdd(&g_fused_cast_timeouts, 1u);
            a = b = 0x7FC00000u;  // NaN: above every magnitude pattern
        } else {
            a = (uint32_t)w0;
            b = (uint32_t)w1;
        }
    }
    a = wave_reduce_max_u32(a);
    b = wave_reduce_max_u32(b);
    __syncthreads();  // red[] has been read by thread 0
    if (lane == 0) {
        red[0][wave] = a;
        red[1][wave] = b;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < WAVES; ++w) {
            a = red[0][w] > a ? red[0][w] : a;
            b = red[1][w] > b ? red[1][w] : b;
        }
        all[0] = a;
        all[1] = b;
    }
    __syncthreads();
    all0 = all[0];
    all1 = all[1];
}

// lane's 16x16 block of wave tile `wt` (a 128x128 quadrant of a 256x256 tile): false if outside
__device__ __forceinline__ bool fused_locate(const FusedTensor &t, int64_t wt, int lane, int64_t &r0, int64_t &c0)
{
    const int64_t big = wt >> 2, by = big / t.tiles_x, bx = big - by * t.tiles_x;
    const int quad = (int)(wt & 3);
    r0 = by * kQuantBigTile + (quad >> 1) * 128 + (lane >> 3) * 16;
    c0 = bx * kQuantBigTile + (quad & 1) * 128 + (lane & 7) * 16;
    return r0 < t.rows && c0 < t.cols;
}

// rows 8*half .. +7 of a lane's block: codes into qd and out to q (16 bytes a row)
template <bool E5M2>
__device__ __forceinline__ void cast_rows8(const uint4 (&in)[8][2], int half, float scale, uint32_t (&qd)[16][4],
                                           uint8_t *__restrict__ q, int64_t r0, int64_t c0, int64_t cols)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = half * 8 + i;
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            const uint4 v = in[i][w];
            qd[r][2 * w] = cvt4_f8<E5M2>(bf16lo_to_f32(v.x) * scale, bf16hi_to_f32(v.x) * scale,
                                     bf16lo_to_f32(v.y) * scale, bf16hi_to_f32(v.y) * scale);
            qd[r][2 * w + 1] = cvt4_f8<E5M2>(bf16lo_to_f32(v.z) * scale, bf16hi_to_f32(v.z) * scale,
                                         bf16lo_to_f32(v.w) * scale, bf16hi_to_f32(v.w) * scale);
        }
        *(uint4 *)(q + (r0 + r) * cols + c0) = make_uint4(qd[r][0], qd[r][1], qd[r][2], qd[r][3]);
    }
}

// the block's codes transposed: column c0 + j of the block is 16 bytes of row c0 + j of qT
// LATER: nobody reads this copy soon (the transposed codes of a forward cast wait for the backward
// pass): the stores carry the streaming hint, the lines leave for memory without displacing what
// the next GEMM reads
template <bool LATER = false>
__device__ __forceinline__ void store_block_transposed(const uint32_t (&qd)[16][4], uint8_t *__restrict__ qT,
                                                       int64_t rows, int64_t r0, int64_t c0)
{
#pragma unroll
    for (int C = 0; C < 4; ++C) {
        uint32_t t[4][4];  // t[R][k]: column 4C+k, rows 4R..4R+3
#pragma unroll
        for (int R = 0; R < 4; ++R)
            transpose4x4_bytes(qd[4 * R][C], qd[4 * R + 1][C], qd[4 * R + 2][C], qd[4 * R + 3][C], t[R][0], t[R][1],
                               t[R][2], t[R][3]);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            typedef uint32_t v4u __attribute__((ext_vector_type(4)));
            v4u *dst = (v4u *)(qT + (c0 + 4 * C + k) * rows + r0);
            const v4u v = {t[0][k], t[1][k], t[2][k], t[3][k]};
            if constexpr (LATER)
                __builtin_nontemporal_store(v, dst);
            else
                *dst = v;
        }
    }
}

template <bool E5M2, bool T_LATER>
__global__ __launch_bounds__(kFusedThreads, 1) void amax_cast_fused_kernel(FusedTensor t0, FusedTensor t1, int64_t wt0,
                                                                           int64_t wt_total, int rounds,
                                                                           FusedSlot *slots, uint64_t token)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int G = gridDim.x;
    auto tile_of = [&](int k) { return ((int64_t)k * G + blockIdx.x) * kFusedWaves + wave; };

    // this wave's tiles are k = 0 .. mine-1 (the last round of the grid may not reach it)
    const int mine = tile_of(rounds - 1) < wt_total ? rounds : rounds - 1;

    // ---- phase 1: maxima; the block of the wave's last tile stays in `keep`, the upper half (rows
    // 0..7 of every lane's block) of the tile before it in LDS (lane-private slots, 16-byte pieces of
    // neighbouring lanes side by side: 128 KB per CU) ------------------------------------------------
    extern __shared__ __attribute__((aligned(16))) uint4 lds_keep[];  // [8 rows][2 pieces][kFusedThreads]
    uint4 keep2[8][2];  // the lower half of that tile: the registers that are left
#pragma unroll
    for (int i = 0; i < 8; ++i)
        keep2[i][0] = keep2[i][1] = make_uint4(0u, 0u, 0u, 0u);
    uint32_t mx0 = 0, mx1 = 0;
    for (int k = 0; k < mine - 1; ++k) {
        const int64_t wt = tile_of(k);
        const bool first = wt < wt0;
        const FusedTensor &t = first ? t0 : t1;
        int64_t r0, c0;
        if (!fused_locate(t, first ? wt : wt - wt0, lane, r0, c0))
            continue;
        uint32_t m = 0;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            uint4 in[8][2];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint4 *src = (const uint4 *)(t.x + (r0 + half * 8 + i) * t.cols + c0);
                in[i][0] = src[0];
                in[i][1] = src[1];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
                m = pk_absmax4(pk_absmax4(m, in[i][0]), in[i][1]);
            if (k == mine - 2) {
                if (half == 0) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        lds_keep[(i * 2 + 0) * kFusedThreads + threadIdx.x] = in[i][0];
                        lds_keep[(i * 2 + 1) * kFusedThreads + threadIdx.x] = in[i][1];
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        keep2[i][0] = in[i][0];
                        keep2[i][1] = in[i][1];
                    }
                }
            }
        }
        if (first)
            mx0 = pk_absmax4(mx0, make_uint4(m, 0u, 0u, 0u));
        else
            mx1 = pk_absmax4(mx1, make_uint4(m, 0u, 0u, 0u));
    }
    uint4 keep[16][2];
    bool kept = false, kept_first = false;
    int64_t kr0 = 0, kc0 = 0;
    {
        if (mine > 0) {
            const int64_t wt = tile_of(mine - 1);
            kept_first = wt < wt0;
            const FusedTensor &t = kept_first ? t0 : t1;
            kept = fused_locate(t, kept_first ? wt : wt - wt0, lane, kr0, kc0);
            if (kept) {
                uint32_t m = 0;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint4 *src = (const uint4 *)(t.x + (kr0 + i) * t.cols + kc0);
                    keep[i][0] = src[0];
                    keep[i][1] = src[1];
                }
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    m = pk_absmax4(pk_absmax4(m, keep[i][0]), keep[i][1]);
                if (kept_first)
                    mx0 = pk_absmax4(mx0, make_uint4(m, 0u, 0u, 0u));
                else
                    mx1 = pk_absmax4(mx1, make_uint4(m, 0u, 0u, 0u));
            }
        }
    }

    // ---- the workgroup's maxima, published; everybody's, collected ---------------------------
    uint32_t all0, all1;
    fused_grid_max<kFusedWaves>(mx0, mx1, slots, token, all0, all1);
    const float amax0 = __uint_as_float(all0), amax1 = __uint_as_float(all1);
    const float scale0 = scale_f8<E5M2>(amax0), scale1 = scale_f8<E5M2>(amax1);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *t0.amax_store = amax0;
        *t0.scale_out = scale0;
        *t0.scale_inv_out = 1.0f / scale0;
        if (wt_total > wt0) {
            *t1.amax_store = amax1;
            *t1.scale_out = scale1;
            *t1.scale_inv_out = 1.0f / scale1;
        }
    }

    // ---- phase 2: the cast, newest data first --------------------------------------------------
    uint32_t qd[16][4];
    if (kept) {
        const FusedTensor &t = kept_first ? t0 : t1;
        const float scale = kept_first ? scale0 : scale1;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            uint4 in[8][2];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                in[i][0] = keep[half * 8 + i][0];
                in[i][1] = keep[half * 8 + i][1];
            }
            cast_rows8<E5M2>(in, half, scale, qd, t.q, kr0, kc0, t.cols);
        }
        store_block_transposed<T_LATER>(qd, t.qT, t.rows, kr0, kc0);
    }
    for (int k = mine - 2; k >= 0; --k) {
        const int64_t wt = tile_of(k);
        const bool first = wt < wt0;
        const FusedTensor &t = first ? t0 : t1;
        const float scale = first ? scale0 : scale1;
        int64_t r0, c0;
        if (!fused_locate(t, first ? wt : wt - wt0, lane, r0, c0))
            continue;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            uint4 in[8][2];
            if (half == 0 && k == mine - 2) {  // what this lane left in LDS in phase 1
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    in[i][0] = lds_keep[(i * 2 + 0) * kFusedThreads + threadIdx.x];
                    in[i][1] = lds_keep[(i * 2 + 1) * kFusedThreads + threadIdx.x];
                }
            } else if (k == mine - 2) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    in[i][0] = keep2[i][0];
                    in[i][1] = keep2[i][1];
                }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint4 *src = (const uint4 *)(t.x + (r0 + half * 8 + i) * t.cols + c0);
                    in[i][0] = src[0];
                    in[i][1] = src[1];
                }
            }
            cast_rows8<E5M2>(in, half, scale, qd, t.q, r0, c0, t.cols);
        }
        store_block_transposed<T_LATER>(qd, t.qT, t.rows, r0, c0);
    }
}

static bool g_fused_cast_on = true;
void set_fused_cast(bool on) { g_fused_cast_on = on; }
bool fused_cast_enabled() { return g_fused_cast_on; }

hipError_t fused_cast_timeouts(uint32_t *count)
{
    return hipMemcpyFromSymbol(count, HIP_SYMBOL(g_fused_cast_timeouts), sizeof(uint32_t));
}

// Tokens start from the clock so that two processes that share a workspace allocation one after
// the other (the allocator hands memory round) do not start from the same number either.
static uint64_t next_fused_token()
{
    static std::atomic<uint64_t> counter{(uint64_t)std::chrono::steady_clock::now().time_since_epoch().count() << 20 | 1u};
    return counter.fetch_add(1, std::memory_order_relaxed);
}

// Whether the fused launch applies: whole 16x16 blocks, enough work to pay for the wait, not under
// stream capture (a replayed graph would replay the token).
bool fused_cast_applies(int64_t rows0, int64_t cols0, int64_t rows1, int64_t cols1, hipStream_t s)
{
    if (!g_fused_cast_on || rows0 % 16 != 0 || cols0 % 16 != 0 || rows1 % 16 != 0 || cols1 % 16 != 0)
        return false;
    // small tensors: two short launches are as fast (measured: no gain below ~16M elements, also not
    // with a form of this kernel in which every lane keeps one 8x8 block and nothing is read twice:
    // GPT-2 block step 0.563 -> 0.561 ms)
    if (rows0 * cols0 + rows1 * cols1 < ((int64_t)1 << 24))
        return false;
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess || st != hipStreamCaptureStatusNone)
        return false;
    return true;
}

// x1 may be nullptr (one tensor).  slots: 16 bytes per workgroup, at most kFusedMaxWorkgroups of
// them, no initial contents assumed.
hipError_t launch_amax_cast_fused(const void *x0_bf16, int64_t rows0, int64_t cols0, float *amax0, uint8_t *q0,
                                  uint8_t *q0T, float *scale0, float *scale0_inv, const void *x1_bf16,
                                  int64_t rows1, int64_t cols1, float *amax1, uint8_t *q1, uint8_t *q1T,
                                  float *scale1, float *scale1_inv, bool e5m2, bool transposed_later, void *slots,
                                  hipStream_t s)
{
    auto tiles = [](int64_t v) { return (v + kQuantBigTile - 1) / kQuantBigTile; };
    const FusedTensor t0{(const uint16_t *)x0_bf16, rows0, cols0, tiles(cols0), q0, q0T, amax0, scale0, scale0_inv};
    FusedTensor t1 = t0;
    int64_t wt1 = 0;
    if (x1_bf16 != nullptr) {
        t1 = FusedTensor{(const uint16_t *)x1_bf16, rows1, cols1, tiles(cols1), q1, q1T, amax1, scale1, scale1_inv};
        wt1 = 4 * tiles(rows1) * tiles(cols1);
    }
    const int64_t wt0 = 4 * tiles(rows0) * tiles(cols0), wt_total = wt0 + wt1;
    int64_t grid = (wt_total + kFusedWaves - 1) / kFusedWaves;
    const int64_t cap = amax_cus() < kFusedMaxWorkgroups ? amax_cus() : kFusedMaxWorkgroups;
    if (grid > cap)
        grid = cap;
    const int rounds = (int)((wt_total + grid * kFusedWaves - 1) / (grid * kFusedWaves));
    const uint64_t token = next_fused_token();
    hipError_t err = hipSuccess;
    auto launch = [&](auto kernel, bool &attr_done) {
        if (!attr_done) {  // more dynamic LDS than a kernel gets without asking
            err = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kFusedLdsBytes);
            if (err != hipSuccess)
                return;
            attr_done = true;
        }
        hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kFusedThreads), kFusedLdsBytes, s, t0, t1, wt0, wt_total,
                           rounds, (FusedSlot *)slots, token);
        err = hipGetLastError();
    };
    static bool done[3] = {false, false, false};
    if (e5m2)
        launch(amax_cast_fused_kernel<true, false>, done[0]);  // gradients: both copies are read at once
    else if (transposed_later)
        launch(amax_cast_fused_kernel<false, true>, done[1]);
    else
        launch(amax_cast_fused_kernel<false, false>, done[2]);
    return err;
}

// ---------------------------------------------------------------------------
// Delayed-scaling state (Sec. 4.3: amax history of length 16).  32 words in device memory:
//   [0..15] amax history ring   [16] amax of the tensor being cast (accumulator, 0 between calls)
//   [17] scale for the next cast, [18] its inverse   [19] ring position   [20] entries filled
//   [21] scale the last cast used, [22] its inverse (what the GEMM dequantises with)
// The scale of step t is 448 / max(history) over the up to 16 amax values of steps t-16..t-1 (the
// paper names the length, not the reduction: max); an empty history bootstraps from the
// tensor's own amax.  Guards as for the current-scaling scale.
__global__ void delayed_state_init_kernel(uint32_t *st)
{
    const int i = threadIdx.x;
    if (i < 32)
        st[i] = (i == 17 || i == 18 || i == 21 || i == 22) ? f32_to_bits(1.0f) : 0u;
}

// Consumes the accumulated amax: remembers the scale that was just used, pushes the amax into
// the ring, derives the next scale, clears the accumulator.  One thread.  sc_out (optional): three
// fp32 of the caller's: this tensor's amax, the scale its cast uses / used, and its inverse.
__device__ __forceinline__ void delayed_state_update(uint32_t *st, int bootstrap, float range, float *sc_out)
{
    int pos = (int)st[19], filled = (int)st[20];
    if (!bootstrap) {  // a bootstrap cast has not happened yet: nothing was "used"
        st[21] = st[17];
        st[22] = st[18];
    }
    const uint32_t mine = st[16];
    st[pos & 15] = mine;
    pos = (pos + 1) & 15;
    filled = filled < 16 ? filled + 1 : 16;
    uint32_t m = 0;
    for (int k = 0; k < 16; ++k)
        m = st[k] > m ? st[k] : m;  // magnitude patterns order like unsigned integers (NaN on top)
    const float scale = scale_from_amax_range(bits_to_f32(m), range);  // 448 (E4M3) or 57344 (E5M2)
    st[17] = f32_to_bits(scale);
    st[18] = f32_to_bits(1.0f / scale);
    st[19] = (uint32_t)pos;
    st[20] = (uint32_t)filled;
    st[16] = 0u;
    if (bootstrap) {  // the cast that follows uses this scale
        st[21] = st[17];
        st[22] = st[18];
    }
    if (sc_out != nullptr) {
        sc_out[0] = bits_to_f32(mine);
        sc_out[1] = bits_to_f32(st[21]);
        sc_out[2] = bits_to_f32(st[22]);
    }
}

__global__ void delayed_state_update_kernel(uint32_t *st, int bootstrap, float range,
                                            const uint32_t *partials = nullptr, int n_partials = 0,
                                            float *sc_out = nullptr)
{
    if (threadIdx.x != 0 || blockIdx.x != 0)
        return;
    if (partials != nullptr) {  // the tensor's amax arrives as one maximum per workgroup of an earlier launch
        uint32_t m = 0;
        for (int i = 0; i < n_partials; ++i)
            m = partials[i] > m ? partials[i] : m;
        st[16] = m;
    }
    delayed_state_update(st, bootstrap, range, sc_out);
}

// two states in one launch (the activation's and the weight's of a linear layer): block b, thread 0
__global__ void delayed_state_update2_kernel(uint32_t *st0, float *sc0, uint32_t *st1, float *sc1, float range)
{
    if (threadIdx.x == 0)
        delayed_state_update(blockIdx.x == 0 ? st0 : st1, 0, range, blockIdx.x == 0 ? sc0 : sc1);
}

hipError_t launch_delayed_state_init(void *state, hipStream_t s)
{
    hipLaunchKernelGGL(delayed_state_init_kernel, dim3(1), dim3(64), 0, s, (uint32_t *)state);
    return hipGetLastError();
}

template <bool E5M2>
static hipError_t launch_quantize_f8_delayed(const void *x_bf16, int64_t rows, int64_t cols, void *state,
                                             int bootstrap, uint8_t *q, uint8_t *qT, hipStream_t s,
                                             float *sc_out = nullptr)
{
    float *st = (float *)state;
    const float range = E5M2 ? 57344.0f : 448.0f;
    hipError_t e;
    if (bootstrap) {
        // empty history: this tensor's own amax makes the scale (two passes, once)
        e = launch_amax(x_bf16, rows * cols, st + 16, s);
        if (e != hipSuccess)
            return e;
        hipLaunchKernelGGL(delayed_state_update_kernel, dim3(1), dim3(64), 0, s, (uint32_t *)state, 1, range,
                           (const uint32_t *)nullptr, 0, sc_out);
        e = hipGetLastError();
        if (e != hipSuccess)
            return e;
        // the history already holds this tensor's amax: the cast returns none
        return launch_quantize_e4m3_impl<true, E5M2>(x_bf16, rows, cols, st + 21, q, qT, nullptr, nullptr,
                                                     nullptr, s);
    }
    e = launch_quantize_e4m3_impl<true, E5M2>(x_bf16, rows, cols, st + 17, q, qT, nullptr, nullptr,
                                              (uint32_t *)st + 16, s);
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(delayed_state_update_kernel, dim3(1), dim3(64), 0, s, (uint32_t *)state, 0, range,
                       (const uint32_t *)nullptr, 0, sc_out);
    return hipGetLastError();
}

hipError_t launch_quantize_e4m3_delayed(const void *x_bf16, int64_t rows, int64_t cols, void *state,
                                        int bootstrap, uint8_t *q, uint8_t *qT, hipStream_t s, float *sc_out)
{
    return launch_quantize_f8_delayed<false>(x_bf16, rows, cols, state, bootstrap, q, qT, s, sc_out);
}

hipError_t launch_quantize_e5m2_delayed(const void *x_bf16, int64_t rows, int64_t cols, void *state,
                                        int bootstrap, uint8_t *q, uint8_t *qT, hipStream_t s, float *sc_out)
{
    return launch_quantize_f8_delayed<true>(x_bf16, rows, cols, state, bootstrap, q, qT, s, sc_out);
}

// The activation and the weight of a linear layer under delayed scaling in one cast launch and one
// state-update launch (each tensor with its transposed copy; rows, cols multiples of 16).
struct QuantTensorDelayed {
    const uint16_t *x;
    int64_t rows, cols, tiles_x;
    const float *scale;
    uint8_t *q, *qT;
    uint32_t *amax_acc;
};

__global__ __launch_bounds__(kQuantThreads) void quantize2_delayed_16x16_kernel(QuantTensorDelayed t0, int64_t blocks0,
                                                                                QuantTensorDelayed t1, int64_t blocks1)
{
    const bool first = (int64_t)blockIdx.x < blocks0;
    const QuantTensorDelayed &t = first ? t0 : t1;
    quantize_e4m3_16x16_body<true, true, false, 0, false, false, true>(t.x, t.rows, t.cols, t.tiles_x, t.scale, t.q, t.qT, nullptr, nullptr, t.amax_acc,
                                         first ? (int64_t)blockIdx.x : (int64_t)blockIdx.x - blocks0,
                                         first ? blocks0 : blocks1);
}

hipError_t launch_quantize2_e4m3_delayed(const void *x0_bf16, int64_t rows0, int64_t cols0, void *state0, uint8_t *q0,
                                         uint8_t *q0T, float *sc0, const void *x1_bf16, int64_t rows1, int64_t cols1,
                                         void *state1, uint8_t *q1, uint8_t *q1T, float *sc1, int bootstrap,
                                         hipStream_t s)
{
    if (bootstrap) {  // empty histories: each tensor's own amax first (once per state)
        hipError_t e = launch_quantize_f8_delayed<false>(x0_bf16, rows0, cols0, state0, 1, q0, q0T, s, sc0);
        if (e != hipSuccess)
            return e;
        return launch_quantize_f8_delayed<false>(x1_bf16, rows1, cols1, state1, 1, q1, q1T, s, sc1);
    }
    auto tiles = [](int64_t v) { return (v + kQuantBigTile - 1) / kQuantBigTile; };
    float *st0 = (float *)state0, *st1 = (float *)state1;
    QuantTensorDelayed t0{(const uint16_t *)x0_bf16, rows0, cols0, tiles(cols0), st0 + 17, q0, q0T, (uint32_t *)st0 + 16};
    QuantTensorDelayed t1{(const uint16_t *)x1_bf16, rows1, cols1, tiles(cols1), st1 + 17, q1, q1T, (uint32_t *)st1 + 16};
    // a bounded grid (its one atomic per workgroup stays a few hundred per tensor), shared out in
    // proportion to the tile counts
    const int64_t n0 = tiles(rows0) * tiles(cols0), n1 = tiles(rows1) * tiles(cols1);
    int64_t b1 = (int64_t)(1024.0 * (double)n1 / (double)(n0 + n1) + 0.5);
    b1 = b1 < 1 ? 1 : (b1 > n1 ? n1 : b1);
    int64_t b0 = 1024 - b1;
    b0 = b0 < 1 ? 1 : (b0 > n0 ? n0 : b0);
    hipLaunchKernelGGL(quantize2_delayed_16x16_kernel, dim3((unsigned)(b0 + b1)), dim3(kQuantThreads), 0, s, t0, b0, t1, b1);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(delayed_state_update2_kernel, dim3(2), dim3(64), 0, s, (uint32_t *)state0, sc0, (uint32_t *)state1,
                       sc1, 448.0f);
    return hipGetLastError();
}

// LayerNorm -> per-tensor E4M3 cast (Sec. 4.3).  Launches: row statistics (2 B/element from
// memory; with a residual it also forms and stores h = bf16(x + r)); for current scaling, or for
// the first call on a delayed-scaling state, an amax-only pass over the normalised tensor (it
// re-reads the rows from the caches); then the cast, which normalises on the way in (re-read from
// the caches, 1 B/element written per copy of the codes, + 2 B/element if y is wanted).
// stats: 2 doubles per row; partials: kAmaxPartialsMax words.  rows, cols multiples of 16.
hipError_t launch_layernorm_quantize(const void *x_bf16, const void *res_bf16, const void *gamma_bf16,
                                     const void *beta_bf16, int64_t rows, int64_t cols, double eps, void *h_out,
                                     void *y_out, uint8_t *q, uint8_t *qT, double *stats, uint32_t *partials,
                                     float *amax_out, float *scale_out, float *scale_inv_out, void *state,
                                     int bootstrap, hipStream_t s)
{
    const int vec = (int)(cols / 8);
    constexpr int WAVES = kLnThreads / kWave;
    int64_t sgrid = (rows + WAVES - 1) / WAVES;
    // small workgroups, as many as fit a CU at once (70 / 80 registers a lane: seven / six waves per
    // SIMD): the pass is a chain of latencies per row (loads, two wave-wide fp64 reductions), so what
    // counts is how many rows are in flight
    const int64_t resident = (res_bf16 != nullptr ? 6 : 7) * (int64_t)amax_cus();
    if (sgrid > resident)
        sgrid = resident;
    if (res_bf16 != nullptr)
        hipLaunchKernelGGL(ln_stats_kernel<true>, dim3((unsigned)sgrid), dim3(kLnThreads), 0, s, (const uint4 *)x_bf16,
                           (const uint4 *)res_bf16, (uint4 *)h_out, rows, vec, eps, stats);
    else
        hipLaunchKernelGGL(ln_stats_kernel<false>, dim3((unsigned)sgrid), dim3(kLnThreads), 0, s, (const uint4 *)x_bf16,
                           (const uint4 *)nullptr, (uint4 *)nullptr, rows, vec, eps, stats);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    const uint16_t *src = (const uint16_t *)(res_bf16 != nullptr ? h_out : x_bf16);
    const LnArgs ln{stats, (const uint16_t *)gamma_bf16, (const uint16_t *)beta_bf16};
    const int64_t tiles_x = (cols + kQuantBigTile - 1) / kQuantBigTile, tiles_y = (rows + kQuantBigTile - 1) / kQuantBigTile;
    const int64_t n_tiles = tiles_x * tiles_y;
    const int64_t bounded = n_tiles < kAmaxMaxPartials ? n_tiles : kAmaxMaxPartials;
    const dim3 block(kQuantThreads);
    float *st = (float *)state;
    const bool delayed = state != nullptr;
    if (!delayed || bootstrap) {
        hipLaunchKernelGGL((quantize_ln_16x16_kernel<false, true, true>), dim3((unsigned)bounded), block, 0, s, src, ln, rows,
                           cols, tiles_x, (const float *)nullptr, (uint8_t *)nullptr, (uint8_t *)nullptr,
                           (uint16_t *)nullptr, (float *)nullptr, (float *)nullptr, partials, (const uint32_t *)nullptr, 0,
                           (float *)nullptr);
        if ((e = hipGetLastError()) != hipSuccess)
            return e;
    }
    if (!delayed) {
        if (qT)
            hipLaunchKernelGGL((quantize_ln_16x16_kernel<true, false, false>), dim3((unsigned)n_tiles), block, 0, s, src, ln,
                               rows, cols, tiles_x, (const float *)amax_out, q, qT, (uint16_t *)y_out, scale_out, scale_inv_out,
                               (uint32_t *)nullptr, (const uint32_t *)partials, (int)bounded, amax_out);
        else
            hipLaunchKernelGGL((quantize_ln_16x16_kernel<false, false, false>), dim3((unsigned)n_tiles), block, 0, s, src, ln,
                               rows, cols, tiles_x, (const float *)amax_out, q, qT, (uint16_t *)y_out, scale_out, scale_inv_out,
                               (uint32_t *)nullptr, (const uint32_t *)partials, (int)bounded, amax_out);
        return hipGetLastError();
    }
    if (bootstrap) {  // empty history: the tensor's own amax makes the scale
        hipLaunchKernelGGL(delayed_state_update_kernel, dim3(1), dim3(64), 0, s, (uint32_t *)state, 1, 448.0f,
                           (const uint32_t *)partials, (int)bounded, (float *)nullptr);
        if ((e = hipGetLastError()) != hipSuccess)
            return e;
    }
    const float *scale_src = bootstrap ? st + 21 : st + 17;
    uint32_t *acc = bootstrap ? nullptr : (uint32_t *)st + 16;
    int64_t n_wg = n_tiles < 1024 ? n_tiles : 1024;
    if (qT)
        hipLaunchKernelGGL((quantize_ln_16x16_kernel<true, true, false>), dim3((unsigned)n_wg), block, 0, s, src, ln, rows, cols,
                           tiles_x, scale_src, q, qT, (uint16_t *)y_out, (float *)nullptr, (float *)nullptr, acc,
                           (const uint32_t *)nullptr, 0, (float *)nullptr);
    else
        hipLaunchKernelGGL((quantize_ln_16x16_kernel<false, true, false>), dim3((unsigned)n_wg), block, 0, s, src, ln, rows, cols,
                           tiles_x, scale_src, q, qT, (uint16_t *)y_out, (float *)nullptr, (float *)nullptr, acc,
                           (const uint32_t *)nullptr, 0, (float *)nullptr);
    if ((e = hipGetLastError()) != hipSuccess)
        return e;
    if (!bootstrap)
        hipLaunchKernelGGL(delayed_state_update_kernel, dim3(1), dim3(64), 0, s, (uint32_t *)state, 0, 448.0f,
                           (const uint32_t *)nullptr, 0, (float *)nullptr);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Static INT8 quantize (Sec. 4.4 Eq. 4, Q_8 = 127): q = clamp(rne(x*inv_step), +-127).
// 16 elements per lane: two 16-byte loads, one 16-byte store.  3 B/element.
constexpr int kQi8Threads = 256;

__device__ __forceinline__ uint32_t q_i8(float v, float inv_step)
{
    float prod = v * inv_step;
    float r = __builtin_rintf(prod);  // v_rndne_f32: ties to even
    r = __builtin_amdgcn_fmed3f(r, -127.0f, 127.0f);
    r = (prod != prod) ? 0.0f : r;  // NaN -> 0
    return (uint32_t)(int)r & 0xFFu;
}

__device__ __forceinline__ uint32_t q_i8x4(uint32_t d0, uint32_t d1, float s)
{
    return q_i8(bf16lo_to_f32(d0), s) | (q_i8(bf16hi_to_f32(d0), s) << 8) |
           (q_i8(bf16lo_to_f32(d1), s) << 16) | (q_i8(bf16hi_to_f32(d1), s) << 24);
}

__global__ __launch_bounds__(kQi8Threads) void quantize_i8_kernel(const uint4 *__restrict__ x,
                                                                  int64_t n_vec, float inv_step,
                                                                  uint2 *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * kQi8Threads;
    for (int64_t i = (int64_t)blockIdx.x * kQi8Threads + threadIdx.x; i < n_vec; i += stride) {
        uint4 v = x[i];
        out[i] = make_uint2(q_i8x4(v.x, v.y, inv_step), q_i8x4(v.z, v.w, inv_step));
    }
}

hipError_t launch_quantize_i8(const void *x_bf16, int64_t n, float inv_step, int8_t *out,
                              hipStream_t s)
{
    int64_t n_vec = n / 8;
    int64_t blocks = (n_vec + kQi8Threads - 1) / kQi8Threads;
    if (blocks > 256 * 16)
        blocks = 256 * 16;
    hipLaunchKernelGGL(quantize_i8_kernel, dim3((unsigned)blocks), dim3(kQi8Threads), 0, s,
                       (const uint4 *)x_bf16, n_vec, inv_step, (uint2 *)out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Row-granular AbsMax INT8 (Sec. 4.4 Eq. 4 with one s per token vector or per output channel):
// s_r = max_c |x_rc| + eps, q = clamp(rne(x * (127 / s_r)), +-127), step_r = s_r / 127.
// TPR lanes share a row (one wave for short rows, four for long ones); the first four 16-byte
// pieces of each lane stay in registers between the maximum and the rounding, so rows of up to
// 32*TPR elements are read from memory once; longer rows read the rest a second time (from L2).
// 3 B/element + 4 B/row.
constexpr int kQrowThreads = 256;
constexpr int kQrowCached = 4;

template <int TPR>
__global__ __launch_bounds__(kQrowThreads) void quantize_i8_rows_kernel(const uint4 *__restrict__ x, int64_t rows,
                                                                        int vec_per_row, float eps,
                                                                        uint2 *__restrict__ q,
                                                                        float *__restrict__ step)
{
    constexpr int RPB = kQrowThreads / TPR;
    const int t = threadIdx.x % TPR;
    const int64_t row_raw = (int64_t)blockIdx.x * RPB + threadIdx.x / TPR;
    const bool live = row_raw < rows;  // uniform over a wave: TPR is a multiple of the wave size
    const int64_t row = live ? row_raw : rows - 1;
    const uint4 *xr = x + row * vec_per_row;
    uint4 c[kQrowCached];
    uint32_t m = 0;
#pragma unroll
    for (int u = 0; u < kQrowCached; ++u) {
        const int i = t + u * TPR;
        c[u] = make_uint4(0u, 0u, 0u, 0u);
        if (i < vec_per_row) {
            c[u] = xr[i];
            m = pk_absmax4(m, c[u]);
        }
    }
    for (int i = t + kQrowCached * TPR; i < vec_per_row; i += TPR)
        m = pk_absmax4(m, xr[i]);
    uint32_t r = (m & 0xFFFFu) > (m >> 16) ? (m & 0xFFFFu) : (m >> 16);
    r = wave_reduce_max_u32(r);
    if constexpr (TPR > kWave) {
        static_assert(TPR == kQrowThreads, "a long row takes the whole workgroup");
        __shared__ uint32_t red[kQrowThreads / kWave];
        if ((threadIdx.x & (kWave - 1)) == 0)
            red[threadIdx.x / kWave] = r;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < kQrowThreads / kWave; ++w)
            r = red[w] > r ? red[w] : r;
    }
    const float s = __uint_as_float(r << 16) + eps;
    const float inv = 127.0f / s;
    if (!live)
        return;
    if (t == 0)
        step[row] = s / 127.0f;
    uint2 *qr = q + row * vec_per_row;
#pragma unroll
    for (int u = 0; u < kQrowCached; ++u) {
        const int i = t + u * TPR;
        if (i < vec_per_row)
            qr[i] = make_uint2(q_i8x4(c[u].x, c[u].y, inv), q_i8x4(c[u].z, c[u].w, inv));
    }
    for (int i = t + kQrowCached * TPR; i < vec_per_row; i += TPR) {
        const uint4 v = xr[i];
        qr[i] = make_uint2(q_i8x4(v.x, v.y, inv), q_i8x4(v.z, v.w, inv));
    }
}

hipError_t launch_quantize_i8_rows(const void *x_bf16, int64_t rows, int64_t cols, float eps, int8_t *q,
                                   float *step, hipStream_t s)
{
    const int vec = (int)(cols / 8);
    if (vec <= kWave * kQrowCached) {
        const int64_t blocks = (rows + kQrowThreads / kWave - 1) / (kQrowThreads / kWave);
        hipLaunchKernelGGL(quantize_i8_rows_kernel<kWave>, dim3((unsigned)blocks), dim3(kQrowThreads), 0, s,
                           (const uint4 *)x_bf16, rows, vec, eps, (uint2 *)q, step);
    } else {
        hipLaunchKernelGGL(quantize_i8_rows_kernel<kQrowThreads>, dim3((unsigned)rows), dim3(kQrowThreads), 0, s,
                           (const uint4 *)x_bf16, rows, vec, eps, (uint2 *)q, step);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Penalty-gradient injection (the derivative of the loss of Sec. 3.3 with
// respect to the penalised activation, added to the incoming output gradient):
//   out = bf16( dy + coef * sign(a) * (|a| / (tau+eps))^(p-1) ),
//   coef = g * p / (tau+eps), g = the caller's lambda / (L * numel).
// 6 B/element of HBM traffic (two 2-byte reads, one 2-byte write); fp32
// arithmetic, the power by repeated multiplication (p is a small integer).
constexpr int kInjectThreads = 256;

template <int P>
__global__ __launch_bounds__(kInjectThreads) void penalty_grad_inject_kernel(
    const uint4 *__restrict__ dy, const uint4 *__restrict__ act, int64_t n_vec, float inv_tau, float coef,
    int p, uint4 *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * kInjectThreads;
    for (int64_t i = (int64_t)blockIdx.x * kInjectThreads + threadIdx.x; i < n_vec; i += stride) {
        const uint4 d = dy[i], a = act[i];
        const uint32_t dd[4] = {d.x, d.y, d.z, d.w}, aa[4] = {a.x, a.y, a.z, a.w};
        uint32_t r[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            r[k] = pack_bf16x2(
                inject_one<P>(bf16lo_to_f32(dd[k]), bf16lo_to_f32(aa[k]), inv_tau, coef, p),
                inject_one<P>(bf16hi_to_f32(dd[k]), bf16hi_to_f32(aa[k]), inv_tau, coef, p));
        out[i] = make_uint4(r[0], r[1], r[2], r[3]);
    }
}

hipError_t launch_penalty_grad_inject(const void *dy_bf16, const void *a_bf16, int64_t n, float inv_tau,
                                      float coef, int p, void *out_bf16, hipStream_t s)
{
    const int64_t n_vec = n / 8;
    int64_t blocks = (n_vec + kInjectThreads - 1) / kInjectThreads;
    if (blocks > 256 * 16)
        blocks = 256 * 16;
    if (p == 4)
        hipLaunchKernelGGL(penalty_grad_inject_kernel<4>, dim3((unsigned)blocks), dim3(kInjectThreads), 0, s,
                           (const uint4 *)dy_bf16, (const uint4 *)a_bf16, n_vec, inv_tau, coef, p,
                           (uint4 *)out_bf16);
    else
        hipLaunchKernelGGL(penalty_grad_inject_kernel<0>, dim3((unsigned)blocks), dim3(kInjectThreads), 0, s,
                           (const uint4 *)dy_bf16, (const uint4 *)a_bf16, n_vec, inv_tau, coef, p,
                           (uint4 *)out_bf16);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Penalty finish: sums the per-workgroup fp32 partials in a fixed order in fp64.
constexpr int kFinishThreads = 256;

__global__ __launch_bounds__(kFinishThreads) void penalty_finish_kernel(
    const float *__restrict__ partials, int n, double *out)
{
    __shared__ double red[kFinishThreads];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += kFinishThreads)
        s += (double)partials[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = kFinishThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w)
            red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0)
        *out = red[0];
}

hipError_t launch_penalty_finish(const float *partials, int n, double *out, hipStream_t s)
{
    hipLaunchKernelGGL(penalty_finish_kernel, dim3(1), dim3(kFinishThreads), 0, s, partials, n, out);
    return hipGetLastError();
}

}  // namespace tweo
