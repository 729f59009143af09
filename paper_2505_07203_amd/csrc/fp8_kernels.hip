// FP8-dynamic variant of the decoder's linear layers: quantisation kernels (gfx950, OCP E4M3).
//
// A row x (bf16) with amax = max|x_k| is stored as codes e4m3(x_k * (448 / amax)) and the float32
// scale amax / 448 (amax == 0: codes 0, scale 1).  Both divisions and the product are single,
// correctly rounded float32 operations and the conversion (v_cvt_pk_fp8_f32) rounds to nearest
// even, so codes and scales are reproducible bit for bit from the bf16 input.  Weights use the same
// kernel, a row being an output channel (fixed at load time); activations are quantised per token
// when they are used (Section 7.1 names FP8-dynamic checkpoints; the scheme is the public
// convention of those checkpoints).
#include "po_internal.h"

namespace po {
namespace {

constexpr int QV = 14;                       // 16-byte vectors per thread: rows of up to 256 * 8 * 14 elements
constexpr float E4M3_MAX = 448.0f;

__device__ __forceinline__ float wg_max(float v, float* part) {
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
}

__device__ __forceinline__ float amax8(const uint4& v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float m = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c)
        m = fmaxf(m, fmaxf(fabsf(__uint_as_float(w[c] << 16)), fabsf(__uint_as_float(w[c] & 0xffff0000u))));
    return m;
}

// 8 bf16 values (one 16-byte vector) -> 8 codes
__device__ __forceinline__ uint2 encode8(const uint4& v, float inv) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float f[8];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        f[2 * c] = __uint_as_float(w[c] << 16) * inv;
        f[2 * c + 1] = __uint_as_float(w[c] & 0xffff0000u) * inv;
    }
    int lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], 0, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
    int hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], 0, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
    return make_uint2((uint32_t)lo, (uint32_t)hi);
}

// One workgroup per row; the row stays in registers, so the codes may overwrite the row itself.
// Source row r goes to destination row (r / blk) * dst_blk_stride + r % blk + dst_off (codes and scale).
__global__ void __launch_bounds__(256) quant_rows_kernel(const bf16_t* x, int64_t ldx, unsigned char* q, int64_t ldq,
                                                         float* scales, int vecs, int blk, int64_t dst_blk_stride,
                                                         int64_t dst_off) {
    __shared__ float part[4];
    const int64_t r = blockIdx.x;
    const int64_t dr = (r / blk) * dst_blk_stride + (r % blk) + dst_off;
    const uint4* xr = (const uint4*)(x + r * ldx);
    uint4 v[QV];
    float m = 0.f;
#pragma unroll
    for (int j = 0; j < QV; ++j) {
        const int i = threadIdx.x + j * 256;
        if (i < vecs) {
            v[j] = xr[i];
            m = fmaxf(m, amax8(v[j]));
        }
    }
    const float amax = wg_max(m, part);                 // (the barrier inside orders all loads before any store)
    const float safe = amax > 0.f ? amax : 1.0f;
    const float inv = __fdiv_rn(E4M3_MAX, safe);
    if (threadIdx.x == 0) scales[dr] = amax > 0.f ? __fdiv_rn(safe, E4M3_MAX) : 1.0f;
    uint2* qr = (uint2*)(q + dr * ldq);
#pragma unroll
    for (int j = 0; j < QV; ++j) {
        const int i = threadIdx.x + j * 256;
        if (i < vecs) qr[i] = encode8(v[j], inv);
    }
}

// RMSNorm whose output goes straight to codes: y = bf16(x * rstd * g) exactly as the bf16 kernel forms it,
// then quantised per row (d % 8 == 0, d <= 8192)
__global__ void __launch_bounds__(256) rmsnorm_quant_kernel(const uint4* __restrict__ x, const uint4* __restrict__ g,
                                                            unsigned char* __restrict__ q, float* __restrict__ scales,
                                                            int vecs, float eps, float inv_d) {
    __shared__ float part[4], partm[4];
    const int64_t row = blockIdx.x;
    const uint4* xr = x + row * vecs;
    uint4 v[4];
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int i = threadIdx.x + j * 256;
        if (i < vecs) {
            v[j] = xr[i];
            const uint32_t w[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float lo = __uint_as_float(w[c] << 16), hi = __uint_as_float(w[c] & 0xffff0000u);
                ss += lo * lo + hi * hi;
            }
        }
    }
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float r = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) * inv_d + eps);
    float m = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int i = threadIdx.x + j * 256;
        if (i < vecs) {
            const uint4 gv = g[i];
            const uint32_t w[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
            const uint32_t gw[4] = {gv.x, gv.y, gv.z, gv.w};
            uint32_t o[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float lo = __uint_as_float(w[c] << 16) * r * __uint_as_float(gw[c] << 16);
                float hi = __uint_as_float(w[c] & 0xffff0000u) * r * __uint_as_float(gw[c] & 0xffff0000u);
                o[c] = (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
            }
            v[j] = make_uint4(o[0], o[1], o[2], o[3]);
            m = fmaxf(m, amax8(v[j]));
        }
    }
    const float amax = wg_max(m, partm);
    const float safe = amax > 0.f ? amax : 1.0f;
    const float inv = __fdiv_rn(E4M3_MAX, safe);
    if (threadIdx.x == 0) scales[row] = amax > 0.f ? __fdiv_rn(safe, E4M3_MAX) : 1.0f;
    uint2* qr = (uint2*)(q + row * (int64_t)vecs * 8);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int i = threadIdx.x + j * 256;
        if (i < vecs) qr[i] = encode8(v[j], inv);
    }
}

}  // namespace

bool quant_rows_supported(int K) { return K > 0 && K % 8 == 0 && K <= 256 * 8 * QV; }

void launch_quant_rows(const bf16_t* x, int64_t ldx, unsigned char* q, int64_t ldq, float* scales, int64_t rows, int K,
                       int blk, int64_t dst_blk_stride, int64_t dst_off, hipStream_t s) {
    if (rows <= 0) return;
    hipLaunchKernelGGL(quant_rows_kernel, dim3((unsigned)rows), dim3(256), 0, s, x, ldx, q, ldq, scales, K / 8,
                       blk > 0 ? blk : (int)rows, dst_blk_stride, dst_off);
}

void launch_rmsnorm_quant(const bf16_t* x, const bf16_t* g, unsigned char* q, float* scales, int64_t rows, int d,
                          float eps, hipStream_t s) {
    if (rows <= 0) return;
    hipLaunchKernelGGL(rmsnorm_quant_kernel, dim3((unsigned)rows), dim3(256), 0, s, (const uint4*)x, (const uint4*)g, q,
                       scales, d / 8, eps, 1.0f / (float)d);
}

}  // namespace po
