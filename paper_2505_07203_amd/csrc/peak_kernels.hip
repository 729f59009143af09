// Micro-peaks of the machine, measured beside the nominal ones: a matrix-instruction loop that touches no memory
// inside the loop, and a streaming copy.  They bound what the path's kernels can reach on THIS board (whose clock
// under matrix load is set by its power limit, well below the 2.4 GHz the nominal peak assumes).
#include "po_internal.h"

namespace po {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

namespace {

// Every wavefront loads one A and one B fragment (16 bytes per lane each) from `operands` and multiplies them
// `iters` times into independent accumulators: KIND 0 = 8 accumulators of v_mfma_f32_32x32x16_bf16, KIND 1 = 32
// of v_mfma_f32_16x16x32_bf16 (262 144 and 524 288 flop per wavefront and iteration).  The MFMAs are written as
// instructions on accumulation registers: from the builtin the compiler makes a loop that copies accumulators and
// pads with s_nop, which a single wavefront per SIMD cannot hide (it then reads 0.61 of the pipe's rate for the
// 16x16x32 instruction where the instruction loop reads 0.93-0.95, the same as two wavefronts per SIMD).
template <int NT, int KIND>
__global__ void __launch_bounds__(NT) mfma_peak_kernel(const uint4* __restrict__ operands, float* sink, int iters) {
    const size_t i = ((size_t)blockIdx.x * NT + threadIdx.x) * 2;
    const bf16x8 a = __builtin_bit_cast(bf16x8, operands[i]);
    const bf16x8 b = __builtin_bit_cast(bf16x8, operands[i + 1]);
    float s = 0.f;
    if (KIND == 0) {
        f32x16 c[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) c[j][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 8; ++j) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c[j]) : "v"(a), "v"(b));
        }
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");      // (the compiler does not know the instruction's latency)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += c[j][0];
    } else {
        f32x4 c[32];
#pragma unroll
        for (int j = 0; j < 32; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) c[j][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 32; ++j) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c[j]) : "v"(a), "v"(b));
        }
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
        for (int j = 0; j < 32; ++j) s += c[j][0];
    }
    if (s == 12345.678f) sink[0] = s;      // keeps the loop; practically never true
}

// four 16-byte loads in flight per lane before the first store; a workgroup copies 16 KiB per step
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) stream_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 1024;
    for (size_t i0 = (size_t)blockIdx.x * 1024 + threadIdx.x; i0 < n16; i0 += stride) {
        u32x4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (i0 + j * 256 < n16) v[j] = __builtin_nontemporal_load(src + i0 + j * 256);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (i0 + j * 256 < n16) __builtin_nontemporal_store(v[j], dst + i0 + j * 256);
    }
}

}  // namespace

// -> flop executed (0: arguments refused).  operand_bytes must cover 32 bytes per launched thread.
double launch_mfma_peak(int kind, int waves_per_simd, int iters, const void* operands, size_t operand_bytes, float* sink,
                        hipStream_t s) {
    if ((kind != 0 && kind != 1) || (waves_per_simd != 1 && waves_per_simd != 2) || iters <= 0) return 0.0;
    const int nt = 256 * waves_per_simd, blocks = 256 * 4;             // four workgroups per compute unit, in turn
    if (operand_bytes < (size_t)blocks * nt * 32) return 0.0;
    const uint4* op = (const uint4*)operands;
    // 96 KiB of (unused) dynamic LDS per workgroup: one workgroup per compute unit at a time, so that the number of
    // wavefronts per SIMD is what the caller asked for
    constexpr int LDS = 96 * 1024;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)mfma_peak_kernel<256, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        (void)hipFuncSetAttribute((const void*)mfma_peak_kernel<512, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        (void)hipFuncSetAttribute((const void*)mfma_peak_kernel<256, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        (void)hipFuncSetAttribute((const void*)mfma_peak_kernel<512, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        attr_set = true;
    }
    if (kind == 0 && nt == 256) hipLaunchKernelGGL((mfma_peak_kernel<256, 0>), dim3(blocks), dim3(256), LDS, s, op, sink, iters);
    if (kind == 0 && nt == 512) hipLaunchKernelGGL((mfma_peak_kernel<512, 0>), dim3(blocks), dim3(512), LDS, s, op, sink, iters);
    if (kind == 1 && nt == 256) hipLaunchKernelGGL((mfma_peak_kernel<256, 1>), dim3(blocks), dim3(256), LDS, s, op, sink, iters);
    if (kind == 1 && nt == 512) hipLaunchKernelGGL((mfma_peak_kernel<512, 1>), dim3(blocks), dim3(512), LDS, s, op, sink, iters);
    // per wavefront and iteration: 8 x (32 x 32 x 16) = 131 072 multiply-adds, or 32 x (16 x 16 x 32) = 262 144
    return (double)blocks * (nt / 64) * (double)iters * (kind == 0 ? 262144.0 : 524288.0);
}

void launch_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return;
    hipLaunchKernelGGL(stream_copy_kernel, dim3(256 * 32), dim3(256), 0, s, (const u32x4*)src, (u32x4*)dst, n16);
}

}  // namespace po
