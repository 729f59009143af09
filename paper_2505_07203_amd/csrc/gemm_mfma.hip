// bf16 MFMA GEMM for the position-wise linear layers (gfx950 / CDNA4).
//
//   C[M, N] = A[M, K] * W[N, K]^T        A: activations (token-major), W: weights in the
//                                        checkpoint layout [out, in]; both K-contiguous.
//
// Block tile 256 x 256 x 64, 512 threads = 8 wavefronts arranged 2 (M) x 4 (N); each
// wavefront owns a 128 x 64 patch = 4 x 2 MFMA 32x32x16 tiles (128 fp32 accumulators per
// lane).  Operand tiles go global -> registers -> LDS (16-byte segments, XOR-swizzled so
// that both the 16-byte row writes and the MFMA fragment reads are bank-conflict free),
// double-buffered in LDS with one barrier per K slice: the global loads of slice k+1 are
// in flight while slice k is multiplied.
//
// Workgroups are dispatched round-robin over the 8 XCDs (each with a private L2), so the
// block id is first split into (XCD, local index) and every XCD walks a contiguous range
// of output tiles in groups of 4 M-tiles x consecutive N-tiles: the 32 tiles resident on
// one XCD then share 4 activation panels and 8 weight panels through that XCD's L2.
//
// A row's K reduction order is fixed by the kernel and independent of how M is tiled or
// chunked, which is what makes the chunk-by-chunk evaluation of Section 4.2 bit-exact.
#include "po_internal.h"

#include <string.h>

namespace po {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NTHREADS = 512;
constexpr int TILE_BYTES = BM * BK * 2;            // 32 KiB per operand per stage
constexpr int STAGE_BYTES = 2 * TILE_BYTES;        // A + W
constexpr int SMEM_BYTES = 2 * STAGE_BYTES;        // double buffer: 128 KiB
constexpr int GROUP_M = 4;

struct GemmParams {
    const bf16_t* A;
    const bf16_t* W;
    const bf16_t* bias;
    const bf16_t* R;
    bf16_t* dst;         // EPI_STORE / EPI_RESIDUAL / EPI_SILU_MUL destination; EPI_QKV_ROPE: Q
    bf16_t* dst_k;       // EPI_QKV_ROPE: K [*, kvd]
    bf16_t* dst_vt;      // EPI_QKV_ROPE: V^T [kvd][ldv]
    const float* rope_cos;   // [positions, hd/2]
    const float* rope_sin;
    int64_t ld, ldv;
    int64_t lda, ldw, ldr;
    int64_t pos0;        // EPI_QKV_ROPE: sequence position of GEMM row 0
    int M, N, K;
    int mt, nt;          // tile counts
    int qd, kvd, hd;     // EPI_QKV_ROPE: segment widths and head size
};

// 16-byte segment swizzle inside a 128-byte tile row: a bijection on the 8 segments for
// any 8 consecutive rows, and rows r, r+8 land in different (row parity, segment) slots.
__device__ __forceinline__ int swz8(int row) { return (row & 7) ^ ((row >> 3) & 1); }

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

template <int EPI>
__global__ void __launch_bounds__(NTHREADS) gemm_bf16_mfma_kernel(const GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    // ---- XCD-aware tile assignment
    const int total = p.mt * p.nt;
    const int per_xcd = (total + 7) >> 3;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int li = xcd * per_xcd + local;
    if (local >= per_xcd || li >= total) return;
    const int group_sz = GROUP_M * p.nt;
    const int g = li / group_sz;
    const int within = li - g * group_sz;
    const int gm_this = min(GROUP_M, p.mt - g * GROUP_M);
    const int tn = within / gm_this;
    const int tm = g * GROUP_M + (within - tn * gm_this);
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l31 = lane & 31, lhi = lane >> 5;
    const int wm = wave >> 2, wn = wave & 3;

    // ---- global -> register staging: thread owns segment `lseg` of rows lrow + 64 i
    const int lseg = tid & 7, lrow = tid >> 3;
    const bf16_t* ga[4];
    const bf16_t* gw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int ra = min(m0 + lrow + 64 * i, p.M - 1);
        const int rw = min(n0 + lrow + 64 * i, p.N - 1);
        ga[i] = p.A + (int64_t)ra * p.lda + lseg * 8;
        gw[i] = p.W + (int64_t)rw * p.ldw + lseg * 8;
    }
    const int st_off = lrow * 128 + ((lseg ^ swz8(lrow)) << 4);   // + 64*i rows = + 8192 i bytes

    // Two register sets hold the next two K slices (prefetch distance 2): the loads of slice
    // k+2 / k+3 are in flight while slice k is multiplied, which covers HBM latency.  Loads
    // and LDS stores are unconditional (slice indices clamp to the last slice, whose extra
    // copies land in an LDS stage nobody reads again), so the sets stay in VGPRs.
    uint4 a0_0, a0_1, a0_2, a0_3, w0_0, w0_1, w0_2, w0_3;     // register set 0
    uint4 a1_0, a1_1, a1_2, a1_3, w1_0, w1_1, w1_2, w1_3;     // register set 1
#define PO_GLOAD(S, kt_)                                           \
    {                                                              \
        const int k0_ = min((kt_), KT - 1) * BK;                   \
        a##S##_0 = *(const uint4*)(ga[0] + k0_);                   \
        w##S##_0 = *(const uint4*)(gw[0] + k0_);                   \
        a##S##_1 = *(const uint4*)(ga[1] + k0_);                   \
        w##S##_1 = *(const uint4*)(gw[1] + k0_);                   \
        a##S##_2 = *(const uint4*)(ga[2] + k0_);                   \
        w##S##_2 = *(const uint4*)(gw[2] + k0_);                   \
        a##S##_3 = *(const uint4*)(ga[3] + k0_);                   \
        w##S##_3 = *(const uint4*)(gw[3] + k0_);                   \
    }
#define PO_SSTORE(S, stage_)                                       \
    {                                                              \
        unsigned char* sa_ = smem + (stage_) * STAGE_BYTES + st_off; \
        unsigned char* sw_ = sa_ + TILE_BYTES;                     \
        *(uint4*)(sa_) = a##S##_0;                                 \
        *(uint4*)(sw_) = w##S##_0;                                 \
        *(uint4*)(sa_ + 8192) = a##S##_1;                          \
        *(uint4*)(sw_ + 8192) = w##S##_1;                          \
        *(uint4*)(sa_ + 16384) = a##S##_2;                         \
        *(uint4*)(sw_ + 16384) = w##S##_2;                         \
        *(uint4*)(sa_ + 24576) = a##S##_3;                         \
        *(uint4*)(sw_ + 24576) = w##S##_3;                         \
    }
#define PO_COMPUTE(stage_)                                                                               \
    {                                                                                                    \
        const unsigned char* sa = smem + (stage_) * STAGE_BYTES;                                         \
        const unsigned char* sw = sa + TILE_BYTES;                                                       \
        _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                               \
            const int seg_off = (((kk * 2 + lhi) ^ fsw) << 4);                                           \
            bf16x8 af[4], wf[2];                                                                         \
            _Pragma("unroll") for (int mi = 0; mi < 4; ++mi)                                             \
                af[mi] = *(const bf16x8*)(sa + a_row_off + mi * 4096 + seg_off);                         \
            _Pragma("unroll") for (int ni = 0; ni < 2; ++ni)                                             \
                wf[ni] = *(const bf16x8*)(sw + w_row_off + ni * 4096 + seg_off);                         \
            _Pragma("unroll") for (int mi = 0; mi < 4; ++mi)                                             \
                _Pragma("unroll") for (int ni = 0; ni < 2; ++ni)                                         \
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ni], af[mi], acc[mi][ni], 0, 0, 0); \
        }                                                                                                \
    }

    f32x16 acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    // fragment read offsets (bytes) for k-step 0; k-step kk toggles segment bits
    const int fsw = swz8(l31);
    const int a_row_off = (wm * 128 + l31) * 128;
    const int w_row_off = (wn * 64 + l31) * 128;
    const int KT = p.K / BK;

    PO_GLOAD(0, 0);
    PO_SSTORE(0, 0);
    PO_GLOAD(0, 1);
    PO_GLOAD(1, 2);
    __syncthreads();
    for (int kt = 0; kt + 1 < KT; kt += 2) {
        PO_COMPUTE(0);                       // slice kt
        PO_SSTORE(0, 1);              // slice kt+1
        PO_GLOAD(0, kt + 3);
        __syncthreads();
        PO_COMPUTE(1);                       // slice kt+1
        PO_SSTORE(1, 0);              // slice kt+2
        PO_GLOAD(1, kt + 4);
        __syncthreads();
    }
    if (KT & 1) PO_COMPUTE(0);               // odd slice count: the last slice sits in stage 0
#undef PO_GLOAD
#undef PO_SSTORE
#undef PO_COMPUTE

    // ---- epilogue.  The MFMA is issued as (W fragment) x (A fragment)^T, so in a 32x32
    // accumulator tile a lane holds ONE token row (lane & 31) and register r holds feature
    // 8*(r/4) + 4*(lane/32) + (r%4): four consecutive features per register quad, which are
    // combined, rounded and moved with 8-byte accesses.
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int row = m0 + wm * 128 + mi * 32 + l31;
        if (row >= p.M) continue;
        const int cb = n0 + wn * 64;                 // first column of this wavefront's patch
        if (cb >= p.N) continue;
        if (EPI == EPI_SILU_MUL) {
            bf16_t* drow = p.dst + (int64_t)row * p.ld + cb / 2 + 4 * lhi;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                float h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) h[e] = silu_f(acc[mi][0][4 * g4 + e]) * acc[mi][1][4 * g4 + e];
                uint2 w;
                w.x = (uint32_t)f2bf(h[0]) | ((uint32_t)f2bf(h[1]) << 16);
                w.y = (uint32_t)f2bf(h[2]) | ((uint32_t)f2bf(h[3]) << 16);
                *(uint2*)(drow + 8 * g4) = w;
            }
        } else if (EPI == EPI_QKV_ROPE) {
            const int half = p.hd >> 1;
            if (cb < p.qd + p.kvd) {
                // Q or K patch: sub-tile 0 holds rotary index i, sub-tile 1 holds i + hd/2 (the
                // weight rows were packed that way), so a pair sits in one lane, same register.
                const bool is_q = cb < p.qd;
                const int c = is_q ? cb : cb - p.qd;
                const int head = c / p.hd;
                const int patch = (c - head * p.hd) >> 6;
                const int i0 = patch * 32 + 4 * lhi;             // rotary index of register quad 0
                bf16_t* drow = (is_q ? p.dst + (int64_t)row * p.qd : p.dst_k + (int64_t)row * p.kvd) +
                               head * p.hd + i0;
                const float* ct = p.rope_cos + (p.pos0 + row) * half + i0;
                const float* st = p.rope_sin + (p.pos0 + row) * half + i0;
                const bf16_t* bp = p.bias ? p.bias + cb + 4 * lhi : nullptr;
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const float4 cs = *(const float4*)(ct + 8 * g4);
                    const float4 sn = *(const float4*)(st + 8 * g4);
                    const float cv[4] = {cs.x, cs.y, cs.z, cs.w}, sv[4] = {sn.x, sn.y, sn.z, sn.w};
                    float lo[4], hi[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float a = acc[mi][0][4 * g4 + e], b = acc[mi][1][4 * g4 + e];
                        if (bp) { a += bf2f(bp[8 * g4 + e]); b += bf2f(bp[32 + 8 * g4 + e]); }
                        lo[e] = a * cv[e] - b * sv[e];
                        hi[e] = b * cv[e] + a * sv[e];
                    }
                    uint2 w;
                    w.x = (uint32_t)f2bf(lo[0]) | ((uint32_t)f2bf(lo[1]) << 16);
                    w.y = (uint32_t)f2bf(lo[2]) | ((uint32_t)f2bf(lo[3]) << 16);
                    *(uint2*)(drow + 8 * g4) = w;
                    w.x = (uint32_t)f2bf(hi[0]) | ((uint32_t)f2bf(hi[1]) << 16);
                    w.y = (uint32_t)f2bf(hi[2]) | ((uint32_t)f2bf(hi[3]) << 16);
                    *(uint2*)(drow + half + 8 * g4) = w;
                }
            } else {
                // V patch: stored transposed, V^T[feature][position]; consecutive lanes are
                // consecutive positions.
                const int f0 = cb - p.qd - p.kvd + 4 * lhi;
                bf16_t* dcol = p.dst_vt + p.pos0 + row;
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int f = f0 + ni * 32 + 8 * (r >> 2) + (r & 3);
                        float v = acc[mi][ni][r];
                        if (p.bias) v += bf2f(p.bias[p.qd + p.kvd + f]);
                        dcol[(int64_t)f * p.ldv] = f2bf(v);
                    }
            }
        } else {
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const int col = cb + ni * 32 + 4 * lhi;
                if (cb + ni * 32 >= p.N) continue;
                bf16_t* drow = p.dst + (int64_t)row * p.ld + col;
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[mi][ni][4 * g4 + e];
                    if (EPI == EPI_STORE && p.bias) {
                        const uint2 bw = *(const uint2*)(p.bias + col + 8 * g4);
                        v[0] += __uint_as_float(bw.x << 16); v[1] += __uint_as_float(bw.x & 0xffff0000u);
                        v[2] += __uint_as_float(bw.y << 16); v[3] += __uint_as_float(bw.y & 0xffff0000u);
                    }
                    if (EPI == EPI_RESIDUAL) {
                        const uint2 rw = *(const uint2*)(p.R + (int64_t)row * p.ldr + col + 8 * g4);
                        v[0] += __uint_as_float(rw.x << 16); v[1] += __uint_as_float(rw.x & 0xffff0000u);
                        v[2] += __uint_as_float(rw.y << 16); v[3] += __uint_as_float(rw.y & 0xffff0000u);
                    }
                    uint2 w;
                    w.x = (uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16);
                    w.y = (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16);
                    *(uint2*)(drow + 8 * g4) = w;
                }
            }
        }
    }
}

template <int EPI>
void launch_t(const GemmParams& p, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)gemm_bf16_mfma_kernel<EPI>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
        attr_set = true;
    }
    const int total = p.mt * p.nt;
    const int per_xcd = (total + 7) / 8;
    hipLaunchKernelGGL(gemm_bf16_mfma_kernel<EPI>, dim3((unsigned)(per_xcd * 8)), dim3(NTHREADS), SMEM_BYTES, s, p);
}

}  // namespace

bool gemm_mfma_supported(int N, int K) { return K > 0 && K % BK == 0 && N > 0 && N % 32 == 0; }

static GemmParams base_params(const bf16_t* A, int64_t lda, const bf16_t* W, int64_t ldw, int64_t M, int N, int K) {
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A = A; p.W = W; p.lda = lda; p.ldw = ldw;
    p.M = (int)M; p.N = N; p.K = K;
    p.mt = (int)((M + BM - 1) / BM);
    p.nt = (N + BN - 1) / BN;
    return p;
}

void launch_gemm_mfma(int epi, const bf16_t* A, int64_t lda, const bf16_t* W, int64_t ldw, bf16_t* C, int64_t ldc,
                      const bf16_t* bias, const bf16_t* R, int64_t ldr, int64_t M, int N, int K, hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    GemmParams p = base_params(A, lda, W, ldw, M, N, K);
    p.bias = bias; p.R = R; p.ldr = ldr; p.dst = C; p.ld = ldc;
    switch (epi) {
        case EPI_STORE: launch_t<EPI_STORE>(p, s); break;
        case EPI_RESIDUAL: launch_t<EPI_RESIDUAL>(p, s); break;
        case EPI_SILU_MUL: launch_t<EPI_SILU_MUL>(p, s); break;
        default: break;
    }
}

void launch_gemm_qkv_rope(const bf16_t* A, int64_t lda, const bf16_t* Wqkv, int64_t ldw, const bf16_t* bias,
                          bf16_t* Q, bf16_t* Kd, bf16_t* Vt, int64_t ldv, const float* rope_cos,
                          const float* rope_sin, int64_t pos0, int64_t M, int qd, int kvd, int hd, int K,
                          hipStream_t s) {
    if (M <= 0) return;
    GemmParams p = base_params(A, lda, Wqkv, ldw, M, qd + 2 * kvd, K);
    p.bias = bias; p.dst = Q; p.dst_k = Kd; p.dst_vt = Vt; p.ldv = ldv;
    p.rope_cos = rope_cos; p.rope_sin = rope_sin; p.pos0 = pos0;
    p.qd = qd; p.kvd = kvd; p.hd = hd;
    launch_t<EPI_QKV_ROPE>(p, s);
}

}  // namespace po
