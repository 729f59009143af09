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
    bf16_t* dst[3];
    int64_t ld[3];
    int col_end[3];
    int64_t lda, ldw, ldr;
    int M, N, K;
    int mt, nt;          // tile counts
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

    // The prefetch registers are plain locals filled and drained unconditionally (the last
    // iteration re-loads the final K slice into the idle LDS stage): no branches around the
    // loads, so they stay in VGPRs and their latency hides behind the MFMA work.
    uint4 ra[4], rw[4];
#define PO_GLOAD(kt_)                                              \
    {                                                              \
        const int k0_ = (kt_) * BK;                                \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {            \
            ra[i] = *(const uint4*)(ga[i] + k0_);                  \
            rw[i] = *(const uint4*)(gw[i] + k0_);                  \
        }                                                          \
    }
#define PO_SSTORE(stage_)                                          \
    {                                                              \
        unsigned char* sa_ = smem + (stage_) * STAGE_BYTES;        \
        unsigned char* sw_ = sa_ + TILE_BYTES;                     \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {            \
            *(uint4*)(sa_ + st_off + i * 8192) = ra[i];            \
            *(uint4*)(sw_ + st_off + i * 8192) = rw[i];            \
        }                                                          \
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
    PO_GLOAD(0);
    PO_SSTORE(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        PO_GLOAD(min(kt + 1, KT - 1));
        const unsigned char* sa = smem + (kt & 1) * STAGE_BYTES;
        const unsigned char* sw = sa + TILE_BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int seg_off = (((kk * 2 + lhi) ^ fsw) << 4);
            bf16x8 af[4], wf[2];
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) af[mi] = *(const bf16x8*)(sa + a_row_off + mi * 4096 + seg_off);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) wf[ni] = *(const bf16x8*)(sw + w_row_off + ni * 4096 + seg_off);
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], wf[ni], acc[mi][ni], 0, 0, 0);
        }
        PO_SSTORE((kt + 1) & 1);
        __syncthreads();
    }
#undef PO_GLOAD
#undef PO_SSTORE

    // ---- epilogue.  Accumulator layout of a 32x32 tile: lane holds column (lane & 31),
    // register r holds row 8*(r/4) + 4*(lane/32) + (r%4).
    const int row_base = m0 + wm * 128 + 4 * lhi;
    if (EPI == EPI_SILU_MUL) {
        const int ocol = (n0 + wn * 64) / 2 + l31;          // column in H[M, N/2]
        if (ocol < p.N / 2) {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = row_base + mi * 32 + 8 * (r >> 2) + (r & 3);
                    if (row < p.M)
                        p.dst[0][(int64_t)row * p.ld[0] + ocol] = f2bf(silu_f(acc[mi][0][r]) * acc[mi][1][r]);
                }
        }
        return;
    }
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        const int col_base = n0 + wn * 64 + ni * 32;
        if (col_base >= p.N) continue;
        int s = 0, col_start = 0;
        if (EPI == EPI_STORE) {
            while (s < 2 && col_base >= p.col_end[s]) { col_start = p.col_end[s]; ++s; }
        }
        const int col = col_base + l31;
        const float bv = (EPI == EPI_STORE && p.bias) ? bf2f(p.bias[col]) : 0.f;
        bf16_t* dptr = p.dst[s] + (col - col_start);
        const int64_t ld = p.ld[s];
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = row_base + mi * 32 + 8 * (r >> 2) + (r & 3);
                if (row < p.M) {
                    float v = acc[mi][ni][r] + bv;
                    if (EPI == EPI_RESIDUAL) v += bf2f(p.R[(int64_t)row * p.ldr + col]);
                    dptr[(int64_t)row * ld] = f2bf(v);
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

void launch_gemm_mfma(int epi, const bf16_t* A, int64_t lda, const bf16_t* W, int64_t ldw, const GemmSeg* segs,
                      int nseg, const bf16_t* bias, const bf16_t* R, int64_t ldr, int64_t M, int N, int K,
                      hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    GemmParams p;
    p.A = A; p.W = W; p.bias = bias; p.R = R;
    p.lda = lda; p.ldw = ldw; p.ldr = ldr;
    for (int i = 0; i < 3; ++i) {
        const int j = i < nseg ? i : nseg - 1;
        p.dst[i] = (bf16_t*)segs[j].ptr;
        p.ld[i] = segs[j].ld;
        p.col_end[i] = i < nseg ? segs[j].col_end : N;
    }
    p.M = (int)M; p.N = N; p.K = K;
    p.mt = (int)((M + BM - 1) / BM);
    p.nt = (N + BN - 1) / BN;
    switch (epi) {
        case EPI_STORE: launch_t<EPI_STORE>(p, s); break;
        case EPI_RESIDUAL: launch_t<EPI_RESIDUAL>(p, s); break;
        case EPI_SILU_MUL: launch_t<EPI_SILU_MUL>(p, s); break;
        default: break;
    }
}

}  // namespace po
