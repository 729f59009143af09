// FP8 (OCP E4M3) MFMA GEMM for the FP8-dynamic variant of the position-wise linear layers (gfx950).
//
//   C[M, N] = (Qa[M, K] * Qw[N, K]^T) * sa[M] * sw[N]      codes one byte each, K-contiguous rows;
//                                                          sa: one scale per token, sw: per output feature
//
// The same design as the bf16 kernel (256 x 256 block, 4 wavefronts x 128 x 128 patch, five-unit LDS
// ring of 32 KiB units filled by buffer_load ... lds, XCD-aware tile order, shared epilogues): a row of a
// unit is again one 128-byte line, which now holds 128 codes, so a slice is 128 k and feeds two k-steps of
// the 32x32x64 MFMA (twice the flops per byte moved, per LDS read and per cycle of the matrix pipe).  A
// fragment is 32 bytes per lane: two 16-byte reads.  The products accumulate in fp32; the scales are
// applied to the accumulators before the (unchanged) epilogue arithmetic.
#include "gemm_common.h"

#include <string.h>

namespace po {

typedef __attribute__((__vector_size__(8 * sizeof(int)))) int i32x8;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;

namespace {

using namespace gemm;

constexpr int BKB = 128;                           // bytes (= codes) of K per slice
constexpr int UNIT_BYTES = BM * BKB;               // one operand's slice: 256 rows x 128 bytes = 32 KiB
constexpr int NUNIT = 5;
constexpr int SMEM_BYTES = NUNIT * UNIT_BYTES;

#define PO_HANDOVER() asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory")

template <int EPI>
__global__ void __launch_bounds__(NTHREADS) gemm_fp8_mfma_kernel(const GemmParams p) {
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
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, lhi = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- global -> LDS map.  A unit (one operand's 256 rows x 64 k) is 32 one-KiB loads; wavefront w issues
    // loads w*8 .. w*8+7, load q fills rows q*8 .. q*8+7: lane l -> row q*8 + l/8, physical segment l & 7,
    // which holds logical segment (l & 7) ^ ((row >> 1) & 7).  Eight lanes fetch one whole 128-byte line.
    // Each operand is addressed through a buffer resource that starts at the tile's first row and ends with
    // the matrix: the per-lane byte offset never changes, the slice offset is one scalar, and rows of a
    // ragged last tile beyond the matrix read as zero instead of needing a clamp (they are never stored).
    // (split-K launches: workgroup row blockIdx.y works on codes [k0, k0 + K) of both operands)
    const int64_t k0 = (EPI == EPI_PARTIAL) ? (int64_t)blockIdx.y * p.K : 0;
    const uint64_t a_bytes = (uint64_t)(p.M - m0) * (uint64_t)p.lda - (uint64_t)k0, w_bytes = (uint64_t)(p.N - n0) * (uint64_t)p.ldw - (uint64_t)k0;
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const unsigned char*)p.A + (int64_t)m0 * p.lda + k0), 0, (int)(uint32_t)(a_bytes > 0xffffffffull ? 0xffffffffull : a_bytes), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const unsigned char*)p.W + (int64_t)n0 * p.ldw + k0), 0, (int)(uint32_t)(w_bytes > 0xffffffffull ? 0xffffffffull : w_bytes), 0x00020000);
    uint32_t voa[8], vow[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = wave * 64 + i * 8 + (lane >> 3);
        const int lseg = (lane & 7) ^ ((row >> 1) & 7);
        voa[i] = (uint32_t)row * (uint32_t)p.lda + lseg * 16;
        vow[i] = (uint32_t)row * (uint32_t)p.ldw + lseg * 16;
    }
    const int KT = p.K / BKB;
    // load i_ (0..7) of this wavefront's share of unit u_ (even: activations of slice u_/2, odd: weights)
    // into ring position pos_
#define PO_DMA(u_, pos_, i_)                                                                                  \
    {                                                                                                         \
        const int t_ = min((u_) >> 1, KT - 1);                                                                \
        unsigned char* sa_ = smem + (pos_) * UNIT_BYTES + wave * 8192 + (i_) * 1024;                          \
        __builtin_amdgcn_raw_ptr_buffer_load_lds((u_) & 1 ? rw : ra, (__attribute__((address_space(3))) void*)sa_, 16, \
                                                 (u_) & 1 ? vow[(i_)] : voa[(i_)], t_ * BKB, 0, 0);      \
    }

    f32x16 acc[4][4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    // fragment read offsets: row l31 of a 32-row tile; k-step kk (64 codes) of its 128 bytes: a lane takes the
    // 32 bytes of logical segments kk*4 + lhi*2 and + 1 (two 16-byte reads); one lane register per k-step,
    // segment, operand and 64 KiB of LDS, the rest of an address is an immediate below 64 KiB
    int a_off[3][2][2], w_off[3][2][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
            const int fo = l31 * 128 + (((kk * 4 + lhi * 2 + h2) ^ ((l31 >> 1) & 7)) << 4);
#pragma unroll
            for (int hb = 0; hb < 3; ++hb) {
                a_off[hb][kk][h2] = hb * 65536 + wm * 16384 + fo;
                w_off[hb][kk][h2] = hb * 65536 + wn * 16384 + fo;
            }
        }

    // Software pipeline inside the wavefront, as in the bf16 kernel: memory instructions are issued one or
    // two at a time between MFMAs (a 32x32x64 MFMA keeps the pipe busy for 64 cycles).  A slice is two blocks
    // of 16 MFMA, one per k-step of 64 codes; a block also reads the 8 fragments (16 reads) of the next k-step
    // on its first 8 MFMAs and issues 8 loads on the other 8:
    //   block 0 of slice s: fragments of (s, k-step 1); the 8 loads of activation unit s+2
    //   hand-over barrier:  slice s+1 has landed; nobody reads slice s's units any more
    //   block 1 of slice s: fragments of (s+1, k-step 0); the 8 loads of weight unit s+2, into the
    //                       position slice s's activations occupied (unit u lives at u mod 5)
    // At the hand-over the loads issued after those of slice s+1 are the 8 of activation unit s+2.
    i32x8 af0[4], wf0[4], af1[4], wf1[4];
#define PO_FRAG1(AF, WF, pa_, pw_, kk_, j_)                                                          \
    {                                                                                               \
        if ((j_) < 4) {                                                                             \
            const i32x4 lo_ = *(const i32x4*)(smem + a_off[(pa_) >> 1][kk_][0] + ((pa_) & 1) * UNIT_BYTES + ((j_) & 3) * 4096); \
            const i32x4 hi_ = *(const i32x4*)(smem + a_off[(pa_) >> 1][kk_][1] + ((pa_) & 1) * UNIT_BYTES + ((j_) & 3) * 4096); \
            AF[(j_) & 3] = __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7);               \
        } else {                                                                                    \
            const i32x4 lo_ = *(const i32x4*)(smem + w_off[(pw_) >> 1][kk_][0] + ((pw_) & 1) * UNIT_BYTES + ((j_) & 3) * 4096); \
            const i32x4 hi_ = *(const i32x4*)(smem + w_off[(pw_) >> 1][kk_][1] + ((pw_) & 1) * UNIT_BYTES + ((j_) & 3) * 4096); \
            WF[(j_) & 3] = __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7);               \
        }                                                                                           \
    }
    // E4M3 x E4M3 (format selectors 0, 0), block scales fixed at 2^0
#define PO_MFMA1(AF, WF, t_)                                                                        \
    acc[(t_) >> 2][(t_) & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(                     \
        WF[(t_) & 3], AF[(t_) >> 2], acc[(t_) >> 2][(t_) & 3], 0, 0, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
    // fragment read in slot t (order of first use: MFMA t needs AF[t >> 2] and WF[t & 3]), or -1
#define PO_READ_SLOT(t_) ((t_) == 0 ? 0 : (t_) >= 1 && (t_) <= 4 ? 3 + (t_) : (t_) >= 5 && (t_) <= 7 ? (t_) - 4 : -1)
    // one block: MFMAs on (AFc, WFc); reads k-step kkn_ of the slice at positions (pa_, pw_) into (AFn, WFn);
    // the 8 loads of unit u_ into position up_
#define PO_BLOCK(AFc, WFc, AFn, WFn, pa_, pw_, kkn_, u_, up_)                                         \
    _Pragma("unroll") for (int t = 0; t < 16; ++t) {                                                \
        PO_MFMA1(AFc, WFc, t);                                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        if (PO_READ_SLOT(t) >= 0) {                                                                 \
            PO_FRAG1(AFn, WFn, pa_, pw_, kkn_, PO_READ_SLOT(t));                                    \
        } else {                                                                                    \
            PO_DMA(u_, up_, t - 8);                                                                 \
        }                                                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                          \
    }
    // slice s_ whose number is j_ modulo 5 (a literal): its units sit at positions 2j mod 5 and 2j+1 mod 5
#define PO_SLICE(s_, j_)                                                                            \
    {                                                                                               \
        PO_BLOCK(af0, wf0, af1, wf1, (2 * (j_)) % 5, (2 * (j_) + 1) % 5, 1, 2 * (s_) + 4, (2 * (j_) + 4) % 5); \
        PO_HANDOVER();                                                                              \
        PO_BLOCK(af1, wf1, af0, wf0, (2 * (j_) + 2) % 5, (2 * (j_) + 3) % 5, 0, 2 * (s_) + 5, (2 * (j_)) % 5); \
    }
    // in flight when the first slice is awaited: units 0..3 (slices 0 and 1)
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 8; ++i) PO_DMA(u, u, i);
    asm volatile("s_waitcnt vmcnt(16)\n\ts_barrier" ::: "memory");     // slice 0 has landed
#pragma unroll
    for (int j = 0; j < 8; ++j) PO_FRAG1(af0, wf0, 0, 1, 0, j);
    int s = 0;
    for (; s + 5 <= KT; s += 5) {
        PO_SLICE(s, 0);
        PO_SLICE(s + 1, 1);
        PO_SLICE(s + 2, 2);
        PO_SLICE(s + 3, 3);
        PO_SLICE(s + 4, 4);
    }
    if (s < KT) { PO_SLICE(s, 0); ++s; }
    if (s < KT) { PO_SLICE(s, 1); ++s; }
    if (s < KT) { PO_SLICE(s, 2); ++s; }
    if (s < KT) { PO_SLICE(s, 3); ++s; }
#undef PO_SLICE
#undef PO_BLOCK
#undef PO_READ_SLOT
#undef PO_DMA
#undef PO_FRAG1
#undef PO_MFMA1
    // the clamped tail loads have landed and every wavefront has finished reading the ring
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // codes -> values: one scale per token row (this lane's) and one per output feature
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const float sx = p.sa[min(m0 + wm * 128 + mi * 32 + l31, p.M - 1)];
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int col = min(n0 + wn * 128 + ni * 32 + 8 * g4 + 4 * lhi, p.N - 4);
                const float4 sw = *(const float4*)(p.sw + col);
                acc[mi][ni][4 * g4] = acc[mi][ni][4 * g4] * sx * sw.x;
                acc[mi][ni][4 * g4 + 1] = acc[mi][ni][4 * g4 + 1] * sx * sw.y;
                acc[mi][ni][4 * g4 + 2] = acc[mi][ni][4 * g4 + 2] * sx * sw.z;
                acc[mi][ni][4 * g4 + 3] = acc[mi][ni][4 * g4 + 3] * sx * sw.w;
            }
    }
    if (EPI == EPI_PARTIAL) {
        GemmParams q = p;
        q.dst = (bf16_t*)((float*)p.dst + (int64_t)blockIdx.y * p.ldr);     // this split's plane of partial sums
        tile_epilogue<EPI>(q, acc, smem, m0, n0, wave, lane);
    } else {
        tile_epilogue<EPI>(p, acc, smem, m0, n0, wave, lane);
    }
}

template <int EPI>
void launch_t(const GemmParams& p, hipStream_t s, int splits = 1) {
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)gemm_fp8_mfma_kernel<EPI>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
        attr_set = true;
    }
    const int total = p.mt * p.nt;
    const int per_xcd = (total + 7) / 8;
    hipLaunchKernelGGL(gemm_fp8_mfma_kernel<EPI>, dim3((unsigned)(per_xcd * 8), (unsigned)splits), dim3(NTHREADS), SMEM_BYTES, s, p);
}

GemmParams base_params(const unsigned char* A, int64_t lda, const float* sa, const unsigned char* W, int64_t ldw,
                       const float* sw, int64_t M, int N, int K) {
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A = (const bf16_t*)A; p.W = (const bf16_t*)W; p.lda = lda; p.ldw = ldw;      // byte pointers, byte pitches
    p.sa = sa; p.sw = sw;
    p.q_scale = 1.0f;
    p.M = (int)M; p.N = N; p.K = K;
    p.mt = (int)((M + BM - 1) / BM);
    p.nt = (N + BN - 1) / BN;
    return p;
}

}  // namespace

// K must be a multiple of 128 (whole slices), N of 64 (the epilogues work on 64-column patches).
bool gemm_fp8_supported(int N, int K) { return K > 0 && K % 128 == 0 && N > 0 && N % 64 == 0; }

void launch_gemm_fp8(int epi, const unsigned char* A, int64_t lda, const float* sa, const unsigned char* W, int64_t ldw,
                     const float* sw, bf16_t* C, int64_t ldc, const bf16_t* bias, const bf16_t* R, int64_t ldr, int64_t M,
                     int N, int K, hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    GemmParams p = base_params(A, lda, sa, W, ldw, sw, M, N, K);
    p.bias = bias; p.R = R; p.ldr = ldr; p.dst = C; p.ld = ldc;
    switch (epi) {
        case EPI_STORE: launch_t<EPI_STORE>(p, s); break;
        case EPI_RESIDUAL: launch_t<EPI_RESIDUAL>(p, s); break;
        case EPI_SILU_MUL: launch_t<EPI_SILU_MUL>(p, s); break;
        default: break;
    }
}

// The split-K forms (few rows): partial sums already carry the row and column scales, so the reduce kernels
// of the bf16 GEMM finish them.  epi: EPI_RESIDUAL (C = sum + R) or EPI_SILU_MUL (C = H [M, N / 2]).
int launch_gemm_fp8_splitk(int epi, const unsigned char* A, int64_t lda, const float* sa, const unsigned char* W,
                           int64_t ldw, const float* sw, bf16_t* C, int64_t ldc, const bf16_t* R, int64_t ldr, int64_t M,
                           int N, int K, float* part, size_t part_bytes, hipStream_t s) {
    if (M <= 0 || !gemm_fp8_supported(N, K) || (epi != EPI_RESIDUAL && epi != EPI_SILU_MUL)) return 0;
    if (epi == EPI_RESIDUAL && ((N & 7) || (ldc & 7) || (ldr & 7))) return 0;
    const int splits = pick_splits(M, N, K / BKB, part_bytes);
    if (splits < 2) return 0;
    GemmParams p = base_params(A, lda, sa, W, ldw, sw, M, N, K / splits);
    p.dst = (bf16_t*)part;
    p.ld = N;
    p.ldr = M * (int64_t)N;
    launch_t<EPI_PARTIAL>(p, s, splits);
    if (epi == EPI_RESIDUAL) launch_splitk_reduce_residual(part, splits, R, ldr, C, ldc, M, N, s);
    else launch_splitk_reduce_silu(part, splits, C, ldc, M, N, s);
    return splits;
}

int launch_gemm_fp8_qkv_rope_splitk(const unsigned char* A, int64_t lda, const float* sa, const unsigned char* Wqkv,
                                    int64_t ldw, const float* sw, const bf16_t* bias, bf16_t* Q, bf16_t* Kd, bf16_t* Vt,
                                    int64_t ldv, const float* rope_cos, const float* rope_sin, int64_t pos0,
                                    const int32_t* row_pos, int64_t M, int qd, int kvd, int hd, int K, float q_scale,
                                    float* part, size_t part_bytes, hipStream_t s) {
    const int N = qd + 2 * kvd;
    if (M <= 0 || !gemm_fp8_supported(N, K) || (qd & 63) || (kvd & 63) || (hd & 63)) return 0;
    const int splits = pick_splits(M, N, K / BKB, part_bytes);
    if (splits < 2) return 0;
    GemmParams p = base_params(A, lda, sa, Wqkv, ldw, sw, M, N, K / splits);
    p.dst = (bf16_t*)part;
    p.ld = N;
    p.ldr = M * (int64_t)N;
    launch_t<EPI_PARTIAL>(p, s, splits);
    GemmParams r = base_params(A, lda, sa, Wqkv, ldw, sw, M, N, K);
    r.bias = bias; r.dst = Q; r.dst_k = Kd; r.dst_vt = Vt; r.ldv = ldv;
    r.rope_cos = rope_cos; r.rope_sin = rope_sin; r.pos0 = pos0; r.row_pos = row_pos;
    r.qd = qd; r.kvd = kvd; r.hd = hd; r.q_scale = q_scale;
    launch_splitk_reduce_qkv(part, splits, r, s);
    return splits;
}

void launch_gemm_fp8_qkv_rope(const unsigned char* A, int64_t lda, const float* sa, const unsigned char* Wqkv, int64_t ldw,
                              const float* sw, const bf16_t* bias, bf16_t* Q, bf16_t* Kd, bf16_t* Vt, int64_t ldv,
                              const float* rope_cos, const float* rope_sin, int64_t pos0, const int32_t* row_pos,
                              int64_t M, int qd, int kvd, int hd, int K, float q_scale, hipStream_t s) {
    if (M <= 0) return;
    GemmParams p = base_params(A, lda, sa, Wqkv, ldw, sw, M, qd + 2 * kvd, K);
    p.q_scale = q_scale;
    p.bias = bias; p.dst = Q; p.dst_k = Kd; p.dst_vt = Vt; p.ldv = ldv;
    p.rope_cos = rope_cos; p.rope_sin = rope_sin; p.pos0 = pos0; p.row_pos = row_pos;
    p.qd = qd; p.kvd = kvd; p.hd = hd;
    launch_t<EPI_QKV_ROPE>(p, s);
}

}  // namespace po
