// Causal grouped-query flash attention over one whole sequence, bf16 MFMA (gfx950).
//
// Section 4.2 of the paper keeps attention un-chunked ("prefill the attention layers
// normally"): one launch covers all N query positions; the N x N score matrix is never
// materialised (online softmax).
//
// Work split: one workgroup = BMQ = NW*QT*32 consecutive query rows of ONE query head;
// each wavefront owns QT tiles of 32 query rows.  K tiles (64 keys x hd) and V^T tiles
// (hd x 64 keys; V is stored transposed in HBM, so both MFMA operands are read from LDS
// with the contraction index contiguous) are staged global -> registers -> LDS, double
// buffered, and shared by all wavefronts of the group.
//
// The wavefront computes S^T = K Q^T (keys x queries) with v_mfma_f32_32x32x16_bf16, so
// that a lane owns ONE query column and 32 of the 64 keys of the tile: row max / row sum
// are in-lane reductions plus a single exchange with lane^32, the running rescale factor
// is a per-lane scalar, and the probabilities (rounded to bf16) are already in the layout
// of the B operand of O^T += V^T P^T.  To make the 8 keys a lane feeds to one MFMA
// contiguous in V^T, the K rows are read from LDS in a permuted order (bits 2 and 3 of
// the row index swapped): accumulator registers 0..7 of a lane then hold keys
// 8*(lane/32) .. +7 and registers 8..15 hold keys 16 + 8*(lane/32) .. +7 of a 32-key tile.
//
// Scheduling: query tiles are issued longest-first; when n_q_heads is a multiple of 8 all
// heads of one KV group are mapped to one XCD so that the group's K/V stream is shared in
// that XCD's L2.
#include "po_internal.h"

namespace po {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace {

constexpr int BNK = 64;   // keys per tile

__device__ __forceinline__ int swz8(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <int HD, int QT, int NW>
__global__ void __launch_bounds__(NW * 64) attn_fwd_kernel(const bf16_t* q, const bf16_t* __restrict__ k,
                                                           const bf16_t* __restrict__ vt, int64_t ldv, bf16_t* o,
                                                           int N, int Hq, int Hkv, float sc_log2e, int nqt,
                                                           int hpx) {
    constexpr int NT = NW * 64;
    constexpr int BMQ = NW * QT * 32;
    constexpr int KS = HD / 16;            // k-steps of S^T = K Q^T
    constexpr int HT = HD / 32;            // 32-row tiles of O^T
    constexpr int KSEG = HD / 8;           // 16-byte segments per K row
    constexpr int TILE_BYTES = BNK * HD * 2;   // K tile == V^T tile size
    constexpr int STAGE_BYTES = 2 * TILE_BYTES;
    constexpr int KLD = (BNK * KSEG) / NT;     // 16-byte loads per thread for K
    constexpr int VLD = (HD * 8) / NT;         // ... for V^T
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    int qtile, head;
    if (hpx > 0) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        qtile = nqt - 1 - j / hpx;
        head = xcd * hpx + j % hpx;
    } else {
        qtile = nqt - 1 - (int)(blockIdx.x / Hq);
        head = blockIdx.x % Hq;
    }
    const int kvh = head / (Hq / Hkv);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l31 = lane & 31, lhi = lane >> 5;
    const int qb = qtile * BMQ;
    const int qw = qb + wave * (QT * 32);
    const int blk_last = min(N, qb + BMQ) - 1;
    const int n_kv_blk = blk_last / BNK + 1;
    const int n_kv_wave = (qw < N) ? (min(N, qw + QT * 32) - 1) / BNK + 1 : 0;

    // ---- Q fragments (B operand: lane = query column, 8 consecutive head-dim values)
    bf16x8 qf[QT][KS];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int qrow = min(qw + qt * 32 + l31, N - 1);
        const bf16_t* qp = q + ((int64_t)qrow * Hq + head) * HD + lhi * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const uint4 t = *(const uint4*)(qp + ks * 16);
            qf[qt][ks] = __builtin_bit_cast(bf16x8, t);
        }
    }

    // ---- staging maps
    const int kseg = tid % KSEG, krow0 = tid / KSEG;           // rows krow0 + (NT/KSEG) i
    const int vseg = tid & 7, vrow0 = tid >> 3;                // rows vrow0 + (NT/8) i
    const bf16_t* kbase = k + (int64_t)kvh * HD + kseg * 8;
    const bf16_t* vbase = vt + (int64_t)kvh * HD * ldv + vseg * 8;
    const int64_t krs = (int64_t)Hkv * HD;
    // Prefetch registers, plain scalars so that they stay in VGPRs: set r holds the tile that
    // goes to LDS next, set n the one after it (prefetch distance 2, which covers the HBM/L2
    // latency of the K/V stream).  Loads are unconditional; tile indices clamp to the last tile.
    uint4 rk0, rk1, rk2, rk3, rv0, rv1, rv2, rv3, nk0, nk1, nk2, nk3, nv0, nv1, nv2, nv3;
    rk1 = rv1 = nk1 = nv1 = rk2 = rk3 = rv2 = rv3 = nk2 = nk3 = nv2 = nv3 = make_uint4(0, 0, 0, 0);
#define PO_KLOAD(i_) (*(const uint4*)(kbase + (int64_t)min(kv0_ + krow0 + (NT / KSEG) * (i_), N - 1) * krs))
#define PO_VLOAD(i_) (*(const uint4*)(vbase + (int64_t)(vrow0 + (NT / 8) * (i_)) * ldv + kv0_))
#define PO_GLOAD(P, j_)                                       \
    {                                                         \
        const int kv0_ = min((j_), n_kv_blk - 1) * BNK;       \
        P##k0 = PO_KLOAD(0);                                  \
        if (KLD > 1) P##k1 = PO_KLOAD(1);                     \
        if (KLD > 2) { P##k2 = PO_KLOAD(2); P##k3 = PO_KLOAD(3); } \
        P##v0 = PO_VLOAD(0);                                  \
        if (VLD > 1) P##v1 = PO_VLOAD(1);                     \
        if (VLD > 2) { P##v2 = PO_VLOAD(2); P##v3 = PO_VLOAD(3); } \
    }
#define PO_KST(i_, val_)                                                                         \
    {                                                                                            \
        const int row_ = krow0 + (NT / KSEG) * (i_);                                             \
        const int ps_ = (KSEG == 16) ? (kseg ^ (row_ & 15)) : (kseg ^ swz8(row_));               \
        *(uint4*)(sk_ + row_ * (HD * 2) + (ps_ << 4)) = val_;                                    \
    }
#define PO_VST(i_, val_)                                                                         \
    {                                                                                            \
        const int row_ = vrow0 + (NT / 8) * (i_);                                                \
        *(uint4*)(sv_ + row_ * 128 + ((vseg ^ swz8(row_)) << 4)) = val_;                         \
    }
#define PO_SSTORE(stage_)                                      \
    {                                                          \
        unsigned char* sk_ = smem + (stage_) * STAGE_BYTES;    \
        unsigned char* sv_ = sk_ + TILE_BYTES;                 \
        PO_KST(0, rk0);                                        \
        if (KLD > 1) PO_KST(1, rk1);                           \
        if (KLD > 2) { PO_KST(2, rk2); PO_KST(3, rk3); }       \
        PO_VST(0, rv0);                                        \
        if (VLD > 1) PO_VST(1, rv1);                           \
        if (VLD > 2) { PO_VST(2, rv2); PO_VST(3, rv3); }       \
    }

    // K fragment rows: MFMA row i of a 32-key tile holds key pi(i) (bits 2,3 swapped)
    const int pk = (l31 & 0x13) | ((l31 & 4) << 1) | ((l31 & 8) >> 1);
    const int k_sw = (KSEG == 16) ? (pk & 15) : swz8(pk);
    const int v_sw = swz8(l31);

    f32x16 oacc[HT][QT];
#pragma unroll
    for (int ht = 0; ht < HT; ++ht)
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[ht][qt][r] = 0.f;
    float mrow[QT], lrow[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) { mrow[qt] = -1.0e30f; lrow[qt] = 0.f; }

    PO_GLOAD(r, 0);
    PO_SSTORE(0);
    PO_GLOAD(r, 1);
    PO_GLOAD(n, 2);
    __syncthreads();
    for (int j = 0; j < n_kv_blk; ++j) {
        if (j < n_kv_wave) {
            const unsigned char* sk = smem + (j & 1) * STAGE_BYTES;
            const unsigned char* sv = sk + TILE_BYTES;
            const int kv0 = j * BNK;
            // ---- S^T = K Q^T  (2 key tiles x QT query tiles)
            f32x16 s[2][QT];
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[a][qt][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const bf16x8 kf = *(const bf16x8*)(sk + (a * 32 + pk) * (HD * 2) + (((ks * 2 + lhi) ^ k_sw) << 4));
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt)
                        s[a][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qt][ks], s[a][qt], 0, 0, 0);
                }
            }
            // ---- causal mask on tiles that touch the diagonal
            if (kv0 + BNK - 1 > qw) {
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    const int qidx = qw + qt * 32 + l31;
#pragma unroll
                    for (int a = 0; a < 2; ++a)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = kv0 + a * 32 + (r & 7) + 8 * lhi + 16 * (r >> 3);
                            if (key > qidx) s[a][qt][r] = -INFINITY;
                        }
                }
            }
            // ---- online softmax (per query column = per lane, partner lane^32)
            float mnew[QT];
            bool grew = false;
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                float mx = s[0][qt][0];
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[a][qt][r]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                mnew[qt] = fmaxf(mrow[qt], mx);
                grew |= mnew[qt] > mrow[qt];
            }
            if (__any(grew)) {      // rescale only when some running maximum moved (exact: else factor == 1)
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    const float alpha = __builtin_amdgcn_exp2f((mrow[qt] - mnew[qt]) * sc_log2e);
                    lrow[qt] *= alpha;
                    mrow[qt] = mnew[qt];
#pragma unroll
                    for (int ht = 0; ht < HT; ++ht)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[ht][qt][r] *= alpha;
                }
            }
            bf16x8 pf[QT][4];
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                const float mb = mrow[qt] * sc_log2e;
                float rs = 0.f;
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float pv = __builtin_amdgcn_exp2f(fmaf(s[a][qt][r], sc_log2e, -mb));
                        rs += pv;
                        pf[qt][a * 2 + (r >> 3)][r & 7] = (__bf16)pv;
                    }
                lrow[qt] += rs;
            }
            // ---- O^T += V^T P^T
#pragma unroll
            for (int j2 = 0; j2 < 4; ++j2) {
#pragma unroll
                for (int ht = 0; ht < HT; ++ht) {
                    const bf16x8 vf = *(const bf16x8*)(sv + (ht * 32 + l31) * 128 + (((j2 * 2 + lhi) ^ v_sw) << 4));
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt)
                        oacc[ht][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qt][j2], oacc[ht][qt], 0, 0, 0);
                }
            }
        }
        PO_SSTORE((j + 1) & 1);              // tile j+1 (loaded two iterations ago)
        rk0 = nk0; rk1 = nk1; rk2 = nk2; rk3 = nk3;
        rv0 = nv0; rv1 = nv1; rv2 = nv2; rv3 = nv3;
        PO_GLOAD(n, j + 3);
        __syncthreads();
    }
#undef PO_GLOAD
#undef PO_SSTORE
#undef PO_KLOAD
#undef PO_VLOAD
#undef PO_KST
#undef PO_VST

    // ---- normalise and store: lane = query row, registers = head-dim rows
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const float ltot = lrow[qt] + __shfl_xor(lrow[qt], 32);
        const float inv = 1.0f / ltot;
        const int qrow = qw + qt * 32 + l31;
        if (qrow < N) {
            bf16_t* op = o + ((int64_t)qrow * Hq + head) * HD + 4 * lhi;
#pragma unroll
            for (int ht = 0; ht < HT; ++ht)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    uint2 w;
                    w.x = (uint32_t)f2bf(oacc[ht][qt][rg * 4 + 0] * inv) | ((uint32_t)f2bf(oacc[ht][qt][rg * 4 + 1] * inv) << 16);
                    w.y = (uint32_t)f2bf(oacc[ht][qt][rg * 4 + 2] * inv) | ((uint32_t)f2bf(oacc[ht][qt][rg * 4 + 3] * inv) << 16);
                    *(uint2*)(op + ht * 32 + rg * 8) = w;
                }
        }
    }
}

template <int HD, int QT, int NW>
void launch_t(const bf16_t* q, const bf16_t* k, const bf16_t* vt, int64_t ldv, bf16_t* o, int64_t N, int Hq,
              int Hkv, hipStream_t s) {
    constexpr int BMQ = NW * QT * 32;
    constexpr int SMEM = 2 * 2 * BNK * HD * 2;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)attn_fwd_kernel<HD, QT, NW>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
        attr_set = true;
    }
    const int nqt = (int)((N + BMQ - 1) / BMQ);
    const int hpx = (Hq % 8 == 0) ? Hq / 8 : 0;
    const float sc_log2e = (float)(1.4426950408889634 / sqrt((double)HD));
    hipLaunchKernelGGL((attn_fwd_kernel<HD, QT, NW>), dim3((unsigned)(nqt * Hq)), dim3(NW * 64), SMEM, s, q, k, vt,
                       ldv, o, (int)N, Hq, Hkv, sc_log2e, nqt, hpx);
}

}  // namespace

bool attention_mfma_supported(int Hq, int Hkv, int hd) {
    return (hd == 128 || hd == 64) && Hkv > 0 && Hq % Hkv == 0;
}

void launch_attention_mfma(const bf16_t* q, const bf16_t* k, const bf16_t* vt, int64_t ldv, bf16_t* o, int64_t N,
                           int Hq, int Hkv, int hd, hipStream_t s) {
    if (N <= 0) return;
    if (hd == 128) launch_t<128, 1, 8>(q, k, vt, ldv, o, N, Hq, Hkv, s);
    else if (hd == 64) launch_t<64, 1, 8>(q, k, vt, ldv, o, N, Hq, Hkv, s);
}

}  // namespace po
