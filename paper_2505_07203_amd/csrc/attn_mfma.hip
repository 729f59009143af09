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

#include <algorithm>

namespace po {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace {

constexpr int BNK = 64;   // keys per tile

__device__ __forceinline__ int swz8(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// SPLIT (few query rows against many keys, e.g. a short suffix behind a long cached prefix): query tiles
// start at row q_row0, and the key tiles of a query tile are divided between n_split workgroups; each
// writes its unnormalised fp32 accumulators to opart[split][row - q_row0][head][HD] and its running
// maximum and row sum to mlpart[split][row - q_row0][head][2]; attn_combine_kernel merges them.
// The first n_tiles2 key tiles are read from a second K / V^T pair (k2, vt2 with pitch ldv2: a prefix-cache
// entry, same layouts), so that a cached prefix need not be copied next to the fresh keys first.
template <int HD, int QT, int NW, bool SPLIT>
__global__ void __launch_bounds__(NW * 64) attn_fwd_kernel(const bf16_t* q, const bf16_t* __restrict__ k,
                                                           const bf16_t* __restrict__ vt, int64_t ldv, bf16_t* o,
                                                           int N, int Hq, int Hkv, float sc_log2e, int nqt,
                                                           int hpx, int q_row0, int n_split, float* opart,
                                                           float* mlpart, const bf16_t* __restrict__ k2,
                                                           const bf16_t* __restrict__ vt2, int64_t ldv2, int n_tiles2,
                                                           int* redo) {
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

    // redo (not SPLIT): one word per (query tile, head), set for the tiles the 64-row kernel below gave up on.  A small
    // grid walks the words (workgroup b looks at b, b + gridDim.x, ...), recomputes the tiles whose word is set and
    // clears it again; with no word set, as for attention inputs of ordinary size, every workgroup reads a few words
    // and exits.
    int redo_item = (int)blockIdx.x;
next_redo_item:
    int qtile, head, split = 0;
    if (!SPLIT && redo) {
        const int total = nqt * Hq;
        while (redo_item < total && redo[redo_item] == 0) redo_item += (int)gridDim.x;
        if (redo_item >= total) return;
        qtile = redo_item / Hq;
        head = redo_item % Hq;
    } else if (SPLIT) {
        split = blockIdx.x % n_split;
        const int rest = blockIdx.x / n_split;
        head = rest % Hq;
        qtile = rest / Hq;
    } else if (hpx > 0) {
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
    const int qb = (SPLIT ? q_row0 : 0) + qtile * BMQ;
    const int qw = qb + wave * (QT * 32);
    const int blk_last = min(N, qb + BMQ) - 1;
    const int n_kv_blk = blk_last / BNK + 1;
    const int n_kv_wave = (qw < N) ? (min(N, qw + QT * 32) - 1) / BNK + 1 : 0;
    // this workgroup's key tiles [j_begin, j_end)
    const int per_split = SPLIT ? (n_kv_blk + n_split - 1) / n_split : n_kv_blk;
    const int j_begin = SPLIT ? min(split * per_split, n_kv_blk) : 0;
    const int j_end = SPLIT ? min(j_begin + per_split, n_kv_blk) : n_kv_blk;

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
    const bf16_t* kbase2 = SPLIT ? k2 + (int64_t)kvh * HD + kseg * 8 : kbase;
    const bf16_t* vbase2 = SPLIT ? vt2 + (int64_t)kvh * HD * ldv2 + vseg * 8 : vbase;
    const int64_t krs = (int64_t)Hkv * HD;
    // Prefetch registers, plain scalars so that they stay in VGPRs: set r holds the tile that
    // goes to LDS next, set n the one after it (prefetch distance 2, which covers the HBM/L2
    // latency of the K/V stream).  Loads are unconditional; tile indices clamp to the last tile.
    uint4 rk0, rk1, rk2, rk3, rv0, rv1, rv2, rv3, nk0, nk1, nk2, nk3, nv0, nv1, nv2, nv3;
    rk1 = rv1 = nk1 = nv1 = rk2 = rk3 = rv2 = rv3 = nk2 = nk3 = nv2 = nv3 = make_uint4(0, 0, 0, 0);
#define PO_KLOAD(i_) (*(const uint4*)(kb_ + (int64_t)min(kv0_ + krow0 + (NT / KSEG) * (i_), N - 1) * krs))
#define PO_VLOAD(i_) (*(const uint4*)(vb_ + (int64_t)(vrow0 + (NT / 8) * (i_)) * ld_ + kv0_))
#define PO_GLOAD(P, j_)                                       \
    {                                                         \
        const int jt_ = min((j_), n_kv_blk - 1);              \
        const int kv0_ = jt_ * BNK;                           \
        const bool second_ = SPLIT && jt_ < n_tiles2;         \
        const bf16_t* kb_ = second_ ? kbase2 : kbase;         \
        const bf16_t* vb_ = second_ ? vbase2 : vbase;         \
        const int64_t ld_ = second_ ? ldv2 : ldv;             \
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

    PO_GLOAD(r, j_begin);
    PO_SSTORE(0);
    PO_GLOAD(r, j_begin + 1);
    PO_GLOAD(n, j_begin + 2);
    __syncthreads();
    for (int j = j_begin; j < j_end; ++j) {
        if (j < n_kv_wave) {
            const unsigned char* sk = smem + ((j - j_begin) & 1) * STAGE_BYTES;
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
        PO_SSTORE((j - j_begin + 1) & 1);    // tile j+1 (loaded two iterations ago)
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
        if (SPLIT) {
            if (qrow < N) {
                const int64_t slot = ((int64_t)split * (N - q_row0) + (qrow - q_row0)) * Hq + head;
                float* op = opart + slot * HD + 4 * lhi;
#pragma unroll
                for (int ht = 0; ht < HT; ++ht)
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const float4 v = {oacc[ht][qt][rg * 4 + 0], oacc[ht][qt][rg * 4 + 1], oacc[ht][qt][rg * 4 + 2],
                                          oacc[ht][qt][rg * 4 + 3]};
                        *(float4*)(op + ht * 32 + rg * 8) = v;
                    }
                if (lhi == 0) *(float2*)(mlpart + slot * 2) = make_float2(mrow[qt], ltot);
            }
            continue;
        }
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
    if (!SPLIT && redo) {
        if (tid == 0) redo[redo_item] = 0;
        __syncthreads();                 // every wavefront is done with the LDS stages before the next tile refills them
        redo_item += (int)gridDim.x;
        goto next_redo_item;
    }
}


// ---------------------------------------------------------------------------------------
// Head dimension 128: 64 query rows per wavefront, one wavefront per SIMD.
//
// The kernel above reads one 1 KiB LDS fragment per MFMA (32 query rows per wavefront), which
// at full matrix rate is the whole LDS bandwidth of the CU.  Here a wavefront owns TWO
// 32-row query tiles, so every K and V^T fragment feeds two MFMAs.  With 4 wavefronts x 64
// rows there is a single wavefront per SIMD, so the softmax arithmetic has to run in the
// shadow of the SAME wavefront's MFMAs; the loop is software-pipelined over blocks of 32 keys:
//
//   iteration i, first half : 16 MFMA  S(i+1) = K(i+1) Q^T      | VALU: 24 of the 32 P(i) = exp2(S(i) - r)
//   iteration i, second half: 16 MFMA  O^T += V^T(i) P(i)^T      | VALU: the other 8, row sums of P(i)
// MFMAs and their LDS fragment reads are written one by one with a slice of the vector work
// behind each (scheduling fences keep that order).
//
// Reference exponent instead of a running maximum.  Every vector instruction issued between
// MFMAs delays the next MFMA by a few cycles (measured: the two do not overlap within a
// wavefront), so the per-score instruction count is what bounds this kernel, and the block
// maximum of the usual online softmax is 18 instructions per block that only guard the number
// range.  Here a query row keeps ONE reference r (the maximum over its first 32 keys, which
// include key 0) and accumulates p = exp2(s - r) in fp32 as it stands: softmax is invariant to
// r, bf16 has the fp32 exponent range, so p > 1 is harmless.  The row sum is watched instead:
// when it passes 2^40 the sums and accumulators are multiplied by an exact power of two and
// r moves by that exponent (rare: not once with the workloads here).  Terms below 2^-126
// relative to r underflow exactly as they would against the true maximum once it is larger.
// A score more than about 127 log2 units (88 nats) above the reference, within a single block, makes its
// exponential overflow before the watch can move the reference.  The row sum then is infinite (every p is
// non-negative, so nothing cancels), which the same watch sees: a row sum that is not below 2^100 after a block
// marks the wavefront's tile as given up.  At the end the four wavefronts agree (one word of LDS); a workgroup
// that gave up stores NOTHING (its query rows, which the output overwrites, stay intact) and sets its word in
// `redo`, and a second launch right behind this one recomputes exactly those (query tile, head) pairs with the
// running-maximum kernel above, which is total on finite inputs.  With `redo` all zero, as it is for attention
// inputs of ordinary size, that launch is a few thousand workgroups that read one word and exit.
//
// Two wavefronts per SIMD do not help here.  A copy of this kernel with eight wavefronts of 32 query rows (each K /
// V^T fragment then feeds one MFMA) was built and is exact, but 7 % slower: vector instructions of one wavefront do
// not run under the MFMAs of the other either (timing-only copies: the exponentials cost 0.20, the multiply-adds
// 0.13, conversions and row sums 0.12 of the MFMA time, all of it added on top), and with one fragment read per MFMA
// the LDS, not the softmax, bounds that layout (74 % MFMA-busy with NO softmax arithmetic at all).  Folding the
// softmax scale into Q (to drop the multiply-add per score) rounds Q to bf16 a second time, which scores of a few
// hundred make visible (2.5e-2 against 3e-3), so the scale stays in fp32; and with Q scaled before its one rounding
// (in the projection's epilogue) and the S accumulators started from minus the reference exponent, the multiply-adds
// do go, but the first MFMA of a block then needs its addend copied into the accumulator registers (the two are
// tied in this register form), 32 moves for 32 multiply-adds: measured 6 % slower in this kernel's schedule.
//
// LDS holds the K tiles of the four stages in its first 64 KiB and the V^T tiles in the second: with
// the stage number known at compile time (main loop unrolled over the four stages) every fragment
// address is a fixed per-lane register plus an immediate offset below 64 KiB.
// K (64 keys x 256 B) and V^T (128 rows x 128 B) tiles go global -> LDS directly
// (global_load_lds, 16 B per lane) through a ring of four 32 KiB stages, three tiles ahead;
// the XOR swizzles of the kernel above are applied on the global side of the copy.  One
// workgroup barrier per 64-key tile hands a stage over.
constexpr int A64_TILE = 64 * 128 * 2;          // one K tile or one V^T tile: 16 KiB
constexpr int A64_NSTAGE = 4;
constexpr int A64_VBASE = A64_NSTAGE * A64_TILE; // LDS: the four K tiles, then the four V^T tiles

__device__ __forceinline__ float half_swap_max(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

// PRE: the caller has multiplied Q by log2(e) / sqrt(hd) before rounding it to bf16 (the QKV projection's epilogue
// does, in fp32: Q is rounded once, as before).  K Q^T then IS the exponent's argument, and no reference exponent is
// subtracted at all: p = exp2(s) as it comes out of the matrix pipe, no multiply-add per score.  fp32 and bf16 hold
// 2^-126 .. 2^127, attention scores of ordinary size are within +-40, and a row whose sum of p leaves 2^-60 .. 2^100
// (scores far above or far below that) gives up and is recomputed by the running-maximum kernel, like an overflow
// in the other form.
template <bool PRE>
__global__ void __launch_bounds__(256) attn_fwd64_kernel(const bf16_t* q, const bf16_t* __restrict__ k,
                                                         const bf16_t* __restrict__ vt, int64_t ldv, bf16_t* o, int N,
                                                         int Hq, int Hkv, float sc_log2e, int nqt, int hpx, int* redo) {
    constexpr int HD = 128, KS = 8, HT = 4;
    constexpr int TILE_BYTES = 64 * HD * 2;
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
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, lhi = lane >> 5;
    const int qb = qtile * 256;
    const int qw = qb + wave * 64;
    const int blk_last = min(N, qb + 256) - 1;
    const int n_tiles = blk_last / 64 + 1;                       // 64-key tiles the workgroup streams
    const int nkb_w = (qw < N) ? (min(N, qw + 64) - 1) / 32 + 1 : 0;   // 32-key blocks this wavefront needs

    // ---- Q fragments (B operand: lane = query column, 8 consecutive head-dim values)
    bf16x8 qf[2][KS];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const int qrow = min(qw + qt * 32 + l31, N - 1);
        const bf16_t* qp = q + ((int64_t)qrow * Hq + head) * HD + lhi * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const uint4 t = *(const uint4*)(qp + ks * 16);
            qf[qt][ks] = __builtin_bit_cast(bf16x8, t);
        }
    }

    // ---- global -> LDS copy maps.  K: round jj (0..3) of wavefront w fills rows jj*16 + w*4 .. +3
    // (16 lanes per 256-byte row); V^T: round jj fills rows jj*32 + w*8 .. +7 (8 lanes per row).
    // Lane l writes physical segment l % 16 (l % 8), so it fetches the logical segment that the
    // swizzle maps there.
    const int krow_l = wave * 4 + (lane >> 4);
    const uint32_t kcol = (uint32_t)(((lane & 15) ^ (krow_l & 15)) << 4);
    const uint32_t krs2 = (uint32_t)(Hkv * HD * 2);
    const uint32_t klane = (uint32_t)krow_l * krs2 + kcol;
    const int vrow_l = wave * 8 + (lane >> 3);
    const uint32_t voff_v = (uint32_t)vrow_l * (uint32_t)(ldv * 2) + (uint32_t)(((lane & 7) ^ swz8(vrow_l)) << 4);
    // K goes through a buffer resource that ends with the last position: rows of the last, ragged tile
    // beyond it read as zero (they are masked keys) instead of needing a clamp per load.
    const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(k + (int64_t)kvh * HD), 0, (int)((uint32_t)(N - 1) * krs2 + 256u), 0x00020000);
    // (V^T of this KV head: 128 rows of ldv positions; its columns are always inside the row)
    const __amdgpu_buffer_rsrc_t vrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(vt + (int64_t)kvh * HD * ldv), 0, (int)((uint32_t)HD * (uint32_t)(ldv * 2)), 0x00020000);
    const uint32_t vrow32 = (uint32_t)(32 * ldv * 2);
    // load jj_ (0..3: K rows, 4..7: V^T rows) of tile tile_ into stage stg_
#define PO_DMA(tile_, stg_, jj_)                                                                               \
    {                                                                                                          \
        const int kv0_ = min((tile_), n_tiles - 1) * 64;                                                       \
        if ((jj_) < 4) {                                                                                       \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                          \
                krsrc, (__attribute__((address_space(3))) void*)(smem + (stg_) * A64_TILE + ((jj_) * 16 + wave * 4) * 256), \
                16, klane, (kv0_ + (jj_) * 16) * krs2, 0, 0);                                                  \
        } else {                                                                                               \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                          \
                vrsrc, (__attribute__((address_space(3))) void*)(smem + A64_VBASE + (stg_) * A64_TILE +        \
                                                                 (((jj_) - 4) * 32 + wave * 8) * 128),          \
                16, voff_v, ((jj_) - 4) * vrow32 + kv0_ * 2, 0, 0);                                            \
        }                                                                                                      \
    }

    // ---- LDS fragment addresses
    const int pk = (l31 & 0x13) | ((l31 & 4) << 1) | ((l31 & 8) >> 1);   // K rows read permuted (see above)
    uint32_t koff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = pk * 256 + (((ks * 2 + lhi) ^ (pk & 15)) << 4);
    uint32_t vofs[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int j2 = 0; j2 < 2; ++j2)      // (the V^T half of LDS starts at 64 KiB: in the register, so that what is left is an immediate)
            vofs[a][j2] = A64_VBASE + l31 * 128 + (((a * 4 + j2 * 2 + lhi) ^ swz8(l31)) << 4);

    f32x16 oacc[HT][2];
#pragma unroll
    for (int ht = 0; ht < HT; ++ht)
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[ht][qt][r] = 0.f;
    float mb[2], lrow[2] = {0.f, 0.f};      // reference exponents (log2 domain) and row sums per query tile
    float lsum[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};       // PRE: the row sums as four partial sums each
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    int gave_up = 0;                        // wavefront-uniform: a row sum left the range the reference scheme covers
    int* const lds_gave_up = (int*)(smem + 2 * A64_NSTAGE * A64_TILE);     // one word behind the ring
    if (tid == 0) *lds_gave_up = 0;         // (read only after the last of the barriers below)

    // causal mask of a 32-key block on the accumulators of one query tile
#define PO_MASK(S, kb_, qt_)                                                                     \
    {                                                                                            \
        const int qidx_ = qw + (qt_) * 32 + l31;                                                 \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                         \
            const int key_ = (kb_) * 32 + (r & 7) + 8 * lhi + 16 * (r >> 3);                     \
            if (key_ > qidx_) S[qt_][r] = -INFINITY;                                             \
        }                                                                                        \
    }
#define PO_BLOCKMAX(S, qt_, out_)                                                                \
    {                                                                                            \
        float m0_ = fmaxf(fmaxf(S[qt_][0], S[qt_][1]), S[qt_][2]);                               \
        float m1_ = fmaxf(fmaxf(S[qt_][3], S[qt_][4]), S[qt_][5]);                               \
        m0_ = fmaxf(fmaxf(m0_, S[qt_][6]), S[qt_][7]);                                           \
        m1_ = fmaxf(fmaxf(m1_, S[qt_][8]), S[qt_][9]);                                           \
        m0_ = fmaxf(fmaxf(m0_, S[qt_][10]), S[qt_][11]);                                         \
        m1_ = fmaxf(fmaxf(m1_, S[qt_][12]), S[qt_][13]);                                         \
        m0_ = fmaxf(fmaxf(m0_, S[qt_][14]), S[qt_][15]);                                         \
        out_ = half_swap_max(fmaxf(m0_, m1_));                                                   \
    }

    // ---- prologue: three tiles in flight, S(0), reference maxima
    _Pragma("unroll") for (int jj = 0; jj < 8; ++jj) PO_DMA(0, 0, jj);
    _Pragma("unroll") for (int jj = 0; jj < 8; ++jj) PO_DMA(1, 1, jj);
    _Pragma("unroll") for (int jj = 0; jj < 8; ++jj) PO_DMA(2, 2, jj);
    asm volatile("s_waitcnt vmcnt(16)\n\ts_barrier" ::: "memory");      // Q fragments and tile 0 have landed

    f32x16 sa[2], sb[2];
    bf16x8 pf[2][2], fr[4];
    {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 kf = *(const bf16x8*)(smem + koff[ks]);
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                if (ks == 0) {
                    const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    sa[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qt][ks], z, 0, 0, 0);
                } else {
                    sa[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qt][ks], sa[qt], 0, 0, 0);
                }
            }
        }
        if (31 > qw) { PO_MASK(sa, 0, 0); PO_MASK(sa, 0, 1); }
        float m0 = 0.f, m1 = 0.f;
        if (!PRE) {
            PO_BLOCKMAX(sa, 0, m0);
            PO_BLOCKMAX(sa, 1, m1);
        }
        mb[0] = m0 * sc_log2e;
        mb[1] = m1 * sc_log2e;
    }

    // Register files.  The vector ALU reaches only the 256 architectural registers; S must live there
    // (softmax), the O^T accumulators (128 registers, touched by MFMAs only) must not.  The compiler puts
    // the results of ALL MFMA builtins of a function in one file or the other, so the S products use the
    // builtin (built with -amdgpu-mfma-vgpr-form: architectural registers) and the O^T products are
    // written as an instruction with accumulation-register constraints.  The compiler does not know that
    // instruction's latency, so before the vector ALU reads O^T (rescale, epilogue) the pipe is drained
    // by hand; MFMA-to-MFMA accumulation on the same registers needs no software wait.
#define PO_MFMA_ACC(ACC, A_, B_) \
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(ACC) : "v"(A_), "v"(B_))
#define PO_MFMA_DRAIN() asm volatile("s_nop 15\n\ts_nop 15" ::: "memory")
    // One iteration over key block i_: SC holds S(i_), SN receives S(i_+1).  It is a chain of 16 steps,
    // each one LDS fragment feeding two MFMAs (steps 0..7: K rows of block i_+1 at KST_/KA_; steps 8..15:
    // V^T of block i_ at VST_/VA_, 16-key half outermost); the fragment of step c+3 is requested right
    // after the first MFMA of step c, into the register step c-1 has just finished with (steps 13..15
    // request the first three K fragments of the next iteration, at NKST_/NKA_).
    //   BAR_: the hand-over barrier sits between the two halves of this iteration.
    //   DMA_T_/DMA_J0_: four global->LDS loads ride on steps 9, 11, 13, 15.
    // The compiler waits for ALL LDS reads in flight before an MFMA written as an instruction (it does
    // not work out which read feeds it).  Three fragment reads are in flight at the first MFMA of a step
    // and LDS reads return in order, so an explicit wait for "all but the two youngest" in front of it
    // is exact, and the compiler, which does account for explicit waits, then adds none.
#define PO_FRAG_ADDR(c_, KST_, KA_, VST_, VA_, NKST_, NKA_)                                                     \
    ((c_) < 8 ? (KST_) + (KA_) * 8192 + koff[(c_) & 7]                                                          \
              : (c_) < 16 ? (VST_) + (((c_) - 8) & 3) * 4096 + vofs[VA_][((c_) - 8) >> 2]                       \
                          : (NKST_) + (NKA_) * 8192 + koff[(c_) & 7])
#define PO_WAIT_LGKM2() __builtin_amdgcn_s_waitcnt(0xC27F)     /* lgkmcnt(2), other counters untouched */
    // job whose exponentials are issued in MFMA slot s_ (-1: none), and the first of its two values
#define PO_JOB_AT(s_) ((s_) < 0 ? -1 : (s_) < 8 ? (s_) : (s_) < 16 ? (((s_) & 1) ? -1 : 8 + ((s_) - 8) / 2) \
                       : (((s_) < 24 && !((s_) & 1)) ? 12 + ((s_) - 16) / 2 : -1))
#define PO_JOB_E(n_) ((n_) < 4 ? 2 * (n_) : (n_) < 8 ? 16 + 2 * ((n_) - 4) : (n_) < 12 ? 8 + 2 * ((n_) - 8) : 24 + 2 * ((n_) - 12))
#define PO_EXP_ARG(n_, SC, mb0_, mb1_)                                                             \
    {                                                                                              \
        const int e_ = PO_JOB_E((n_) & 15);                                                        \
        const float mb_ = (e_ >> 4) ? mb1_ : mb0_;                                                 \
        ea_[(n_) & 15][0] = fmaf(SC[e_ >> 4][e_ & 15], sc_log2e, -mb_);                            \
        ea_[(n_) & 15][1] = fmaf(SC[e_ >> 4][(e_ & 15) + 1], sc_log2e, -mb_);                      \
    }
#define PO_ITER(i_, SC, SN, KST_, KA_, VST_, VA_, NKST_, NKA_, BAR_, DMA_T_, DMA_S_, DMA_J0_, MASK_)            \
    {                                                                                                           \
        const float mb0_ = mb[0], mb1_ = mb[1];                                                                 \
        float ea_[16][2];                                                                                       \
        _Pragma("unroll") for (int c = 0; c < 16; ++c) {                                                        \
            if (c == 8) {                                                                                       \
                if (MASK_) {                                                                                    \
                    PO_MASK(SN, (i_) + 1, 0);                                                                   \
                    PO_MASK(SN, (i_) + 1, 1);                                                                   \
                }                                                                                               \
                if (BAR_) asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");                         \
                __builtin_amdgcn_sched_barrier(0);                                                              \
            }                                                                                                   \
            PO_WAIT_LGKM2();                                                                                    \
            __builtin_amdgcn_sched_barrier(0);                                                                  \
            _Pragma("unroll") for (int qt = 0; qt < 2; ++qt) {                                                  \
                if (c < 8) {                                                                                    \
                    if (c == 0) {                                                                               \
                        const f32x16 z_ = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}; \
                        SN[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[c & 3], qf[qt][c & 7], z_, 0, 0, 0); \
                    } else {                                                                                    \
                        SN[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[c & 3], qf[qt][c & 7], SN[qt], 0, 0, 0); \
                    }                                                                                           \
                } else {                                                                                        \
                    PO_MFMA_ACC(oacc[(c - 8) & 3][qt], fr[c & 3], pf[qt][(c - 8) >> 2]);                        \
                }                                                                                               \
                __builtin_amdgcn_sched_barrier(0);                                                              \
                if (qt == 0) {                                                                                  \
                    fr[(c + 3) & 3] = *(const bf16x8*)PO_FRAG_ADDR(c + 3, KST_, KA_, VST_, VA_, NKST_, NKA_);   \
                    __builtin_amdgcn_sched_barrier(0);                                                          \
                }                                                                                               \
                /* Probabilities of S(i): 16 jobs of two values (one packed conversion each).  The            \
                   exponential is a quarter-rate instruction, so 12 jobs go into the first half (slots 0..7:    \
                   the 16 values the first four V^T steps need; slots 8, 10, 12, 14: query tile 0, registers    \
                   8..15) and 4 (query tile 1, registers 8..15, needed from V^T step 4 on) into slots 16, 18,   \
                   20, 22.  Each job is spread over three MFMA slots (exponent arguments | exponentials |       \
                   conversion) so that no instruction waits for the one issued just before it. */               \
                const int slot_ = 2 * c + qt;                    /* 0..31 over the iteration */                 \
                {                                                                                               \
                    const int na_ = PO_JOB_AT(slot_ + 1), nb_ = PO_JOB_AT(slot_), nc_ = PO_JOB_AT(slot_ - 1);   \
                    if (!PRE && slot_ == 0) { PO_EXP_ARG(0, SC, mb0_, mb1_); }                                  \
                    if (!PRE && na_ > 0) { PO_EXP_ARG(na_, SC, mb0_, mb1_); }                                   \
                    if (nb_ >= 0) {                                                                             \
                        /* PRE: the accumulator IS the exponent's argument */                                   \
                        const int eb_ = PO_JOB_E(nb_ & 15);                                                     \
                        ea_[nb_ & 15][0] = __builtin_amdgcn_exp2f(PRE ? SC[eb_ >> 4][eb_ & 15] : ea_[nb_ & 15][0]);       \
                        ea_[nb_ & 15][1] = __builtin_amdgcn_exp2f(PRE ? SC[eb_ >> 4][(eb_ & 15) + 1] : ea_[nb_ & 15][1]); \
                    }                                                                                           \
                    if (nc_ >= 0) {                                                                             \
                        const int e_ = PO_JOB_E(nc_ & 15);                                                      \
                        pf[e_ >> 4][(e_ & 15) >> 3][e_ & 7] = (__bf16)ea_[nc_ & 15][0];                         \
                        pf[e_ >> 4][(e_ & 15) >> 3][(e_ & 7) + 1] = (__bf16)ea_[nc_ & 15][1];                   \
                    }                                                                                           \
                }                                                                                               \
                if (c >= 8) {                                                                                   \
                    const int c_ = (c - 8) * 2 + qt;             /* 0..15 */                                    \
                    if (c_ == 8 || c_ == 9) {                                                                   \
                        const int sq_ = c_ - 8;                                                                 \
                        /* four independent chains: a dependent dot product waits about 6 cycles.  PRE: the     \
                           four partial sums live across blocks (nothing looks at the row sum before the end) */\
                        float l_[4] = {lrow[sq_], 0.f, 0.f, 0.f};                                               \
                        _Pragma("unroll") for (int h2 = 0; h2 < 2; ++h2)                                        \
                        _Pragma("unroll") for (int e2 = 0; e2 < 4; ++e2) {                                      \
                            const bf16x2 pr2_ = {pf[sq_][h2][2 * e2], pf[sq_][h2][2 * e2 + 1]};                 \
                            if (PRE) lsum[sq_][e2] = __builtin_amdgcn_fdot2_f32_bf16(pr2_, ones, lsum[sq_][e2], false); \
                            else l_[e2] = __builtin_amdgcn_fdot2_f32_bf16(pr2_, ones, l_[e2], false);           \
                        }                                                                                       \
                        if (!PRE) lrow[sq_] = (l_[0] + l_[1]) + (l_[2] + l_[3]);                                \
                    }                                                                                           \
                    if ((c_ & 3) == 3) { PO_DMA(DMA_T_, DMA_S_, (DMA_J0_) + (c_ >> 2)); }                       \
                }                                                                                               \
                __builtin_amdgcn_sched_barrier(0);                                                              \
            }                                                                                                   \
        }                                                                                                       \
        /* ---- renormalise when a row sum has grown past 2^40 (rare; see the note on the reference) */         \
        /* (PRE: nothing to watch.  The sums only grow, an overflow stays an overflow: one look at the end does) */ \
        if (!PRE && __any(!(lrow[0] <= 0x1p40f) || !(lrow[1] <= 0x1p40f))) {                                    \
            const float t0_ = half_swap_sum(lrow[0]), t1_ = half_swap_sum(lrow[1]);                             \
            if (__any(!(t0_ < 0x1p100f) || !(t1_ < 0x1p100f))) gave_up = 1;                                     \
            int e0_ = ilogbf(t0_), e1_ = ilogbf(t1_);                                                           \
            asm volatile("" : "+v"(e0_), "+v"(e1_));   /* keeps the rescale inside this rarely taken branch */  \
            PO_MFMA_DRAIN();                                                                                    \
            const float a0_ = ldexpf(1.0f, -e0_), a1_ = ldexpf(1.0f, -e1_);                                     \
            mb[0] += (float)e0_;                                                                                \
            mb[1] += (float)e1_;                                                                                \
            lrow[0] *= a0_;                                                                                     \
            lrow[1] *= a1_;                                                                                     \
            _Pragma("unroll") for (int ht = 0; ht < HT; ++ht)                                                   \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) { oacc[ht][0][r] *= a0_; oacc[ht][1][r] *= a1_; }    \
        }                                                                                                       \
    }

    // Pair j = key blocks 2j, 2j+1 (one 64-key tile).  Block 2j multiplies with K of block 2j+1 (tile j,
    // second half) and V^T of block 2j (tile j, first half); block 2j+1 with K of block 2j+2 (tile j+1,
    // first half) and V^T of block 2j+1.  Hand-over between the halves of block 2j: tile j+1 has landed
    // (the 8 loads of tile j+2 may still be in flight) and every wavefront is done with tile j-1, whose
    // stage the loads of tile j+3 overwrite: its K rows ride on the rest of block 2j, its V^T rows on
    // block 2j+1.  The causal mask touches S(i+1) only in the last three blocks of a wavefront
    // (i + 1 >= qw / 32), so the loop is split by pair into: no mask | second block masked | both masked |
    // nothing left to compute (the wavefront still copies its share and meets the barriers).
    // s_ = j & 3: the stage of tile j (a literal in the unrolled main loop, so that every LDS address
    // below is a lane register plus an immediate)
#define PO_PAIR(s_, M0_, M1_)                                                                      \
    {                                                                                              \
        const unsigned char* kst = smem + (s_) * A64_TILE;                                         \
        const unsigned char* kstn = smem + (((s_) + 1) & 3) * A64_TILE;                            \
        const unsigned char* vst = smem + (s_) * A64_TILE;                  /* (+ A64_VBASE, in vofs) */ \
        PO_ITER(2 * j, sa, sb, kst, 1, vst, 0, kstn, 0, 1, j + 3, ((s_) + 3) & 3, 0, M0_);         \
        PO_ITER(2 * j + 1, sb, sa, kstn, 0, vst, 1, kstn, 1, 0, j + 3, ((s_) + 3) & 3, 4, M1_);    \
    }
    const int wt = qw >> 6;                      // pair that holds this wavefront's first query row
    const int j_last = (nkb_w > 0) ? wt : -1;    // last pair with work
    fr[0] = *(const bf16x8*)(smem + 8192 + koff[0]);      // K fragments 0, 1, 2 of block 1
    fr[1] = *(const bf16x8*)(smem + 8192 + koff[1]);
    fr[2] = *(const bf16x8*)(smem + 8192 + koff[2]);
    int j = 0;
    for (; j + 4 <= j_last - 1; j += 4) {
        PO_PAIR(0, 0, 0);
        ++j;
        PO_PAIR(1, 0, 0);
        ++j;
        PO_PAIR(2, 0, 0);
        ++j;
        PO_PAIR(3, 0, 0);
        j -= 3;
    }
    for (; j < j_last - 1; ++j) PO_PAIR(j & 3, 0, 0);
    if (j == j_last - 1) { PO_PAIR(j & 3, 0, 1); ++j; }
    if (j == j_last) { PO_PAIR(j & 3, 1, 1); ++j; }
    for (; j < n_tiles; ++j) {
        asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
        _Pragma("unroll") for (int jj = 0; jj < 8; ++jj) PO_DMA(j + 3, (j + 3) & 3, jj);
    }
#undef PO_PAIR
#undef PO_FRAG_ADDR
#undef PO_WAIT_LGKM2
#undef PO_ITER
#undef PO_JOB_AT
#undef PO_JOB_E
#undef PO_EXP_ARG
#undef PO_DMA
#undef PO_MASK
#undef PO_BLOCKMAX
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    PO_MFMA_DRAIN();
#undef PO_MFMA_ACC
#undef PO_MFMA_DRAIN

    if (PRE) {
        lrow[0] = (lsum[0][0] + lsum[0][1]) + (lsum[0][2] + lsum[0][3]);
        lrow[1] = (lsum[1][0] + lsum[1][1]) + (lsum[1][2] + lsum[1][3]);
        // a row sum of 2^100 or more (or infinite) means probabilities near or past the top of the float range; one
        // below 2^-60 that the row's scores sit so far below zero that terms were flushed away
        const float t0 = half_swap_sum(lrow[0]), t1 = half_swap_sum(lrow[1]);
        if (nkb_w > 0 && __any(!(t0 >= 0x1p-60f) || !(t0 < 0x1p100f) || !(t1 >= 0x1p-60f) || !(t1 < 0x1p100f))) gave_up = 1;
    }
    // ---- did any wavefront give up?  (every wavefront has met the same number of barriers and arrives here)
    if (gave_up && lane == 0) *(volatile int*)lds_gave_up = 1;
    __syncthreads();
    if (*(volatile int*)lds_gave_up) {
        if (tid == 0) redo[qtile * Hq + head] = 1;
        return;
    }

    // ---- normalise and store: lane = query row, registers = head-dim rows
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const float inv = 1.0f / half_swap_sum(lrow[qt]);
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

// o[row][head][:] = sum_s w_s O_s / sum_s w_s l_s with w_s = 2^((m_s - max m) sc_log2e); one thread per 4 values.
template <int HD>
__global__ void __launch_bounds__(256) attn_combine_kernel(const float* __restrict__ opart, const float* __restrict__ mlpart,
                                                           int n_split, int nq, int Hq, float sc_log2e, bf16_t* o,
                                                           int q_row0) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    constexpr int PER = HD / 4;
    if (i >= (int64_t)nq * Hq * PER) return;
    const int64_t rh = i / PER;                       // (row - q_row0) * Hq + head
    const int f = (int)(i - rh * PER) * 4;
    const int64_t plane = (int64_t)nq * Hq;
    float mx = -1.0e30f;
    for (int sp = 0; sp < n_split; ++sp) mx = fmaxf(mx, mlpart[(sp * plane + rh) * 2]);
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
    for (int sp = 0; sp < n_split; ++sp) {
        const float2 ml = *(const float2*)(mlpart + (sp * plane + rh) * 2);
        const float w = __builtin_amdgcn_exp2f((ml.x - mx) * sc_log2e);
        const float4 v = *(const float4*)(opart + (sp * plane + rh) * HD + f);
        acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
        l += w * ml.y;
    }
    const float inv = 1.0f / l;
    const int64_t row = q_row0 + rh / Hq;
    const int head = (int)(rh % Hq);
    uint2 w2;
    w2.x = (uint32_t)f2bf(acc.x * inv) | ((uint32_t)f2bf(acc.y * inv) << 16);
    w2.y = (uint32_t)f2bf(acc.z * inv) | ((uint32_t)f2bf(acc.w * inv) << 16);
    *(uint2*)(o + (row * Hq + head) * HD + f) = w2;
}

void launch_fwd64(const bf16_t* q, const bf16_t* k, const bf16_t* vt, int64_t ldv, bf16_t* o, int64_t N, int Hq,
                  int Hkv, int64_t q_row0, int* redo, bool q_prescaled, hipStream_t s) {
    constexpr int SMEM = 2 * A64_NSTAGE * A64_TILE + 16;             // the ring and the give-up word
    constexpr int SMEM_REDO = 2 * 2 * BNK * 128 * 2;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)attn_fwd64_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
        (void)hipFuncSetAttribute((const void*)attn_fwd64_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
        (void)hipFuncSetAttribute((const void*)attn_fwd_kernel<128, 1, 8, false>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_REDO);
        attr_set = true;
    }
    const int nqt = (int)((N + 255) / 256);
    const int hpx = (Hq % 8 == 0) ? Hq / 8 : 0;
    const float sc_log2e = q_prescaled ? 1.0f : attention_q_scale(128);
    // workgroups enumerate query tiles from the last one down: fewer of them = only the last tiles
    const int nsel = nqt - (int)((q_row0 > 0 && q_row0 < N) ? q_row0 / 256 : 0);
    if (q_prescaled)
        hipLaunchKernelGGL(attn_fwd64_kernel<true>, dim3((unsigned)(nsel * Hq)), dim3(256), SMEM, s, q, k, vt, ldv, o, (int)N,
                           Hq, Hkv, sc_log2e, nqt, hpx, redo);
    else
        hipLaunchKernelGGL(attn_fwd64_kernel<false>, dim3((unsigned)(nsel * Hq)), dim3(256), SMEM, s, q, k, vt, ldv, o, (int)N,
                           Hq, Hkv, sc_log2e, nqt, hpx, redo);
    // the (query tile, head) pairs given up above, by the running-maximum kernel with the same 256-row tiles
    // (8 wavefronts x 32 rows); item b = query tile * Hq + head
    hipLaunchKernelGGL((attn_fwd_kernel<128, 1, 8, false>), dim3((unsigned)std::min(nqt * Hq, 256)), dim3(512), SMEM_REDO, s, q, k, vt, ldv,
                       o, (int)N, Hq, Hkv, sc_log2e, nqt, 0, 0, 1, nullptr, nullptr, nullptr, nullptr, 0, 0, redo);
}

template <int HD, int QT, int NW>
void launch_t(const bf16_t* q, const bf16_t* k, const bf16_t* vt, int64_t ldv, bf16_t* o, int64_t N, int Hq,
              int Hkv, int64_t q_row0, bool q_prescaled, hipStream_t s) {
    constexpr int BMQ = NW * QT * 32;
    constexpr int SMEM = 2 * 2 * BNK * HD * 2;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)attn_fwd_kernel<HD, QT, NW, false>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
        attr_set = true;
    }
    const int nqt = (int)((N + BMQ - 1) / BMQ);
    const int hpx = (Hq % 8 == 0) ? Hq / 8 : 0;
    const float sc_log2e = q_prescaled ? 1.0f : attention_q_scale(HD);
    // workgroups enumerate query tiles from the last one down: fewer of them = only the last tiles
    const int nsel = nqt - (int)((q_row0 > 0 && q_row0 < N) ? q_row0 / BMQ : 0);
    hipLaunchKernelGGL((attn_fwd_kernel<HD, QT, NW, false>), dim3((unsigned)(nsel * Hq)), dim3(NW * 64), SMEM, s, q, k, vt,
                       ldv, o, (int)N, Hq, Hkv, sc_log2e, nqt, hpx, 0, 1, nullptr, nullptr, nullptr, nullptr, 0, 0, nullptr);
}

template <int HD>
int launch_split_t(const bf16_t* q, const bf16_t* k, const bf16_t* vt, int64_t ldv, bf16_t* o, int64_t N, int Hq,
                   int Hkv, int64_t q_row0, float* scratch, size_t scratch_bytes, bool launch, const bf16_t* k2,
                   const bf16_t* vt2, int64_t ldv2, int64_t n2, bool q_prescaled, hipStream_t s) {
    constexpr int NW = 8, BMQ = NW * 32;
    constexpr int SMEM = 2 * 2 * BNK * HD * 2;
    const int64_t nq = N - q_row0;
    if (nq <= 0 || nq > 4 * BMQ) return 0;
    const int nqt = (int)((nq + BMQ - 1) / BMQ);
    const int n_kv_first = (int)((std::min<int64_t>(N, q_row0 + BMQ) - 1) / BNK + 1);     // key tiles of the first query tile
    // at most 8 splits (measured at 32 heads of 128: 150 rows behind 14 000 keys take 116 / 73 / 84 / 104 us per
    // layer with 4 / 8 / 16 / 32 splits, 600 rows 213 / 195 with 4 / 8), at least two key tiles per split
    int n_split = 1;
    while (n_split < 8 && (int64_t)nqt * Hq * n_split < 1024 && n_kv_first >= 4 * n_split) n_split *= 2;
    const size_t o_bytes = (size_t)n_split * nq * Hq * HD * sizeof(float), ml_bytes = (size_t)n_split * nq * Hq * 2 * sizeof(float);
    if (n_split < 2 || o_bytes + ml_bytes > scratch_bytes) return 0;
    if (!launch) return n_split;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)attn_fwd_kernel<HD, 1, NW, true>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
        attr_set = true;
    }
    float* opart = scratch;
    float* mlpart = scratch + o_bytes / sizeof(float);
    const float sc_log2e = q_prescaled ? 1.0f : attention_q_scale(HD);
    hipLaunchKernelGGL((attn_fwd_kernel<HD, 1, NW, true>), dim3((unsigned)(nqt * Hq * n_split)), dim3(NW * 64), SMEM, s, q,
                       k, vt, ldv, o, (int)N, Hq, Hkv, sc_log2e, nqt, 0, (int)q_row0, n_split, opart, mlpart,
                       k2 ? k2 : k, vt2 ? vt2 : vt, vt2 ? ldv2 : ldv, (k2 && vt2) ? (int)(n2 / BNK) : 0, nullptr);
    const int64_t n = nq * Hq * (HD / 4);
    hipLaunchKernelGGL(attn_combine_kernel<HD>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, opart, mlpart, n_split,
                       (int)nq, Hq, sc_log2e, o, (int)q_row0);
    return n_split;
}

}  // namespace

bool attention_mfma_supported(int Hq, int Hkv, int hd) {
    return (hd == 128 || hd == 64) && Hkv > 0 && Hq % Hkv == 0;
}

int launch_attention_mfma_split(const bf16_t* q, const bf16_t* k, const bf16_t* vt, int64_t ldv, bf16_t* o, int64_t N,
                                int Hq, int Hkv, int hd, int64_t q_row0, float* scratch, size_t scratch_bytes,
                                bool launch, const bf16_t* k2, const bf16_t* vt2, int64_t ldv2, int64_t n2,
                                bool q_prescaled, hipStream_t s) {
    if (hd == 128)
        return launch_split_t<128>(q, k, vt, ldv, o, N, Hq, Hkv, q_row0, scratch, scratch_bytes, launch, k2, vt2, ldv2, n2,
                                   q_prescaled, s);
    if (hd == 64)
        return launch_split_t<64>(q, k, vt, ldv, o, N, Hq, Hkv, q_row0, scratch, scratch_bytes, launch, k2, vt2, ldv2, n2,
                                  q_prescaled, s);
    return 0;
}

size_t attention_mfma_redo_bytes(int64_t N, int Hq) { return (size_t)((N + 255) / 256) * (size_t)Hq * sizeof(int); }

void launch_attention_mfma(const bf16_t* q, const bf16_t* k, const bf16_t* vt, int64_t ldv, bf16_t* o, int64_t N,
                           int Hq, int Hkv, int hd, int64_t q_row0, int* redo, bool q_prescaled, hipStream_t s) {
    if (N <= 0) return;
    if (hd == 128) launch_fwd64(q, k, vt, ldv, o, N, Hq, Hkv, q_row0, redo, q_prescaled, s);
    else if (hd == 64) launch_t<64, 1, 8>(q, k, vt, ldv, o, N, Hq, Hkv, q_row0, q_prescaled, s);
}

}  // namespace po
