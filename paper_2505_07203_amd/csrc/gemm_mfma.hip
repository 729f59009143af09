// bf16 MFMA GEMM for the position-wise linear layers (gfx950 / CDNA4).
//
//   C[M, N] = A[M, K] * W[N, K]^T        A: activations (token-major), W: weights in the
//                                        checkpoint layout [out, in]; both K-contiguous.
//
// Design (what bounds it: the matrix pipe, and the board's power limit, which sets the clock: every byte
// moved costs clock):
//  * Block tile 256 x 256, 256 threads = 4 wavefronts (one per SIMD) arranged 2 x 2; each
//    wavefront owns a 128 x 128 patch = 4 x 4 MFMA 32x32x16 tiles (256 fp32 accumulators per
//    lane).  The large per-wavefront patch is what keeps LDS traffic down: 8 fragment reads
//    feed 16 MFMAs per k-step (0.5 KiB of LDS reads per MFMA).
//  * K is consumed in slices of 64, so that a row of an operand slice is one whole 128-byte cache
//    line: eight lanes of a load fetch one line.  (With 64-byte rows every line was requested twice,
//    in two successive slices, and the L2 serves half lines at the cost of whole ones: 9-12 % slower.)
//    Operand slices go straight from global memory into LDS (buffer_load ... lds, 16 bytes per lane,
//    no staging registers).  One operand's slice is a 32 KiB unit; LDS (160 KiB) is a ring of five
//    units filled in the order A0 W0 A1 W1 ...: two units are being multiplied while up to three are
//    in flight, which covers HBM latency; one workgroup barrier per slice (64 MFMAs per wavefront)
//    hands units over.
//  * LDS layout: 128-byte rows (64 bf16), the eight 16-byte segments of a row XOR-swizzled with
//    (row >> 1) & 7, so that the MFMA fragment reads (16 lanes = 16 consecutive rows, same logical
//    segment; two rows share the 256 bytes the banks span) touch 16 distinct 16-byte bank groups.
//    The DMA writes a wavefront's 64 x 16 bytes contiguously, so the swizzle is applied on the global
//    side: lane l of a load fetches logical segment (l & 7) ^ swizzle(row).
//  * Workgroups are dispatched round-robin over the 8 XCDs (each with a private L2), so the
//    block id is first split into (XCD, local index) and every XCD walks a contiguous range
//    of output tiles in groups of 4 M-tiles x consecutive N-tiles: the 32 tiles resident on
//    one XCD share 4 activation panels and 8 weight panels through that XCD's L2.
//  * The MFMA is issued as (W fragment) x (A fragment)^T: in an accumulator tile a lane
//    holds ONE token row and four consecutive output features per register quad, so the
//    epilogue arithmetic (bias, residual add in fp32, SiLU-multiply of gate/up pairs, rotary embedding
//    of Q/K pairs) works on whole lanes; the position-wise results then pass through LDS so that
//    they leave as whole cache lines (see the epilogue).
//
// A row's K reduction order is fixed by the kernel and independent of how M is tiled or
// chunked, which is what makes the chunk-by-chunk evaluation of Section 4.2 bit-exact.
#include "gemm_common.h"

#include <stdlib.h>
#include <string.h>

namespace po {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;

namespace {

using namespace gemm;

constexpr int BK = 64;
constexpr int UNIT_BYTES = BM * BK * 2;            // one operand's slice: 256 rows x 128 bytes = 32 KiB
constexpr int NUNIT = 5;                           // ring of five units: the whole 160 KiB of LDS
constexpr int SMEM_BYTES = NUNIT * UNIT_BYTES;

// Stage hand-over: wait until this wavefront's global->LDS loads of the NEXT slice have landed (all
// but the 8 youngest, the activation unit after it, may stay in flight) and its own LDS reads have
// returned, then meet the other wavefronts.  A plain __syncthreads() would also wait for every load
// in flight and so cancel the prefetch distance; the "memory" clobber keeps the compiler from moving
// LDS accesses across the barrier.
#define PO_HANDOVER() asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory")

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
    // (split-K launches: workgroup row blockIdx.y works on columns [k0, k0 + K) of both operands; the
    // resources start k0 elements later and end with the matrix all the same)
    const int64_t k0 = (EPI == EPI_PARTIAL) ? (int64_t)blockIdx.y * p.K : 0;
    const uint64_t a_bytes = (uint64_t)(p.M - m0) * (uint64_t)p.lda * 2 - (uint64_t)k0 * 2,
                   w_bytes = (uint64_t)(p.N - n0) * (uint64_t)p.ldw * 2 - (uint64_t)k0 * 2;
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.A + (int64_t)m0 * p.lda + k0), 0, (int)(uint32_t)(a_bytes > 0xffffffffull ? 0xffffffffull : a_bytes), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.W + (int64_t)n0 * p.ldw + k0), 0, (int)(uint32_t)(w_bytes > 0xffffffffull ? 0xffffffffull : w_bytes), 0x00020000);
    uint32_t voa[8], vow[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = wave * 64 + i * 8 + (lane >> 3);
        const int lseg = (lane & 7) ^ ((row >> 1) & 7);
        voa[i] = (uint32_t)row * (uint32_t)(p.lda * 2) + lseg * 16;
        vow[i] = (uint32_t)row * (uint32_t)(p.ldw * 2) + lseg * 16;
    }
    const int KT = p.K / BK;
    // load i_ (0..7) of this wavefront's share of unit u_ (even: activations of slice u_/2, odd: weights)
    // into ring position pos_
#define PO_DMA(u_, pos_, i_)                                                                                  \
    {                                                                                                         \
        const int t_ = min((u_) >> 1, KT - 1);                                                                \
        unsigned char* sa_ = smem + (pos_) * UNIT_BYTES + wave * 8192 + (i_) * 1024;                          \
        __builtin_amdgcn_raw_ptr_buffer_load_lds((u_) & 1 ? rw : ra, (__attribute__((address_space(3))) void*)sa_, 16, \
                                                 (u_) & 1 ? vow[(i_)] : voa[(i_)], t_ * (BK * 2), 0, 0);      \
    }

    f32x16 acc[4][4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    // fragment read offsets: row l31 of a 32-row tile, logical segment kk*2 + lhi of its 128 bytes; one lane
    // register per k-step, operand and 64 KiB of LDS, the rest of an address is an immediate below 64 KiB
    int a_off[3][4], w_off[3][4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int fo = l31 * 128 + (((kk * 2 + lhi) ^ ((l31 >> 1) & 7)) << 4);
#pragma unroll
        for (int hb = 0; hb < 3; ++hb) {
            a_off[hb][kk] = hb * 65536 + wm * 16384 + fo;
            w_off[hb][kk] = hb * 65536 + wn * 16384 + fo;
        }
    }

    // Software pipeline inside the wavefront.  There is only one wavefront per SIMD, so every
    // cycle it spends issuing something other than an MFMA while the matrix pipe is empty is
    // lost, and the four wavefronts run in lockstep, so whatever they issue together queues
    // up in the CU's single address unit.  Memory instructions are therefore issued ONE AT A
    // TIME between MFMAs (a 32x32x16 MFMA keeps the pipe busy for 32 cycles).  A slice is four blocks
    // of 16 MFMA, one per k-step; block kk also reads the 8 fragments of the next k-step and issues loads:
    //   block 0..2 of slice s: the 8 loads of activation unit s+2, 3 + 3 + 2
    //   hand-over barrier:     slice s+1 has landed; nobody reads slice s's units any more
    //   block 3 of slice s:    fragments of (s+1, k-step 0); the 8 loads of weight unit s+2, into the
    //                          position slice s's activations occupied (unit u lives at u mod 5)
    // At the hand-over the loads issued after those of slice s+1 are the 8 of activation unit s+2.
    bf16x8 af0[4], wf0[4], af1[4], wf1[4];
#define PO_FRAG1(AF, WF, pa_, pw_, kk_, j_)                                                          \
    {                                                                                               \
        if ((j_) < 4) AF[(j_) & 3] = *(const bf16x8*)(smem + a_off[(pa_) >> 1][kk_] + ((pa_) & 1) * UNIT_BYTES + ((j_) & 3) * 4096); \
        else          WF[(j_) & 3] = *(const bf16x8*)(smem + w_off[(pw_) >> 1][kk_] + ((pw_) & 1) * UNIT_BYTES + ((j_) & 3) * 4096); \
    }
#define PO_MFMA1(AF, WF, t_)                                                                        \
    acc[(t_) >> 2][(t_) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WF[(t_) & 3], AF[(t_) >> 2], acc[(t_) >> 2][(t_) & 3], 0, 0, 0);
    // slot t of a block: fragment read number, or -1 (reads go in the order of first use:
    // MFMA t needs AF[t >> 2] and WF[t & 3])
#define PO_READ_SLOT(t_) ((t_) == 0 ? 0 : (t_) == 1 ? 4 : (t_) == 3 ? 5 : (t_) == 4 ? 6 : (t_) == 5 ? 7 : \
                          (t_) == 7 ? 1 : (t_) == 8 ? 2 : (t_) == 9 ? 3 : -1)
    // load slots of blocks 0..2 (3, 3, 2 loads) and of block 3 (all eight free slots)
#define PO_LOAD_SLOT_A(t_) ((t_) == 2 ? 0 : (t_) == 6 ? 1 : (t_) == 10 ? 2 : -1)
#define PO_LOAD_SLOT_W(t_) ((t_) == 2 ? 0 : (t_) == 6 ? 1 : (t_) >= 10 ? (t_) - 8 : -1)
    // one block: MFMAs on (AFc, WFc); reads k-step kkn_ of the slice at positions (pa_, pw_) into (AFn, WFn);
    // loads of unit u_ into position up_: numbers base_ + slot, nl_ of them (block 3: nl_ = 8, W slots)
#define PO_BLOCK(AFc, WFc, AFn, WFn, pa_, pw_, kkn_, u_, up_, base_, nl_)                             \
    _Pragma("unroll") for (int t = 0; t < 16; ++t) {                                                \
        PO_MFMA1(AFc, WFc, t);                                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        if (PO_READ_SLOT(t) >= 0) {                                                                 \
            PO_FRAG1(AFn, WFn, pa_, pw_, kkn_, PO_READ_SLOT(t));                                    \
            __builtin_amdgcn_sched_barrier(0);                                                      \
        } else if (((nl_) == 8 ? PO_LOAD_SLOT_W(t) : PO_LOAD_SLOT_A(t)) >= 0 &&                     \
                   ((nl_) == 8 ? PO_LOAD_SLOT_W(t) : PO_LOAD_SLOT_A(t)) < (nl_)) {                  \
            PO_DMA(u_, up_, (base_) + ((nl_) == 8 ? PO_LOAD_SLOT_W(t) : PO_LOAD_SLOT_A(t)));        \
            __builtin_amdgcn_sched_barrier(0);                                                      \
        }                                                                                           \
    }
    // slice s_ whose number is j_ modulo 5 (a literal): its units sit at positions 2j mod 5 and 2j+1 mod 5
#define PO_SLICE(s_, j_)                                                                            \
    {                                                                                               \
        PO_BLOCK(af0, wf0, af1, wf1, (2 * (j_)) % 5, (2 * (j_) + 1) % 5, 1, 2 * (s_) + 4, (2 * (j_) + 4) % 5, 0, 3); \
        PO_BLOCK(af1, wf1, af0, wf0, (2 * (j_)) % 5, (2 * (j_) + 1) % 5, 2, 2 * (s_) + 4, (2 * (j_) + 4) % 5, 3, 3); \
        PO_BLOCK(af0, wf0, af1, wf1, (2 * (j_)) % 5, (2 * (j_) + 1) % 5, 3, 2 * (s_) + 4, (2 * (j_) + 4) % 5, 6, 2); \
        PO_HANDOVER();                                                                              \
        PO_BLOCK(af1, wf1, af0, wf0, (2 * (j_) + 2) % 5, (2 * (j_) + 3) % 5, 0, 2 * (s_) + 5, (2 * (j_)) % 5, 0, 8); \
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
#undef PO_LOAD_SLOT_A
#undef PO_LOAD_SLOT_W
#undef PO_READ_SLOT
#undef PO_DMA
#undef PO_FRAG1
#undef PO_MFMA1
    // the clamped tail loads have landed and every wavefront has finished reading the ring
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    if (EPI == EPI_PARTIAL) {
        GemmParams q = p;
        q.dst = (bf16_t*)((float*)p.dst + (int64_t)blockIdx.y * p.ldr);     // this split's plane
        tile_epilogue<EPI>(q, acc, smem, m0, n0, wave, lane);
    } else {
        tile_epilogue<EPI>(p, acc, smem, m0, n0, wave, lane);
    }
}

// ---------------------------------------------------------------------------------------------------------
// The same GEMM on v_mfma_f32_16x16x32_bf16 with eight wavefronts (two per SIMD).
//
// Why: the board runs these GEMMs at its power limit, so what counts is energy per flop, and the matrix
// instruction with the smaller accumulator tile does 15-20 % more work per joule (bare loops on random operands:
// 2.12-2.16 PFLOP/s against 1.78-1.88 for 32x32x16).  One wavefront per SIMD cannot issue it at full rate, two can;
// with two, each has half the registers, so a wavefront owns a 128-row x 64-column patch (8 x 4 tiles, 128 fp32
// accumulators per lane) and reads 12 fragments per 32 MFMAs.  Block tile, K slices of 64, the ring of five
// 32 KiB units filled by global->LDS loads, the swizzle, the XCD-aware tile order and the reduction order over K
// (one fp32 accumulator per output runs over K in steps of 32) do not depend on how M is tiled, as before.
// Schedule of a slice (two k-steps x eight 16-row blocks = 16 groups of 4 MFMAs): the four W fragments of a k-step
// stay in registers, the A fragment of the next group is read while this group multiplies, and every group issues
// at most one more memory instruction (a W fragment of the next k-step, or one of the 4 + 4 global->LDS loads of
// W(s+1) and A(s+2)); the second wavefront of the SIMD fills the issue gaps, so nothing finer is needed.
constexpr int NTHREADS16 = 512;

template <int EPI>
__global__ void __launch_bounds__(NTHREADS16) gemm_bf16_mfma16_kernel(const GemmParams p) {
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
    const int l15 = lane & 15, l4 = lane >> 4;
    const int wm = wave >> 2, wn = wave & 3;

    // ---- global -> LDS map: a unit is 32 one-KiB loads, wavefront w issues loads 4w .. 4w+3; load q fills rows
    // 8q .. 8q+7 (lane l -> row 8q + l/8, physical segment l & 7 <- logical segment (l & 7) ^ ((row >> 1) & 7))
    const int64_t k0 = (EPI == EPI_PARTIAL) ? (int64_t)blockIdx.y * p.K : 0;
    const uint64_t a_bytes = (uint64_t)(p.M - m0) * (uint64_t)p.lda * 2 - (uint64_t)k0 * 2,
                   w_bytes = (uint64_t)(p.N - n0) * (uint64_t)p.ldw * 2 - (uint64_t)k0 * 2;
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.A + (int64_t)m0 * p.lda + k0), 0, (int)(uint32_t)(a_bytes > 0xffffffffull ? 0xffffffffull : a_bytes), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.W + (int64_t)n0 * p.ldw + k0), 0, (int)(uint32_t)(w_bytes > 0xffffffffull ? 0xffffffffull : w_bytes), 0x00020000);
    uint32_t voa[4], vow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (wave * 4 + i) * 8 + (lane >> 3);
        const int lseg = (lane & 7) ^ ((row >> 1) & 7);
        voa[i] = (uint32_t)row * (uint32_t)(p.lda * 2) + lseg * 16;
        vow[i] = (uint32_t)row * (uint32_t)(p.ldw * 2) + lseg * 16;
    }
    const int KT = p.K / BK;
#define PO_DMA16(is_w_, slice_, pos_, i_)                                                                              \
    {                                                                                                                  \
        unsigned char* d_ = smem + (pos_) * UNIT_BYTES + (wave * 4 + (i_)) * 1024;                                     \
        __builtin_amdgcn_raw_ptr_buffer_load_lds((is_w_) ? rw : ra, (__attribute__((address_space(3))) void*)d_, 16,   \
                                                 (is_w_) ? vow[(i_)] : voa[(i_)], min((slice_), KT - 1) * (BK * 2), 0, 0); \
    }
    // fragment offsets: row l15 of a 16-row block, logical segment 4 ks + l4 of its 128 bytes
    int f_off[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) f_off[ks] = l15 * 128 + (((ks * 4 + l4) ^ ((l15 >> 1) & 7)) << 4);
    const int a_base = wm * 128 * 128, w_base = wn * 64 * 128;     // byte offset of the wavefront's rows inside a unit

    f32x4 acc[8][4];
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[u][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // prologue: A0 W0 A1 in flight; W1 follows at the top of slice 0
#pragma unroll
    for (int i = 0; i < 4; ++i) PO_DMA16(0, 0, 0, i)
#pragma unroll
    for (int i = 0; i < 4; ++i) PO_DMA16(1, 0, 1, i)
#pragma unroll
    for (int i = 0; i < 4; ++i) PO_DMA16(0, 1, 2, i)
    asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");      // slice 0 has landed
    int pa = 0;                                                        // ring position of slice s's A unit; W at pa + 1
    for (int s = 0; s < KT; ++s) {
        const int pw = pa + 1 >= NUNIT ? pa + 1 - NUNIT : pa + 1;
        const int pw1 = pa + 3 >= NUNIT ? pa + 3 - NUNIT : pa + 3;    // W(s+1): the position A(s-1) left
        const int pa2 = pa + 4 >= NUNIT ? pa + 4 - NUNIT : pa + 4;    // A(s+2): the position W(s-1) left
        const unsigned char* ua = smem + pa * UNIT_BYTES + a_base;
        const unsigned char* uw = smem + pw * UNIT_BYTES + w_base;
        bf16x8 wf[2][4], afc, afn;
#pragma unroll
        for (int t = 0; t < 4; ++t) wf[0][t] = *(const bf16x8*)(uw + t * 2048 + f_off[0]);
        afc = *(const bf16x8*)(ua + f_off[0]);
#pragma unroll
        for (int gi = 0; gi < 16; ++gi) {                              // group gi: k-step gi / 8, row block gi % 8
            const int ks = gi >> 3, u = gi & 7;
            if (gi < 15) afn = *(const bf16x8*)(ua + ((gi + 1) & 7) * 2048 + f_off[(gi + 1) >> 3]);
            if (gi >= 4 && gi < 8) wf[1][gi - 4] = *(const bf16x8*)(uw + (gi - 4) * 2048 + f_off[1]);
            if (gi < 4) PO_DMA16(1, s + 1, pw1, gi)
            if (gi >= 8 && gi < 12) PO_DMA16(0, s + 2, pa2, gi - 8)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < 4; ++t)
                acc[u][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[ks][t], afc, acc[u][t], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            afc = afn;
        }
        // hand-over: slice s+1 has landed (everything but the 4 loads of A(s+2)), nobody reads slice s any more
        asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        pa = pa + 2 >= NUNIT ? pa + 2 - NUNIT : pa + 2;
    }
#undef PO_DMA16
    // the clamped tail loads have landed and every wavefront has finished reading the ring
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    if (EPI == EPI_PARTIAL) {
        GemmParams q = p;
        q.dst = (bf16_t*)((float*)p.dst + (int64_t)blockIdx.y * p.ldr);     // this split's plane
        tile_epilogue16<EPI>(q, acc, smem, m0, n0, wave, lane);
    } else {
        tile_epilogue16<EPI>(p, acc, smem, m0, n0, wave, lane);
    }
}

// C[row][col .. col+7] = bf16(sum over splits of part[s][row][col ..] + R[row][col ..]); one thread per 8 features.
__global__ void __launch_bounds__(256) splitk_reduce_residual_kernel(const float* __restrict__ part, int64_t plane,
                                                                     int splits, const bf16_t* R, int64_t ldr,
                                                                     bf16_t* C, int64_t ldc, int M, int N) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int n8 = N >> 3;
    if (i >= (int64_t)M * n8) return;
    const int row = (int)(i / n8), col = (int)(i - (int64_t)row * n8) * 8;
    const float* pp = part + (int64_t)row * N + col;
    float4 a = *(const float4*)pp, b = *(const float4*)(pp + 4);
    for (int sidx = 1; sidx < splits; ++sidx) {
        const float4 x = *(const float4*)(pp + sidx * plane), y = *(const float4*)(pp + sidx * plane + 4);
        a.x += x.x; a.y += x.y; a.z += x.z; a.w += x.w;
        b.x += y.x; b.y += y.y; b.z += y.z; b.w += y.w;
    }
    const uint4 r = *(const uint4*)(R + (int64_t)row * ldr + col);
    uint4 o;
    o.x = (uint32_t)f2bf(a.x + __uint_as_float(r.x << 16)) | ((uint32_t)f2bf(a.y + __uint_as_float(r.x & 0xffff0000u)) << 16);
    o.y = (uint32_t)f2bf(a.z + __uint_as_float(r.y << 16)) | ((uint32_t)f2bf(a.w + __uint_as_float(r.y & 0xffff0000u)) << 16);
    o.z = (uint32_t)f2bf(b.x + __uint_as_float(r.z << 16)) | ((uint32_t)f2bf(b.y + __uint_as_float(r.z & 0xffff0000u)) << 16);
    o.w = (uint32_t)f2bf(b.z + __uint_as_float(r.w << 16)) | ((uint32_t)f2bf(b.w + __uint_as_float(r.w & 0xffff0000u)) << 16);
    *(uint4*)(C + (int64_t)row * ldc + col) = o;
}

// QKV after a split-K GEMM: one workgroup = one 64-column patch x 8 token rows.  Sums the splits' partials,
// then does what the fused QKV epilogue does with an accumulator patch: + bias, rotary embedding of the
// pair (column j, column j + 32) of a Q / K patch, V stored transposed.  Thread mapping: Q / K patches
// column-fastest (row stores are contiguous), V patches row-fastest (V^T columns are contiguous).
__global__ void __launch_bounds__(256) splitk_reduce_qkv_kernel(const float* __restrict__ part, int64_t plane, int splits,
                                                                const GemmParams p) {
    const int cb = blockIdx.x * 64;
    const bool is_v = cb >= p.qd + p.kvd;
    const int j = is_v ? (int)(threadIdx.x >> 3) : (int)(threadIdx.x & 31);
    const int row = blockIdx.y * 8 + (is_v ? (int)(threadIdx.x & 7) : (int)(threadIdx.x >> 5));
    if (row >= p.M) return;
    const float* pp = part + (int64_t)row * p.N + cb + j;
    float a = pp[0], b = pp[32];
    for (int sidx = 1; sidx < splits; ++sidx) {
        a += pp[sidx * plane];
        b += pp[sidx * plane + 32];
    }
    if (p.bias) {
        a += bf2f(p.bias[cb + j]);
        b += bf2f(p.bias[cb + 32 + j]);
    }
    if (!is_v) {
        const bool is_q = cb < p.qd;
        const int c = is_q ? cb : cb - p.qd;
        const int head = c / p.hd;
        const int half = p.hd >> 1;
        const int i0 = (((c - head * p.hd) >> 6) << 5) + j;                  // rotary index
        const int64_t pos = p.row_pos ? (int64_t)p.row_pos[p.pos0 + row] : p.pos0 + row;
        const float cs = p.rope_cos[pos * half + i0], sn = p.rope_sin[pos * half + i0];
        bf16_t* drow = (is_q ? p.dst + (int64_t)row * p.qd : p.dst_k + (int64_t)row * p.kvd) + head * p.hd + i0;
        drow[0] = f2bf(a * cs - b * sn);
        drow[half] = f2bf(b * cs + a * sn);
    } else {
        const int f = cb - p.qd - p.kvd + j;
        bf16_t* dcol = p.dst_vt + p.pos0 + row;
        dcol[(int64_t)f * p.ldv] = f2bf(a);
        dcol[(int64_t)(f + 32) * p.ldv] = f2bf(b);
    }
}

// Gate/up after a split-K GEMM: H[row][cb/2 + j] = silu(sum gate column cb + j) * (sum up column cb + 32 + j),
// the interleaving of the fused SiLU-multiply epilogue; one thread per output feature.
__global__ void __launch_bounds__(256) splitk_reduce_silu_kernel(const float* __restrict__ part, int64_t plane, int splits,
                                                                 bf16_t* H, int64_t ldh, int M, int N) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int nf = N >> 1;
    if (i >= (int64_t)M * nf) return;
    const int row = (int)(i / nf), f = (int)(i - (int64_t)row * nf);
    const float* pp = part + (int64_t)row * N + ((f >> 5) << 6) + (f & 31);
    float g = pp[0], u = pp[32];
    for (int sidx = 1; sidx < splits; ++sidx) {
        g += pp[sidx * plane];
        u += pp[sidx * plane + 32];
    }
    H[(int64_t)row * ldh + f] = f2bf(silu_f(g) * u);
}

int gemm_variant() {
    static int v = -1;
    if (v < 0) {
        const char* e = getenv("PO_GEMM_VARIANT");
        v = e ? atoi(e) : 16;
    }
    return v;
}

template <int EPI>
void launch_t(const GemmParams& p, hipStream_t s, int splits = 1) {
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)gemm_bf16_mfma_kernel<EPI>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
        (void)hipFuncSetAttribute((const void*)gemm_bf16_mfma16_kernel<EPI>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
        attr_set = true;
    }
    const int total = p.mt * p.nt;
    const int per_xcd = (total + 7) / 8;
    if (gemm_variant() == 32)
        hipLaunchKernelGGL(gemm_bf16_mfma_kernel<EPI>, dim3((unsigned)(per_xcd * 8), (unsigned)splits), dim3(NTHREADS), SMEM_BYTES, s, p);
    else
        hipLaunchKernelGGL(gemm_bf16_mfma16_kernel<EPI>, dim3((unsigned)(per_xcd * 8), (unsigned)splits), dim3(NTHREADS16), SMEM_BYTES, s, p);
}

GemmParams base_params(const bf16_t* A, int64_t lda, const bf16_t* W, int64_t ldw, int64_t M, int N, int K) {
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A = A; p.W = W; p.lda = lda; p.ldw = ldw;
    p.M = (int)M; p.N = N; p.K = K;
    p.mt = (int)((M + BM - 1) / BM);
    p.nt = (N + BN - 1) / BN;
    return p;
}

}  // namespace

// K must be a multiple of 64 (whole slices), N of 64 (the epilogues work on 64-column patches).
bool gemm_mfma_supported(int N, int K) { return K > 0 && K % 64 == 0 && N > 0 && N % 64 == 0; }

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

namespace gemm {

int pick_splits(int64_t M, int N, int kt, size_t part_bytes) {
    const int64_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    int splits = 1;
    // (8 against 16 splits measured equal on the 8B shape's O / down projections at 150 rows, 4 a quarter slower)
    while (splits < 8 && tiles * splits * 2 <= 256 && kt % (splits * 2) == 0 && kt / (splits * 2) >= 2) splits *= 2;
    while (splits > 1 && (size_t)splits * (size_t)M * (size_t)N * sizeof(float) > part_bytes) splits /= 2;
    return splits;
}

void launch_splitk_reduce_residual(const float* part, int splits, const bf16_t* R, int64_t ldr, bf16_t* C, int64_t ldc,
                                   int64_t M, int N, hipStream_t s) {
    const int64_t n = M * (int64_t)(N >> 3);
    hipLaunchKernelGGL(splitk_reduce_residual_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, part,
                       M * (int64_t)N, splits, R, ldr, C, ldc, (int)M, N);
}

void launch_splitk_reduce_silu(const float* part, int splits, bf16_t* H, int64_t ldh, int64_t M, int N, hipStream_t s) {
    const int64_t n = M * (int64_t)(N >> 1);
    hipLaunchKernelGGL(splitk_reduce_silu_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, part, M * (int64_t)N,
                       splits, H, ldh, (int)M, N);
}

void launch_splitk_reduce_qkv(const float* part, int splits, const GemmParams& r, hipStream_t s) {
    hipLaunchKernelGGL(splitk_reduce_qkv_kernel, dim3((unsigned)(r.N / 64), (unsigned)((r.M + 7) / 8)), dim3(256), 0, s, part,
                       (int64_t)r.M * r.N, splits, r);
}

}  // namespace gemm

int launch_gemm_qkv_rope_splitk(const bf16_t* A, int64_t lda, const bf16_t* Wqkv, int64_t ldw, const bf16_t* bias,
                                bf16_t* Q, bf16_t* Kd, bf16_t* Vt, int64_t ldv, const float* rope_cos,
                                const float* rope_sin, int64_t pos0, const int32_t* row_pos, int64_t M, int qd, int kvd,
                                int hd, int K, float* part, size_t part_bytes, bool launch, hipStream_t s) {
    const int N = qd + 2 * kvd;
    if (M <= 0 || !gemm_mfma_supported(N, K) || (qd & 63) || (kvd & 63) || (hd & 63)) return 0;
    const int splits = pick_splits(M, N, K / BK, part_bytes);
    if (splits < 2) return 0;
    if (!launch) return splits;
    GemmParams p = base_params(A, lda, Wqkv, ldw, M, N, K / splits);
    p.dst = (bf16_t*)part;
    p.ld = N;
    p.ldr = M * (int64_t)N;
    launch_t<EPI_PARTIAL>(p, s, splits);
    GemmParams r = base_params(A, lda, Wqkv, ldw, M, N, K);
    r.bias = bias; r.dst = Q; r.dst_k = Kd; r.dst_vt = Vt; r.ldv = ldv;
    r.rope_cos = rope_cos; r.rope_sin = rope_sin; r.pos0 = pos0; r.row_pos = row_pos;
    r.qd = qd; r.kvd = kvd; r.hd = hd;
    launch_splitk_reduce_qkv(part, splits, r, s);
    return splits;
}

int launch_gemm_mfma_splitk_silu(const bf16_t* A, int64_t lda, const bf16_t* W, int64_t ldw, bf16_t* H, int64_t ldh,
                                 int64_t M, int N, int K, float* part, size_t part_bytes, bool launch, hipStream_t s) {
    if (M <= 0 || !gemm_mfma_supported(N, K)) return 0;
    const int splits = pick_splits(M, N, K / BK, part_bytes);
    if (splits < 2) return 0;
    if (!launch) return splits;
    GemmParams p = base_params(A, lda, W, ldw, M, N, K / splits);
    p.dst = (bf16_t*)part;
    p.ld = N;
    p.ldr = M * (int64_t)N;
    launch_t<EPI_PARTIAL>(p, s, splits);
    launch_splitk_reduce_silu(part, splits, H, ldh, M, N, s);
    return splits;
}

int launch_gemm_mfma_splitk_residual(const bf16_t* A, int64_t lda, const bf16_t* W, int64_t ldw, bf16_t* C,
                                     int64_t ldc, const bf16_t* R, int64_t ldr, int64_t M, int N, int K,
                                     float* part, size_t part_bytes, bool launch, hipStream_t s) {
    if (M <= 0 || N <= 0 || !gemm_mfma_supported(N, K) || (N & 7) || (ldc & 7) || (ldr & 7)) return 0;
    const int splits = pick_splits(M, N, K / BK, part_bytes);
    if (splits < 2) return 0;
    if (!launch) return splits;
    GemmParams p = base_params(A, lda, W, ldw, M, N, K / splits);
    p.dst = (bf16_t*)part;
    p.ld = N;
    p.ldr = M * (int64_t)N;              // floats between two splits' planes
    launch_t<EPI_PARTIAL>(p, s, splits);
    launch_splitk_reduce_residual(part, splits, R, ldr, C, ldc, M, N, s);
    return splits;
}

void launch_gemm_qkv_rope(const bf16_t* A, int64_t lda, const bf16_t* Wqkv, int64_t ldw, const bf16_t* bias,
                          bf16_t* Q, bf16_t* Kd, bf16_t* Vt, int64_t ldv, const float* rope_cos,
                          const float* rope_sin, int64_t pos0, const int32_t* row_pos, int64_t M, int qd, int kvd,
                          int hd, int K, hipStream_t s) {
    if (M <= 0) return;
    GemmParams p = base_params(A, lda, Wqkv, ldw, M, qd + 2 * kvd, K);
    p.bias = bias; p.dst = Q; p.dst_k = Kd; p.dst_vt = Vt; p.ldv = ldv;
    p.rope_cos = rope_cos; p.rope_sin = rope_sin; p.pos0 = pos0; p.row_pos = row_pos;
    p.qd = qd; p.kvd = kvd; p.hd = hd;
    launch_t<EPI_QKV_ROPE>(p, s);
}

}  // namespace po
