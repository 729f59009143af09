// bf16 MFMA GEMM for the position-wise linear layers (gfx950 / CDNA4).
//
//   C[M, N] = A[M, K] * W[N, K]^T        A: activations (token-major), W: weights in the
//                                        checkpoint layout [out, in]; both K-contiguous.
//
// What bounds it: the board's power limit.  These GEMMs keep the matrix pipe busy 64-72 % of their cycles (counters), and
// the clock the board grants (1.6-1.9 GHz of a nominal 2.4) falls with every joule spent per flop, so the design
// minimises energy per flop, not instruction slots:
//  * v_mfma_f32_16x16x32_bf16.  A bare loop of it on random operands sustains 2.1-2.2 PFLOP/s on this board, against
//    1.9 for 32x32x16 (both power-limited, with one wavefront per SIMD as with two).  The workgroup is eight
//    wavefronts, two per SIMD, arranged 2 x 4 over a 256 x 256 block tile: each owns a 128-row x 64-column patch of
//    8 x 4 tiles (128 fp32 accumulators per lane) and reads 12 fragments per 32 MFMAs.  The second wavefront of a
//    SIMD is there for the waits, not for the issue rate: it multiplies while the first waits for a fragment or at
//    the hand-over barrier, and it halves the time of the epilogue.  (A four-wavefront form with 128 x 128 patches,
//    16 fragment reads per 64 MFMAs, was built on the same ring and gives the same bits: 2-18 % slower.)  Memory
//    instructions simply sit one behind each MFMA.
//  * K is consumed in slices of 64, so that a row of an operand slice is one whole 128-byte cache line: eight
//    lanes of a load fetch one line.  Operand slices go straight from global memory into LDS (buffer_load ... lds,
//    16 bytes per lane, no staging registers; copies of this kernel that stage them through registers, with the
//    ds_writes early or late in the slice, clock 5 % higher but keep the matrix pipe 9-11 points less busy: vector
//    memory returns and LDS writes take issue slots that MFMAs of neither wavefront of the SIMD can use).  One operand's slice is a 32 KiB unit; LDS (160 KiB) is a
//    ring of five units filled in the order A0 W0 A1 W1 ...: two are being multiplied while up to three are in
//    flight.  These loads are the largest single item of the energy bill (a timing-only copy without them runs
//    15-18 % faster, one without the LDS fragment reads 7 %); their bytes per flop are fixed by the 256 x 256 tile,
//    the largest whose accumulators fit the register file.
//  * A slice is four phases of 16 MFMAs (k-step 0 rows 0-63, k-step 0 rows 64-127, k-step 1 rows 0-63, k-step 1
//    rows 64-127).  Fragments are read a whole phase ahead of their MFMAs into the A / W register set that is idle,
//    so at the hand-over barrier, which sits BEHIND PHASE 2, every LDS read of the slice is done: phase 3 multiplies
//    from registers while it reads the first fragments of the next slice, which the barrier has just handed over,
//    and the loads that overwrite this slice's two units are issued right behind the barrier.  No wavefront starts
//    a slice by waiting for LDS (worth 3-4 % over a barrier at the slice's end).
//  * LDS layout: 128-byte rows (64 bf16), the eight 16-byte segments of a row XOR-swizzled with (row >> 1) & 7, so
//    that a fragment read (16 lanes = 16 consecutive rows, same logical segment; two rows share the 256 bytes the
//    banks span) touches 16 distinct 16-byte bank groups.  The DMA writes a wavefront's 64 x 16 bytes contiguously,
//    so the swizzle is applied on the global side: lane l of a load fetches logical segment (l & 7) ^ swizzle(row).
//  * Workgroups are dispatched round-robin over the 8 XCDs (each with a private L2), so the block id is first
//    split into (XCD, local index) and every XCD walks a contiguous range of output tiles in groups of 4 M-tiles x
//    consecutive N-tiles: the 32 tiles resident on one XCD share 4 activation panels and 8 weight panels through
//    that XCD's L2.
//  * The MFMA is issued as (W fragment) x (A fragment)^T: in an accumulator tile a lane holds ONE token row and
//    four consecutive output features, so the epilogue arithmetic (bias, residual add in fp32, SiLU-multiply of
//    gate/up pairs, rotary embedding of Q/K pairs) works on whole lanes; the position-wise results then pass through
//    LDS so that they leave as whole row segments (see tile_epilogue16).
//
// A row's K reduction order (one fp32 accumulator per output runs over K in steps of 32) is fixed by the kernel and
// independent of how M is tiled or chunked, which is what makes the chunk-by-chunk evaluation of Section 4.2
// bit-exact.
#include "gemm_common.h"

#include <string.h>

namespace po {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;

namespace {

using namespace gemm;

constexpr int BK = 64;
constexpr int UNIT_BYTES = BM * BK * 2;            // one operand's slice: 256 rows x 128 bytes = 32 KiB
constexpr int NUNIT = 5;                           // ring of five units: the whole 160 KiB of LDS
constexpr int SMEM_BYTES = NUNIT * UNIT_BYTES;
constexpr int NT_BF16 = 512;                       // eight wavefronts (the FP8 kernel keeps gemm::NTHREADS = 256)

// MU = 16-row groups per wavefront patch: 8 (256-row block tile, the form described above) or 4 (128-row block tile:
// wavefront patches of 64 x 64, a slice is two phases of 16 MFMAs with the hand-over barrier behind the first, the A
// unit is half full).  Every output element still is ONE fp32 accumulator running over K in steps of 32 in the same
// order, so the two forms give the same bits, and the launcher may pick by tile count alone: launches whose 256-row
// tiles would leave compute units idle (short requests, N of 4096-5120) take the 128-row form.
template <int EPI, int MU>
__global__ void __launch_bounds__(NT_BF16) gemm_bf16_mfma_kernel(const GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int BM_ = 32 * MU;                   // block tile rows
    constexpr int NA = MU / 2;                     // global->LDS loads per wavefront for an A unit (W: always 4)

    const int total = p.mt * p.nt;
    const int per_xcd = (total + 7) >> 3;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int li = xcd * per_xcd + local;
    if (local >= per_xcd || li >= total) return;
    constexpr int GM = MU == 8 ? GROUP_M : 2 * GROUP_M;       // M-tiles per group: 1024 rows either way
    const int group_sz = GM * p.nt;
    const int g = li / group_sz;
    const int within = li - g * group_sz;
    const int gm_this = min(GM, p.mt - g * GM);
    const int tn = within / gm_this;
    const int tm = g * GM + (within - tn * gm_this);
    const int m0 = tm * BM_, n0 = tn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l15 = lane & 15, l4 = lane >> 4;
    const int wm = wave >> 2, wn = wave & 3;

    const int64_t k0 = (EPI == EPI_PARTIAL) ? (int64_t)blockIdx.y * p.K : 0;
    const uint64_t a_bytes = (uint64_t)(p.M - m0) * (uint64_t)p.lda * 2 - (uint64_t)k0 * 2,
                   w_bytes = (uint64_t)(p.N - n0) * (uint64_t)p.ldw * 2 - (uint64_t)k0 * 2;
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.A + (int64_t)m0 * p.lda + k0), 0, (int)(uint32_t)(a_bytes > 0xffffffffull ? 0xffffffffull : a_bytes), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.W + (int64_t)n0 * p.ldw + k0), 0, (int)(uint32_t)(w_bytes > 0xffffffffull ? 0xffffffffull : w_bytes), 0x00020000);
    uint32_t voa[4] = {0, 0, 0, 0}, vow[4];      // (voa: NA entries used)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (wave * 4 + i) * 8 + (lane >> 3);
        const int lseg = (lane & 7) ^ ((row >> 1) & 7);
        vow[i] = (uint32_t)row * (uint32_t)(p.ldw * 2) + lseg * 16;
    }
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int row = (wave * NA + i) * 8 + (lane >> 3);
        const int lseg = (lane & 7) ^ ((row >> 1) & 7);
        voa[i] = (uint32_t)row * (uint32_t)(p.lda * 2) + lseg * 16;
    }
    const int KT = p.K / BK;
    // load i_ (W: 0..3, A: 0..NA-1) of this wavefront's share of the A (is_w_ = 0) or W unit of slice slice_, into ring
    // position pos_
#define PO_DMA(is_w_, slice_, pos_, i_)                                                                              \
    {                                                                                                                  \
        unsigned char* d_ = smem + (pos_) * UNIT_BYTES + (wave * ((is_w_) ? 4 : NA) + (i_)) * 1024;                    \
        __builtin_amdgcn_raw_ptr_buffer_load_lds((is_w_) ? rw : ra, (__attribute__((address_space(3))) void*)d_, 16,   \
                                                 (is_w_) ? vow[(i_)] : voa[(i_)],                    \
                                                 min((slice_), KT - 1) * (BK * 2), 0, 0);                              \
    }
    int f_off[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) f_off[ks] = l15 * 128 + (((ks * 4 + l4) ^ ((l15 >> 1) & 7)) << 4);
    const int a_base = wm * (MU * 16) * 128, w_base = wn * 64 * 128;

    f32x4 acc[MU][4];
#pragma unroll
    for (int u = 0; u < MU; ++u)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[u][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // prologue: A0 W0 A1 W1 in flight (A2 follows in slice 0); slice 0's first fragments
#pragma unroll
    for (int u4 = 0; u4 < 4; ++u4)
#pragma unroll
        for (int i = 0; i < ((u4 & 1) ? 4 : NA); ++i) PO_DMA(u4 & 1, u4 >> 1, u4, i)
    if (MU == 8) asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");      // slice 0 has landed
    else asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");
    bf16x8 A0[4], A1[4], W0[4], W1[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        W0[j] = *(const bf16x8*)(smem + UNIT_BYTES + w_base + j * 2048 + f_off[0]);
        A0[j] = *(const bf16x8*)(smem + a_base + j * 2048 + f_off[0]);
    }
    // One phase: 16 MFMAs, rows 64 uh_ .. +63 of the patch (A fragments AC, W fragments WC); behind MFMA m the
    // memory instruction number m of the phase, if it has one:
    //   RA_: read the four A fragments (rows 64 rah_ .., k-step rak_) of the unit at ua_ into AN
    //   RW_: read the four W fragments (k-step rwk_) of the unit at uw_ into WN (behind the A reads)
    //   DMA_: the four global->LDS loads of (dw_ ? W : A) unit of slice ds_ into position dp_ (behind the reads)
#define PO_PHASE(AC, WC, uh_, RA_, AN, ua_, rah_, rak_, RW_, WN, uw_, rwk_, DMA_, dw_, ds_, dp_)                    \
    _Pragma("unroll") for (int m = 0; m < 16; ++m) {                                                                  \
        const int u_ = (uh_) * 4 + (m >> 2), t_ = m & 3;                                                              \
        acc[u_][t_] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(WC[t_], AC[m >> 2], acc[u_][t_], 0, 0, 0);              \
        __builtin_amdgcn_sched_barrier(0);                                                                            \
        const int nra_ = (RA_) ? 4 : 0, nrw_ = (RW_) ? 4 : 0;                                                         \
        if (m < nra_) {                                                                                               \
            AN[m & 3] = *(const bf16x8*)((ua_) + ((rah_) * 4 + (m & 3)) * 2048 + f_off[rak_]);     \
            __builtin_amdgcn_sched_barrier(0);                                                                        \
        } else if (m < nra_ + nrw_) {                                                                                 \
            WN[(m - nra_) & 3] = *(const bf16x8*)((uw_) + ((m - nra_) & 3) * 2048 + f_off[rwk_]);  \
            __builtin_amdgcn_sched_barrier(0);                                                                        \
        } else if ((DMA_) && m < nra_ + nrw_ + ((dw_) ? 4 : NA)) {                                                    \
            PO_DMA(dw_, ds_, dp_, (m - nra_ - nrw_) & 3)                                         \
            __builtin_amdgcn_sched_barrier(0);                                                                        \
        }                                                                                                             \
    }
    int pa = 0;                                  // ring position of slice s's A unit; its W unit at pa + 1
    for (int s = 0; s < KT; ++s) {
        const int pw = pa + 1 >= NUNIT ? pa + 1 - NUNIT : pa + 1;
        const int pa1 = pa + 2 >= NUNIT ? pa + 2 - NUNIT : pa + 2;    // A(s+1)
        const int pw1 = pa + 3 >= NUNIT ? pa + 3 - NUNIT : pa + 3;    // W(s+1)
        const unsigned char* ua = smem + pa * UNIT_BYTES + a_base;
        const unsigned char* uw = smem + pw * UNIT_BYTES + w_base;
        const unsigned char* ua1 = smem + pa1 * UNIT_BYTES + a_base;
        const unsigned char* uw1 = smem + pw1 * UNIT_BYTES + w_base;
        if constexpr (MU == 8) {
            // phase 0: k-step 0, rows 0-63 | reads A(k0, rows 64-127) and W(k1)
            PO_PHASE(A0, W0, 0, 1, A1, ua, 1, 0, 1, W1, uw, 1, 0, 0, 0, 0)
            // phase 1: k-step 0, rows 64-127 | reads A(k1, rows 0-63); loads A(s+2) into the position W(s-1) left
            PO_PHASE(A1, W0, 1, 1, A0, ua, 0, 1, 0, W1, uw, 1, 1, 0, s + 2, (pa + 4 >= NUNIT ? pa + 4 - NUNIT : pa + 4))
            // phase 2: k-step 1, rows 0-63 | reads A(k1, rows 64-127)
            PO_PHASE(A0, W1, 0, 1, A1, ua, 1, 1, 0, W0, uw, 0, 0, 0, 0, 0)
            // hand-over: slice s+1 has landed (all but the 4 youngest loads), every LDS read of slice s is done
            asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            // phase 3: k-step 1, rows 64-127 | reads W(k0) and A(k0, rows 0-63) of slice s+1; loads W(s+2) into A(s)'s position
            PO_PHASE(A1, W1, 1, 1, A0, ua1, 0, 0, 1, W0, uw1, 0, 1, 1, s + 2, pa)
        } else {
            // phase 0: k-step 0 | reads A(k1) and W(k1); loads A(s+2) into the position W(s-1) left
            PO_PHASE(A0, W0, 0, 1, A1, ua, 0, 1, 1, W1, uw, 1, 1, 0, s + 2, (pa + 4 >= NUNIT ? pa + 4 - NUNIT : pa + 4))
            // hand-over: slice s+1 has landed (all but the NA youngest loads), every LDS read of slice s is done
            asm volatile("s_waitcnt vmcnt(2) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            // phase 1: k-step 1 | reads A(k0) and W(k0) of slice s+1; loads W(s+2) into A(s)'s position
            PO_PHASE(A1, W1, 0, 1, A0, ua1, 0, 0, 1, W0, uw1, 0, 1, 1, s + 2, pa)
        }
        pa = pa1;
    }
#undef PO_PHASE
#undef PO_DMA
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    if (EPI == EPI_PARTIAL) {
        GemmParams q = p;
        q.dst = (bf16_t*)((float*)p.dst + (int64_t)blockIdx.y * p.ldr);
        tile_epilogue16<EPI, MU>(q, acc, smem, m0, n0, wave, lane);
    } else {
        tile_epilogue16<EPI, MU>(p, acc, smem, m0, n0, wave, lane);
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
        const float qs = is_q ? p.q_scale : 1.0f;
        drow[0] = f2bf((a * cs - b * sn) * qs);
        drow[half] = f2bf((b * cs + a * sn) * qs);
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

// 256-row or 128-row block tiles: the cheaper by rounds of tiles over the 256 compute units, a 128-row tile counted
// as 0.66 of a 256-row one.  Measured: 0.51-0.55 in launches of one round (O- and down projections of up to 2048
// rows: 185 against 248 us at 1920 rows), 0.63-0.68 in launches of many rounds (gate/up: every tile streams a whole W
// slice for half the rows), where the 256-row form stays the better one unless it wastes most of a round.  Same bits
// either way.
constexpr double COST_128_ROW_TILE = 0.66;
double cost_256(int64_t M, int N) { return (double)((((M + 255) / 256) * ((N + BN - 1) / BN) + 255) / 256); }
double cost_128(int64_t M, int N) {
    return COST_128_ROW_TILE * (double)((((M + 127) / 128) * ((N + BN - 1) / BN) + 255) / 256);
}
bool prefer_128_row_tiles(int64_t M, int N) { return cost_128(M, N) < cost_256(M, N); }

template <int E2, int M2>
void launch_mu(GemmParams p, hipStream_t s, int splits) {
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)gemm_bf16_mfma_kernel<E2, M2>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
        attr_set = true;
    }
    p.mt = (p.M + 32 * M2 - 1) / (32 * M2);
    const int total = p.mt * p.nt;
    const int per_xcd = (total + 7) / 8;
    hipLaunchKernelGGL((gemm_bf16_mfma_kernel<E2, M2>), dim3((unsigned)(per_xcd * 8), (unsigned)splits), dim3(NT_BF16),
                       SMEM_BYTES, s, p);
}

template <int EPI>
void launch_t(const GemmParams& p, hipStream_t s, int splits = 1) {
    if (EPI != EPI_PARTIAL && prefer_128_row_tiles(p.M, p.N)) launch_mu<EPI, 4>(p, s, splits);
    else launch_mu<EPI, 8>(p, s, splits);
}

GemmParams base_params(const bf16_t* A, int64_t lda, const bf16_t* W, int64_t ldw, int64_t M, int N, int K) {
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A = A; p.W = W; p.lda = lda; p.ldw = ldw;
    p.M = (int)M; p.N = N; p.K = K;
    p.q_scale = 1.0f;
    p.mt = (int)((M + BM - 1) / BM);
    p.nt = (N + BN - 1) / BN;
    return p;
}

}  // namespace

// K must be a multiple of 64 (whole slices), N of 64 (the epilogues work on 64-column patches).
bool gemm_mfma_supported(int N, int K) { return K > 0 && K % 64 == 0 && N > 0 && N % 64 == 0; }

double gemm_mfma_launch_cost(int64_t M, int N) { return prefer_128_row_tiles(M, N) ? cost_128(M, N) : cost_256(M, N); }

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
                                int hd, int K, float q_scale, float* part, size_t part_bytes, bool launch, hipStream_t s) {
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
    r.qd = qd; r.kvd = kvd; r.hd = hd; r.q_scale = q_scale;
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
                          int hd, int K, float q_scale, hipStream_t s) {
    if (M <= 0) return;
    GemmParams p = base_params(A, lda, Wqkv, ldw, M, qd + 2 * kvd, K);
    p.q_scale = q_scale;
    p.bias = bias; p.dst = Q; p.dst_k = Kd; p.dst_vt = Vt; p.ldv = ldv;
    p.rope_cos = rope_cos; p.rope_sin = rope_sin; p.pos0 = pos0; p.row_pos = row_pos;
    p.qd = qd; p.kvd = kvd; p.hd = hd;
    launch_t<EPI_QKV_ROPE>(p, s);
}

}  // namespace po
