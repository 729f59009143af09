// Shared by the bf16 and the FP8 GEMM (gfx950): launch parameters and the epilogues.
#pragma once
#include "po_internal.h"

#include <type_traits>

namespace po {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace gemm {

constexpr int BM = 256, BN = 256;
constexpr int NTHREADS = 256;
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
    int64_t pos0;        // EPI_QKV_ROPE: buffer row (= V^T column) of GEMM row 0, and its sequence position
    const int32_t* row_pos;  // EPI_QKV_ROPE: sequence position of every buffer row when several requests are
                             // packed into one buffer (indexed by buffer row); null = position == buffer row
    int M, N, K;
    int mt, nt;          // tile counts
    int qd, kvd, hd;     // EPI_QKV_ROPE: segment widths and head size
    const float* sa;     // FP8 kernel: scale per token row [M] and per output feature [N]
    const float* sw;
    float q_scale;       // EPI_QKV_ROPE: factor on the rotated Q values before they are rounded (1, or the softmax
                         // scale in log2 units when the attention kernel expects Q scaled; K and V are never scaled)
};

// g * sigmoid(g).  The reciprocal is the hardware's (v_rcp_f32, 1 ulp) instead of an IEEE division: the division expands
// to ten dependent instructions per value, 64 values per lane in a gate/up tile's epilogue, which no MFMA overlaps.
__device__ __forceinline__ float silu_f(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) {
    uint2 w;
    w.x = (uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16);
    w.y = (uint32_t)f2bf(c) | ((uint32_t)f2bf(d) << 16);
    return w;
}

// Epilogue of one 64-column patch of one token row.  c0 / c1 are the accumulator tiles of
// the patch's two 32-column sub-tiles; the lane holds features 8*(r/4) + 4*lhi + (r%4) of
// each.  cb = first GEMM column of the patch (a multiple of 64).
template <int EPI>
__device__ __forceinline__ void epilogue_patch(const GemmParams& p, int row, int64_t pos, int cb, int lhi,
                                               const f32x16& c0, const f32x16& c1) {
    if (EPI == EPI_SILU_MUL) {
        // sub-tile 0 = gate, sub-tile 1 = up of the same 32 features (weight rows interleaved)
        bf16_t* drow = p.dst + (int64_t)row * p.ld + cb / 2 + 4 * lhi;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
            *(uint2*)(drow + 8 * g4) =
                pack4(silu_f(c0[4 * g4]) * c1[4 * g4], silu_f(c0[4 * g4 + 1]) * c1[4 * g4 + 1],
                      silu_f(c0[4 * g4 + 2]) * c1[4 * g4 + 2], silu_f(c0[4 * g4 + 3]) * c1[4 * g4 + 3]);
    } else if (EPI == EPI_QKV_ROPE) {
        const int half = p.hd >> 1;
        if (cb < p.qd + p.kvd) {
            // Q or K patch: sub-tile 0 holds rotary index i, sub-tile 1 holds i + hd/2 (the
            // weight rows were packed that way), so a pair sits in one lane, same register.
            const bool is_q = cb < p.qd;
            const float qs = is_q ? p.q_scale : 1.0f;
            const int c = is_q ? cb : cb - p.qd;
            const int head = c / p.hd;
            const int patch = (c - head * p.hd) >> 6;
            const int i0 = patch * 32 + 4 * lhi;             // rotary index of register quad 0
            bf16_t* drow = (is_q ? p.dst + (int64_t)row * p.qd : p.dst_k + (int64_t)row * p.kvd) + head * p.hd + i0;
            const float* ct = p.rope_cos + pos * half + i0;
            const float* st = p.rope_sin + pos * half + i0;
            const bf16_t* bp = p.bias ? p.bias + cb + 4 * lhi : nullptr;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const float4 cs = *(const float4*)(ct + 8 * g4);
                const float4 sn = *(const float4*)(st + 8 * g4);
                const float cv[4] = {cs.x, cs.y, cs.z, cs.w}, sv[4] = {sn.x, sn.y, sn.z, sn.w};
                float lo[4], hi[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float a = c0[4 * g4 + e], b = c1[4 * g4 + e];
                    if (bp) { a += bf2f(bp[8 * g4 + e]); b += bf2f(bp[32 + 8 * g4 + e]); }
                    lo[e] = (a * cv[e] - b * sv[e]) * qs;
                    hi[e] = (b * cv[e] + a * sv[e]) * qs;
                }
                *(uint2*)(drow + 8 * g4) = pack4(lo[0], lo[1], lo[2], lo[3]);
                *(uint2*)(drow + half + 8 * g4) = pack4(hi[0], hi[1], hi[2], hi[3]);
            }
        } else {
            // V patch: stored transposed, V^T[feature][position]; consecutive lanes are
            // consecutive positions.
            const int f0 = cb - p.qd - p.kvd + 4 * lhi;
            bf16_t* dcol = p.dst_vt + p.pos0 + row;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int f = f0 + 8 * (r >> 2) + (r & 3);
                float v0 = c0[r], v1 = c1[r];
                if (p.bias) { v0 += bf2f(p.bias[p.qd + p.kvd + f]); v1 += bf2f(p.bias[p.qd + p.kvd + f + 32]); }
                dcol[(int64_t)f * p.ldv] = f2bf(v0);
                dcol[(int64_t)(f + 32) * p.ldv] = f2bf(v1);
            }
        }
    } else {
        // (N is a multiple of 64, so a patch is either wholly inside or wholly outside)
        // The residual may alias the destination (in-place update of the residual stream):
        // all eight 8-byte pieces of this lane are read before the first one is written,
        // so the loads are issued back to back instead of one per store.
        uint2 rw[2][4];
        if (EPI == EPI_RESIDUAL) {
            const bf16_t* rrow = p.R + (int64_t)row * p.ldr + cb + 4 * lhi;
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) rw[ni][g4] = *(const uint2*)(rrow + ni * 32 + 8 * g4);
        }
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const f32x16& cc = ni ? c1 : c0;
            const int col = cb + ni * 32 + 4 * lhi;
            bf16_t* drow = p.dst + (int64_t)row * p.ld + col;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                float v[4] = {cc[4 * g4], cc[4 * g4 + 1], cc[4 * g4 + 2], cc[4 * g4 + 3]};
                if (EPI == EPI_STORE && p.bias) {
                    const uint2 bw = *(const uint2*)(p.bias + col + 8 * g4);
                    v[0] += __uint_as_float(bw.x << 16); v[1] += __uint_as_float(bw.x & 0xffff0000u);
                    v[2] += __uint_as_float(bw.y << 16); v[3] += __uint_as_float(bw.y & 0xffff0000u);
                }
                if (EPI == EPI_RESIDUAL) {
                    v[0] += __uint_as_float(rw[ni][g4].x << 16); v[1] += __uint_as_float(rw[ni][g4].x & 0xffff0000u);
                    v[2] += __uint_as_float(rw[ni][g4].y << 16); v[3] += __uint_as_float(rw[ni][g4].y & 0xffff0000u);
                }
                *(uint2*)(drow + 8 * g4) = pack4(v[0], v[1], v[2], v[3]);
            }
        }
    }
}

// Epilogue of a 256 x 256 block tile whose accumulators sit in the 2 x 2 wavefront layout of both GEMM
// kernels (wavefront = 128 x 128 patch of 4 x 4 MFMA 32x32 tiles; a lane holds one token row and runs of
// four consecutive features).  smem: at least 8 KiB per wavefront, free to overwrite (callers synchronise
// the workgroup before).
// In an accumulator tile a lane holds one token row and runs of four consecutive
// features, so storing from there puts 8 bytes per lane into 32 different rows: partial cache lines,
// which the memory side handles several times slower than whole ones.  The position-wise epilogues
// therefore pass their results through LDS (the ring is free now; every wavefront uses 8 KiB of its
// own, so no further workgroup barrier is needed) one 32-row tile row at a time and store 16 bytes per
// lane, a wavefront covering whole row segments.  16-byte groups of a staged row are XOR-swizzled with
// the row number so that both the writes (lane = row) and the reads (lanes along a row) are free of
// bank conflicts.  The arithmetic (fp32 bias / residual add / SiLU-multiply, one round-to-nearest-even
// conversion) is the per-lane one.  QKV keeps the per-lane path (rotary pairs, V^T).
template <int EPI>
__device__ __forceinline__ void tile_epilogue(const GemmParams& p, const f32x16 (&acc)[4][4], unsigned char* smem,
                                              int m0, int n0, int wave, int elane) {
    const int e31 = elane & 31, ehi = elane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    unsigned char* stg = smem + wave * 8192;
    const int row_base = m0 + wm * 128, col_base = n0 + wn * 128;
    if (EPI == EPI_QKV_ROPE) {
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
            const int row = row_base + mi * 32 + e31;
            if (row >= p.M) continue;
            const int64_t pos = p.row_pos ? (int64_t)p.row_pos[p.pos0 + row] : p.pos0 + row;
#pragma unroll
            for (int pt = 0; pt < 2; ++pt) {
                const int cb = col_base + pt * 64;
                if (cb >= p.N) continue;
                epilogue_patch<EPI>(p, row, pos, cb, ehi, acc[mi][2 * pt], acc[mi][2 * pt + 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else if (EPI == EPI_RESIDUAL) {
        // 32 rows x 64 features at a time as fp32 (256-byte rows, 16 groups), then 8 consecutive features
        // per lane: + residual (read 16 bytes per lane; it may alias the destination), convert, store
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
#pragma unroll
                for (int n2 = 0; n2 < 2; ++n2)
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4) {
                        const f32x16& cc = acc[mi][2 * hf + n2];
                        float4 v = {cc[4 * g4], cc[4 * g4 + 1], cc[4 * g4 + 2], cc[4 * g4 + 3]};
                        const int grp = n2 * 8 + 2 * g4 + ehi;             // 4 features = one 16-byte group
                        *(float4*)(stg + e31 * 256 + ((grp ^ (e31 & 15)) << 4)) = v;
                    }
                asm volatile("" ::: "memory");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_sched_barrier(0);
                const int col = col_base + hf * 64 + (elane & 7) * 8;
                uint4 rr[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = row_base + mi * 32 + i * 8 + (elane >> 3);
                    rr[i] = make_uint4(0, 0, 0, 0);
                    if (row < p.M && col < p.N) rr[i] = *(const uint4*)(p.R + (int64_t)row * p.ldr + col);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int rl = i * 8 + (elane >> 3);
                    const int row = row_base + mi * 32 + rl;
                    const int g0 = (elane & 7) * 2;
                    const float4 x0 = *(const float4*)(stg + rl * 256 + ((g0 ^ (rl & 15)) << 4));
                    const float4 x1 = *(const float4*)(stg + rl * 256 + (((g0 + 1) ^ (rl & 15)) << 4));
                    uint4 o;
                    o.x = (uint32_t)f2bf(x0.x + __uint_as_float(rr[i].x << 16)) | ((uint32_t)f2bf(x0.y + __uint_as_float(rr[i].x & 0xffff0000u)) << 16);
                    o.y = (uint32_t)f2bf(x0.z + __uint_as_float(rr[i].y << 16)) | ((uint32_t)f2bf(x0.w + __uint_as_float(rr[i].y & 0xffff0000u)) << 16);
                    o.z = (uint32_t)f2bf(x1.x + __uint_as_float(rr[i].z << 16)) | ((uint32_t)f2bf(x1.y + __uint_as_float(rr[i].z & 0xffff0000u)) << 16);
                    o.w = (uint32_t)f2bf(x1.z + __uint_as_float(rr[i].w << 16)) | ((uint32_t)f2bf(x1.w + __uint_as_float(rr[i].w & 0xffff0000u)) << 16);
                    if (row < p.M && col < p.N) *(uint4*)(p.dst + (int64_t)row * p.ld + col) = o;
                }
                asm volatile("" ::: "memory");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
    } else if (EPI == EPI_PARTIAL) {
        // split-K partial sums: staged like the residual epilogue, stored as fp32 (32 bytes per lane, a
        // wavefront covering 8 rows x 256 bytes); p.dst is the split's float plane, p.ld its row pitch in floats
        float* part = (float*)p.dst;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
#pragma unroll
                for (int n2 = 0; n2 < 2; ++n2)
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4) {
                        const f32x16& cc = acc[mi][2 * hf + n2];
                        float4 v = {cc[4 * g4], cc[4 * g4 + 1], cc[4 * g4 + 2], cc[4 * g4 + 3]};
                        const int grp = n2 * 8 + 2 * g4 + ehi;
                        *(float4*)(stg + e31 * 256 + ((grp ^ (e31 & 15)) << 4)) = v;
                    }
                asm volatile("" ::: "memory");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_sched_barrier(0);
                const int col = col_base + hf * 64 + (elane & 7) * 8;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int rl = i * 8 + (elane >> 3);
                    const int row = row_base + mi * 32 + rl;
                    const int g0 = (elane & 7) * 2;
                    const float4 x0 = *(const float4*)(stg + rl * 256 + ((g0 ^ (rl & 15)) << 4));
                    const float4 x1 = *(const float4*)(stg + rl * 256 + (((g0 + 1) ^ (rl & 15)) << 4));
                    if (row < p.M && col < p.N) {
                        *(float4*)(part + (int64_t)row * p.ld + col) = x0;
                        *(float4*)(part + (int64_t)row * p.ld + col + 4) = x1;
                    }
                }
                asm volatile("" ::: "memory");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
    } else if (EPI == EPI_STORE) {
        // 32 rows x 128 features at a time as bf16 (256-byte rows, 16 groups)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const f32x16& cc = acc[mi][ni];
                    const int c = ni * 32 + 8 * g4 + 4 * ehi;
                    float v[4] = {cc[4 * g4], cc[4 * g4 + 1], cc[4 * g4 + 2], cc[4 * g4 + 3]};
                    if (p.bias && col_base + c < p.N) {
                        const uint2 bw = *(const uint2*)(p.bias + col_base + c);
                        v[0] += __uint_as_float(bw.x << 16); v[1] += __uint_as_float(bw.x & 0xffff0000u);
                        v[2] += __uint_as_float(bw.y << 16); v[3] += __uint_as_float(bw.y & 0xffff0000u);
                    }
                    const int grp = ni * 4 + g4;                           // 8 features = one 16-byte group
                    *(uint2*)(stg + e31 * 256 + ((grp ^ (e31 & 15)) << 4) + ehi * 8) = pack4(v[0], v[1], v[2], v[3]);
                }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
            const int col = col_base + (elane & 15) * 8;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int rl = i * 4 + (elane >> 4);
                const int row = row_base + mi * 32 + rl;
                const uint4 o = *(const uint4*)(stg + rl * 256 + (((elane & 15) ^ (rl & 15)) << 4));
                if (row < p.M && col < p.N) *(uint4*)(p.dst + (int64_t)row * p.ld + col) = o;
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        // SiLU-multiply: a 64-column patch (32 gate, 32 up) gives 32 features; 32 rows x 64 features at a
        // time as bf16 (128-byte rows, 8 groups, two rows per 256 bytes of banks: swizzle with row / 2);
        // a wavefront then stores 8 rows x 128 bytes per instruction
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const f32x16& c0 = acc[mi][2 * pt];
                    const f32x16& c1 = acc[mi][2 * pt + 1];
                    const int grp = pt * 4 + g4;
                    *(uint2*)(stg + e31 * 128 + ((grp ^ ((e31 >> 1) & 7)) << 4) + ehi * 8) =
                        pack4(silu_f(c0[4 * g4]) * c1[4 * g4], silu_f(c0[4 * g4 + 1]) * c1[4 * g4 + 1],
                              silu_f(c0[4 * g4 + 2]) * c1[4 * g4 + 2], silu_f(c0[4 * g4 + 3]) * c1[4 * g4 + 3]);
                }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
            const int col = col_base / 2 + (elane & 7) * 8;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rl = i * 8 + (elane >> 3);
                const int row = row_base + mi * 32 + rl;
                const uint4 o = *(const uint4*)(stg + rl * 128 + (((elane & 7) ^ ((rl >> 1) & 7)) << 4));
                if (row < p.M && col < p.N / 2) *(uint4*)(p.dst + (int64_t)row * p.ld + col) = o;
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

// Epilogue of a 256 x 256 block tile whose accumulators sit in the layout of the bf16 GEMM: eight wavefronts
// arranged 2 x 4, each a 128-row x 64-column patch of 8 x 4 MFMA 16x16 tiles; in tile (u, t) a lane holds token
// row 16 u + (lane & 15) and the four consecutive features 16 t + 4 (lane >> 4) + r.  A wavefront's 64 columns are
// exactly one patch of the packed weights: tiles 0, 1 hold the gate values / the first rotary halves of 32
// features, tiles 2, 3 the up values / second halves, so a lane finds a pair in the same register of tiles t, t + 2.
// The position-wise results pass through LDS (8 KiB per wavefront, wave-private, 16-byte groups XOR-swizzled with
// the row so that the writes, lane = row, and the reads, lanes along a row, are free of bank conflicts) and leave
// as 16 bytes per lane covering whole row segments; QKV keeps a per-lane path (rotary pairs, V^T).
// smem: at least 8 KiB per wavefront, free to overwrite (callers synchronise the workgroup before).
template <int EPI, int MU>
__device__ __forceinline__ void tile_epilogue16(const GemmParams& p, const f32x4 (&acc)[MU][4], unsigned char* smem,
                                                int m0, int n0, int wave, int lane) {
    const int l15 = lane & 15, l4 = lane >> 4;
    const int wm = wave >> 2, wn = wave & 3;
    unsigned char* stg = smem + wave * 8192;
    const int row_base = m0 + wm * (MU * 16), col_base = n0 + wn * 64;
    if (col_base >= p.N) return;                       // (N is a multiple of 64: a patch is wholly in or out)
    if (EPI == EPI_QKV_ROPE) {
        const int half = p.hd >> 1;
        const int cb = col_base;
        // (bias or not, whole patch or ragged: decided once per patch, wavefront-uniform, outside the unrolled loops --
        //  a test per element costs a scalar branch each, hundreds per patch, in a part of the kernel no MFMA overlaps)
        if (cb < p.qd + p.kvd) {
            const bool is_q = cb < p.qd;
            const float qs = is_q ? p.q_scale : 1.0f;
            const int c = is_q ? cb : cb - p.qd;
            const int head = c / p.hd;
            const int patch = (c - head * p.hd) >> 6;
            auto qk_patch = [&](auto has_bias) {
                constexpr bool HB = decltype(has_bias)::value;
                float ba[2][4], bb[2][4];
                if (HB) {
#pragma unroll
                    for (int t = 0; t < 2; ++t)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            ba[t][e] = bf2f(p.bias[cb + t * 16 + 4 * l4 + e]);
                            bb[t][e] = bf2f(p.bias[cb + 32 + t * 16 + 4 * l4 + e]);
                        }
                }
#pragma unroll
                for (int u = 0; u < MU; ++u) {
                    const int row = row_base + u * 16 + l15;
                    if (row >= p.M) continue;
                    const int64_t pos = p.row_pos ? (int64_t)p.row_pos[p.pos0 + row] : p.pos0 + row;
                    bf16_t* drow = (is_q ? p.dst + (int64_t)row * p.qd : p.dst_k + (int64_t)row * p.kvd) + head * p.hd;
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const int i0 = patch * 32 + t * 16 + 4 * l4;             // rotary index of register 0
                        const float4 cs = *(const float4*)(p.rope_cos + pos * half + i0);
                        const float4 sn = *(const float4*)(p.rope_sin + pos * half + i0);
                        const float cv[4] = {cs.x, cs.y, cs.z, cs.w}, sv[4] = {sn.x, sn.y, sn.z, sn.w};
                        float lo[4], hi[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float a = acc[u][t][e], b = acc[u][t + 2][e];
                            if (HB) { a += ba[t][e]; b += bb[t][e]; }
                            lo[e] = (a * cv[e] - b * sv[e]) * qs;
                            hi[e] = (b * cv[e] + a * sv[e]) * qs;
                        }
                        *(uint2*)(drow + i0) = pack4(lo[0], lo[1], lo[2], lo[3]);
                        *(uint2*)(drow + half + i0) = pack4(hi[0], hi[1], hi[2], hi[3]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            if (p.bias) qk_patch(std::true_type{});
            else qk_patch(std::false_type{});
        } else {
            // V patch: stored transposed, V^T[feature][position]; consecutive lanes are consecutive positions.  One
            // address per (tile column, register) and lane; the eight row groups of the patch are fixed offsets from it.
            const int f0 = cb - p.qd - p.kvd;
            bf16_t* const dbase = p.dst_vt + p.pos0 + row_base + l15;
            auto v_patch = [&](auto has_bias, auto whole) {
                constexpr bool HB = decltype(has_bias)::value, WHOLE = decltype(whole)::value;
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int f = f0 + t * 16 + 4 * l4 + e;
                        bf16_t* const dp = dbase + (int64_t)f * p.ldv;
                        float bv = 0.f;
                        if (HB) bv = bf2f(p.bias[p.qd + p.kvd + f]);
#pragma unroll
                        for (int u = 0; u < MU; ++u) {
                            float v = acc[u][t][e];
                            if (HB) v += bv;
                            if (WHOLE || row_base + u * 16 + l15 < p.M) dp[u * 16] = f2bf(v);
                        }
                    }
            };
            const bool whole = row_base + MU * 16 <= p.M;
            if (p.bias) {
                if (whole) v_patch(std::true_type{}, std::true_type{});
                else v_patch(std::true_type{}, std::false_type{});
            } else {
                if (whole) v_patch(std::false_type{}, std::true_type{});
                else v_patch(std::false_type{}, std::false_type{});
            }
        }
    } else if (EPI == EPI_RESIDUAL || EPI == EPI_PARTIAL) {
        // 16 rows x 64 features at a time as fp32 (256-byte rows, 16 groups of 4 features = one accumulator tile
        // register quad), then 8 consecutive features per lane, 8 rows per pass
        const int col = col_base + (lane & 7) * 8;
#pragma unroll
        for (int u = 0; u < MU; ++u) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                *(f32x4*)(stg + l15 * 256 + (((t * 4 + l4) ^ l15) << 4)) = acc[u][t];
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
            uint4 rr[2];
            if (EPI == EPI_RESIDUAL) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int row = row_base + u * 16 + i * 8 + (lane >> 3);
                    rr[i] = make_uint4(0, 0, 0, 0);
                    if (row < p.M) rr[i] = *(const uint4*)(p.R + (int64_t)row * p.ldr + col);
                }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int rl = i * 8 + (lane >> 3);
                const int row = row_base + u * 16 + rl;
                const int g0 = (lane & 7) * 2;
                const float4 x0 = *(const float4*)(stg + rl * 256 + ((g0 ^ rl) << 4));
                const float4 x1 = *(const float4*)(stg + rl * 256 + (((g0 + 1) ^ rl) << 4));
                if (EPI == EPI_PARTIAL) {
                    float* part = (float*)p.dst;                 // this split's float plane, p.ld its row pitch in floats
                    if (row < p.M) {
                        *(float4*)(part + (int64_t)row * p.ld + col) = x0;
                        *(float4*)(part + (int64_t)row * p.ld + col + 4) = x1;
                    }
                } else {
                    uint4 o;
                    o.x = (uint32_t)f2bf(x0.x + __uint_as_float(rr[i].x << 16)) | ((uint32_t)f2bf(x0.y + __uint_as_float(rr[i].x & 0xffff0000u)) << 16);
                    o.y = (uint32_t)f2bf(x0.z + __uint_as_float(rr[i].y << 16)) | ((uint32_t)f2bf(x0.w + __uint_as_float(rr[i].y & 0xffff0000u)) << 16);
                    o.z = (uint32_t)f2bf(x1.x + __uint_as_float(rr[i].z << 16)) | ((uint32_t)f2bf(x1.y + __uint_as_float(rr[i].z & 0xffff0000u)) << 16);
                    o.w = (uint32_t)f2bf(x1.z + __uint_as_float(rr[i].w << 16)) | ((uint32_t)f2bf(x1.w + __uint_as_float(rr[i].w & 0xffff0000u)) << 16);
                    if (row < p.M) *(uint4*)(p.dst + (int64_t)row * p.ld + col) = o;
                }
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
    } else if (EPI == EPI_STORE) {
        // 16 rows x 64 features at a time as bf16 (128-byte rows, 8 groups of 8 features; two rows per 256 bytes of
        // banks: swizzle with row / 2), then 8 features per lane, 8 rows per pass
        const int col = col_base + (lane & 7) * 8;
#pragma unroll
        for (int u = 0; u < MU; ++u) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                float v[4] = {acc[u][t][0], acc[u][t][1], acc[u][t][2], acc[u][t][3]};
                if (p.bias) {
                    const uint2 bw = *(const uint2*)(p.bias + col_base + t * 16 + 4 * l4);
                    v[0] += __uint_as_float(bw.x << 16); v[1] += __uint_as_float(bw.x & 0xffff0000u);
                    v[2] += __uint_as_float(bw.y << 16); v[3] += __uint_as_float(bw.y & 0xffff0000u);
                }
                const int grp = t * 2 + (l4 >> 1);
                *(uint2*)(stg + l15 * 128 + ((grp ^ ((l15 >> 1) & 7)) << 4) + (l4 & 1) * 8) = pack4(v[0], v[1], v[2], v[3]);
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int rl = i * 8 + (lane >> 3);
                const int row = row_base + u * 16 + rl;
                const uint4 o = *(const uint4*)(stg + rl * 128 + (((lane & 7) ^ ((rl >> 1) & 7)) << 4));
                if (row < p.M) *(uint4*)(p.dst + (int64_t)row * p.ld + col) = o;
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        // SiLU-multiply: the patch (32 gate, 32 up) gives 32 features; 16 rows x 32 features at a time as bf16
        // (64-byte rows, 4 groups of 8 features; four rows per 256 bytes of banks: swizzle with row / 4), then 8
        // features per lane: one pass stores all 16 rows, 64 contiguous bytes each
        const int col = col_base / 2 + (lane & 3) * 8;
#pragma unroll
        for (int u = 0; u < MU; ++u) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const f32x4& g = acc[u][t];
                const f32x4& up = acc[u][t + 2];
                const int grp = t * 2 + (l4 >> 1);
                *(uint2*)(stg + l15 * 64 + ((grp ^ ((l15 >> 2) & 3)) << 4) + (l4 & 1) * 8) =
                    pack4(silu_f(g[0]) * up[0], silu_f(g[1]) * up[1], silu_f(g[2]) * up[2], silu_f(g[3]) * up[3]);
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
            {
                const int rl = lane >> 2;
                const int row = row_base + u * 16 + rl;
                const uint4 o = *(const uint4*)(stg + rl * 64 + (((lane & 3) ^ ((rl >> 2) & 3)) << 4));
                if (row < p.M) *(uint4*)(p.dst + (int64_t)row * p.ld + col) = o;
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// ---- split-K support shared by the bf16 and the FP8 GEMM (defined with the bf16 kernel)
// splits of the reduction for a GEMM with few output tiles whose K range has kt slices: enough workgroups for
// the chip's 256 compute units, whole slices, at least two per split, fp32 partials within part_bytes; 1 = none
int pick_splits(int64_t M, int N, int kt, size_t part_bytes);
// the kernels that add up part[split][M][N] in split order and apply an epilogue
void launch_splitk_reduce_residual(const float* part, int splits, const bf16_t* R, int64_t ldr, bf16_t* C, int64_t ldc,
                                   int64_t M, int N, hipStream_t s);
void launch_splitk_reduce_silu(const float* part, int splits, bf16_t* H, int64_t ldh, int64_t M, int N, hipStream_t s);
// r: the parameters launch_gemm_qkv_rope would pass (bias, destinations, rotary table, positions, widths)
void launch_splitk_reduce_qkv(const float* part, int splits, const GemmParams& r, hipStream_t s);

}  // namespace gemm
}  // namespace po
