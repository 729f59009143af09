// Float32-path kernels on the float32 matrix instruction (gfx950): causal GQA attention and the GEMM.
// Operands, products and sums are float32 throughout (v_mfma_f32_32x32x2_f32); nothing is rounded to a narrower
// type.  The float32 path is the one that is held to 1e-4 against the float64 definition and that stands in for it
// at configurations no CPU run reaches, so what matters here is that every output is one float32 dot product in a
// fixed order that depends on nothing but its own row and column; speed only has to be enough for whole
// configurations (32 layers x 32768 tokens) to run in seconds.
#include "po_internal.h"

namespace po {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__device__ __forceinline__ f32x16 mfma_f32(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// ------------------------------------------------------------------ attention
// softmax(Q K^T / sqrt(hd)) V with the causal mask, grouped-query heads (Section 4.2 of the paper: attention runs
// over the whole sequence, unchunked).  Workgroup = 128 query rows of one head, wavefront = 32 of them.  Keys go by
// in tiles of 32 staged in LDS (K rows padded by 4 floats, V rows as they are).  Per tile a wavefront forms
// S^T[key][query] = K Q^T with 64 (hd 128) matrix instructions, so that a lane owns ONE query column -- lane l and
// lane l ^ 32 share it, 16 keys each -- and the online softmax needs one exchange with the partner lane per tile;
// the probabilities never leave their registers: register r of S^T is exactly the B operand of step r of
// O^T[hd][query] += V^T P^T when the V fragment of that step is read at the key that register r holds.
// The contraction index of Q K^T is split between the lane halves (half h takes elements [h hd/2, (h+1) hd/2)), so
// that a lane's K fragment is contiguous in LDS (16-byte reads).
// A query's result depends only on its own column of S^T and on the tile grid, which starts at key 0 for every
// workgroup: it is the same bits wherever the row sits in a workgroup and whichever rows are computed beside it
// (tiles wholly above a wavefront's rows are skipped; they would contribute p = 0 and a rescale by 1, exactly).
// o may alias q: a wavefront reads its own 32 query rows before it writes them, and nobody else touches them.
template <int HD>
__global__ void __launch_bounds__(256, HD == 128 ? 1 : 2) attention_f32_mfma_kernel(const float* q, const float* __restrict__ k,
                                                                    const float* __restrict__ v, float* o, int64_t N,
                                                                    int Hq, int Hkv, int64_t blk0) {
    constexpr int KP = HD + 4;        // padded K row: 8 lanes' 16-byte reads fall into different banks
    constexpr int HH = HD / 2;        // contraction elements per lane half
    constexpr int NB = HD / 32;       // 32-row blocks of O^T
    constexpr int V4 = HD / 32;       // float4 per thread and operand of one staged tile (32 rows x HD floats, 256 threads)
    constexpr int RV = HD / 4;        // float4 per row
    __shared__ __align__(16) float Ks[32 * KP];
    __shared__ __align__(16) float Vs[32 * HD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int h = blockIdx.y;
    const int c = h / (Hq / Hkv);
    const int64_t r0 = ((int64_t)(gridDim.x - 1 - blockIdx.x) + blk0) * 128;      // longest rows first
    const int64_t q0 = r0 + wave * 32;          // this wavefront's first query row
    const int64_t t = q0 + col;                 // this lane's query row
    const bool live = t < N;
    const float scale = 1.0f / sqrtf((float)HD);

    float qf[HH];
    {
        const float* qp = q + (t * Hq + h) * HD + half * HH;
#pragma unroll
        for (int i = 0; i < HH / 4; ++i) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (live) x = *(const float4*)(qp + 4 * i);
            qf[4 * i] = x.x; qf[4 * i + 1] = x.y; qf[4 * i + 2] = x.z; qf[4 * i + 3] = x.w;
        }
    }
    f32x16 O[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[b][r] = 0.f;
    float m = -INFINITY, l = 0.f;

    const int64_t kv_end = (r0 + 128 < N) ? r0 + 128 : N;
    float4 pk[V4], pv[V4];
    auto fetch = [&](int64_t kv0) {
#pragma unroll
        for (int j = 0; j < V4; ++j) {
            const int idx = tid + 256 * j;
            const int64_t s = kv0 + idx / RV;
            const int c4 = idx % RV;
            pk[j] = pv[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (s < N) {
                pk[j] = *(const float4*)(k + (s * Hkv + c) * HD + 4 * c4);
                pv[j] = *(const float4*)(v + (s * Hkv + c) * HD + 4 * c4);
            }
        }
    };
    fetch(0);
    for (int64_t kv0 = 0; kv0 < kv_end; kv0 += 32) {
        __syncthreads();                        // everybody is done reading the previous tile
#pragma unroll
        for (int j = 0; j < V4; ++j) {
            const int idx = tid + 256 * j;
            const int row = idx / RV, c4 = idx % RV;
            *(float4*)(Ks + row * KP + 4 * c4) = pk[j];
            *(float4*)(Vs + row * HD + 4 * c4) = pv[j];
        }
        __syncthreads();
        if (kv0 + 32 < kv_end) fetch(kv0 + 32);          // in flight during this tile's arithmetic
        if (kv0 > q0 + 31) continue;                     // wavefront-uniform: every key of the tile is masked for these rows

        f32x16 S;
#pragma unroll
        for (int r = 0; r < 16; ++r) S[r] = 0.f;
        const float* kr = Ks + col * KP + half * HH;
#pragma unroll
        for (int i = 0; i < HH / 4; ++i) {
            const float4 kk = *(const float4*)(kr + 4 * i);
            S = mfma_f32(kk.x, qf[4 * i], S);
            S = mfma_f32(kk.y, qf[4 * i + 1], S);
            S = mfma_f32(kk.z, qf[4 * i + 2], S);
            S = mfma_f32(kk.w, qf[4 * i + 3], S);
        }
        // register r holds key kv0 + 8 (r / 4) + 4 half + r % 4 of query t
        float p[16];
        float tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t key = kv0 + 8 * (r / 4) + 4 * half + (r % 4);
            p[r] = key > t ? -INFINITY : S[r] * scale;
            tmax = fmaxf(tmax, p[r]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float mn = fmaxf(m, tmax);                 // finite: key kv0 <= q0 <= t is never masked
        const float a = expf(m - mn);                    // exp(-inf) = 0 on the first tile
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            p[r] = expf(p[r] - mn);
            psum += p[r];
        }
        l = l * a + psum;                                // this lane's 16 keys; the partner's are added at the end
        m = mn;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) O[b][r] *= a;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float vv = Vs[(8 * (r / 4) + 4 * half + (r % 4)) * HD + 32 * b + col];
                O[b] = mfma_f32(vv, p[r], O[b]);
            }
        }
    }
    l += __shfl_xor(l, 32);
    if (!live) return;
    const float inv = 1.0f / l;
    float* op = o + (t * Hq + h) * HD;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g)
            *(float4*)(op + 32 * b + 8 * g + 4 * half) =
                make_float4(O[b][4 * g] * inv, O[b][4 * g + 1] * inv, O[b][4 * g + 2] * inv, O[b][4 * g + 3] * inv);
}

// q_row0: rows below it need no result (the workgroup that holds it still computes its rows from the 128-row
// boundary on; what it writes below q_row0 nobody reads)
bool launch_attention_f32_mfma(const float* q, const float* k, const float* v, float* o, int64_t N, int Hq, int Hkv, int hd,
                               int64_t q_row0, hipStream_t s) {
    if (N <= 0) return true;
    if (hd != 64 && hd != 128) return false;
    const int64_t blk0 = (q_row0 > 0 && q_row0 < N) ? q_row0 / 128 : 0;
    const dim3 grid((unsigned)((N + 127) / 128 - blk0), (unsigned)Hq);
    if (hd == 128)
        hipLaunchKernelGGL(attention_f32_mfma_kernel<128>, grid, dim3(256), 0, s, q, k, v, o, N, Hq, Hkv, blk0);
    else
        hipLaunchKernelGGL(attention_f32_mfma_kernel<64>, grid, dim3(256), 0, s, q, k, v, o, N, Hq, Hkv, blk0);
    return true;
}

// ------------------------------------------------------------------ GEMM
// C[M,N] = A[M,K] W[N,K]^T (+bias) (+R), all float32.  Workgroup = 128 x 128 outputs, wavefront = 64 x 64 (2 x 2
// tiles of 32 x 32), K in slices of 32 staged in LDS (rows padded to 36 floats).  The instruction is issued as
// W-fragment x A-fragment^T, so a lane holds one row of C and four consecutive columns per register group (16-byte
// stores); within a slice lane half h multiplies elements [16 h, 16 h + 16) so that its fragments are contiguous.
// Every output is one running sum over K in one fixed order, whatever M, N and the tiling: row results do not
// depend on which other rows a launch computes.  C may alias R (a lane reads the residual it then overwrites).
__global__ void __launch_bounds__(256, 2) gemm_f32_mfma_kernel(const float* __restrict__ A, int64_t lda,
                                                               const float* __restrict__ W, int64_t ldw, float* C,
                                                               int64_t ldc, const float* __restrict__ bias, const float* R,
                                                               int64_t ldr, int64_t M, int N, int K) {
    constexpr int SP = 36;
    __shared__ __align__(16) float As[128 * SP];
    __shared__ __align__(16) float Ws[128 * SP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.y * 128;
    const int n0 = blockIdx.x * 128;
    f32x16 acc[2][2];                       // [feature tile][token tile]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    float4 pa[4], pw[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = tid + 256 * j;
            const int row = idx >> 3, gk = k0 + 4 * (idx & 7);
            pa[j] = pw[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (gk < K) {
                if (m0 + row < M) pa[j] = *(const float4*)(A + (m0 + row) * lda + gk);
                if (n0 + row < N) pw[j] = *(const float4*)(W + (int64_t)(n0 + row) * ldw + gk);
            }
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += 32) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = tid + 256 * j;
            const int row = idx >> 3, c4 = idx & 7;
            *(float4*)(As + row * SP + 4 * c4) = pa[j];
            *(float4*)(Ws + row * SP + 4 * c4) = pw[j];
        }
        __syncthreads();
        if (k0 + 32 < K) fetch(k0 + 32);
        const float* ar = As + (wm * 64 + col) * SP + half * 16;
        const float* wr = Ws + (wn * 64 + col) * SP + half * 16;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 a0 = *(const float4*)(ar + 4 * i), a1 = *(const float4*)(ar + 32 * SP + 4 * i);
            const float4 w0 = *(const float4*)(wr + 4 * i), w1 = *(const float4*)(wr + 32 * SP + 4 * i);
            const float av[2][4] = {{a0.x, a0.y, a0.z, a0.w}, {a1.x, a1.y, a1.z, a1.w}};
            const float wv[2][4] = {{w0.x, w0.y, w0.z, w0.w}, {w1.x, w1.y, w1.z, w1.w}};
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int fi = 0; fi < 2; ++fi)
#pragma unroll
                    for (int ti = 0; ti < 2; ++ti) acc[fi][ti] = mfma_f32(wv[fi][e], av[ti][e], acc[fi][ti]);
        }
    }
    const bool vec = (N % 4 == 0) && (ldc % 4 == 0) && (!R || ldr % 4 == 0);
#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
        const int64_t gm = m0 + wm * 64 + ti * 32 + col;
        if (gm >= M) continue;
#pragma unroll
        for (int fi = 0; fi < 2; ++fi)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int gn = n0 + wn * 64 + fi * 32 + 8 * g + 4 * half;
                if (gn >= N) continue;
                float x[4] = {acc[fi][ti][4 * g], acc[fi][ti][4 * g + 1], acc[fi][ti][4 * g + 2], acc[fi][ti][4 * g + 3]};
                if (vec) {          // N % 4 == 0 and gn % 4 == 0: the four columns exist
                    if (bias) {
                        const float4 b = *(const float4*)(bias + gn);
                        x[0] += b.x; x[1] += b.y; x[2] += b.z; x[3] += b.w;
                    }
                    if (R) {
                        const float4 r = *(const float4*)(R + gm * ldr + gn);
                        x[0] += r.x; x[1] += r.y; x[2] += r.z; x[3] += r.w;
                    }
                    *(float4*)(C + gm * ldc + gn) = make_float4(x[0], x[1], x[2], x[3]);
                } else {
                    for (int e = 0; e < 4 && gn + e < N; ++e) {
                        float y = x[e];
                        if (bias) y += bias[gn + e];
                        if (R) y += R[gm * ldr + gn + e];
                        C[gm * ldc + gn + e] = y;
                    }
                }
            }
    }
}

// false (nothing launched) when the operands do not allow 16-byte loads along K
bool launch_gemm_f32_mfma(const float* A, int64_t lda, const float* W, int64_t ldw, float* C, int64_t ldc, const float* bias,
                          const float* R, int64_t ldr, int64_t M, int N, int K, hipStream_t s) {
    if (M <= 0 || N <= 0) return true;
    if (K <= 0 || K % 4 || lda % 4 || ldw % 4 || ((uintptr_t)A | (uintptr_t)W | (uintptr_t)C | (uintptr_t)bias | (uintptr_t)R) % 16)
        return false;
    const dim3 grid((unsigned)((N + 127) / 128), (unsigned)((M + 127) / 128));
    hipLaunchKernelGGL(gemm_f32_mfma_kernel, grid, dim3(256), 0, s, A, lda, W, ldw, C, ldc, bias, R, ldr, M, N, K);
    return true;
}

}  // namespace po
