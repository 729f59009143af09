// Bandwidth-bound and fp32-path kernels of libpo (gfx950): embedding gather, RMSNorm,
// rotary table + rotation, a plain fp32-accumulating tiled GEMM, SiLU-multiply, a plain
// attention (one thread per query row), the last-row LM head, candidate log-probs, weight
// packing and the V transpose used by the bf16 attention.  Templated on the storage type
// (float | bf16).  The float32 path takes the plain GEMM and attention only for shapes the
// float32 matrix-instruction kernels (f32_mfma.hip) do not cover.
#include "po_internal.h"

namespace po {

// ------------------------------------------------------------------ embedding gather
// X[t, :] = E[tok[t], :]; one block per token, 16-byte copies (d * elem size % 16 == 0).
__global__ void __launch_bounds__(256) embed_kernel(const int32_t* __restrict__ tok,
                                                    const uint4* __restrict__ E,
                                                    uint4* __restrict__ X, int vec_per_row) {
    const int64_t t = blockIdx.x;
    const uint4* src = E + (int64_t)tok[t] * vec_per_row;
    uint4* dst = X + t * vec_per_row;
    for (int i = threadIdx.x; i < vec_per_row; i += 256) dst[i] = src[i];
}

void launch_embed(int dtype, const int32_t* tok, const void* E, void* X, int64_t n, int d, hipStream_t s) {
    const int esz = dtype == 0 ? 4 : 2;
    hipLaunchKernelGGL(embed_kernel, dim3((unsigned)n), dim3(256), 0, s, tok, (const uint4*)E, (uint4*)X,
                       d * esz / 16);
}

// ------------------------------------------------------------------ RMSNorm
// y = x * rsqrt(mean(x^2) + eps) * g, fp32 reduction; one block per row.
template <typename T>
__global__ void __launch_bounds__(256) rmsnorm_kernel(const T* __restrict__ x, const T* __restrict__ g,
                                                      T* __restrict__ y, int d, float eps) {
    const int64_t row = blockIdx.x;
    const T* xr = x + row * d;
    T* yr = y + row * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) {
        float v = to_f32(xr[i]);
        ss += v * v;
    }
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = part[0] + part[1] + part[2] + part[3];
    const float r = 1.0f / sqrtf(tot / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256) yr[i] = from_f32<T>(to_f32(xr[i]) * r * to_f32(g[i]));
}

// bf16 fast path: 16-byte loads, the row stays in registers (d % 8 == 0, d <= 256*8*4)
__global__ void __launch_bounds__(256) rmsnorm_bf16_vec_kernel(const uint4* __restrict__ x,
                                                               const uint4* __restrict__ g,
                                                               uint4* __restrict__ y, int vecs, float eps,
                                                               float inv_d) {
    const int64_t row = blockIdx.x;
    const uint4* xr = x + row * vecs;
    uint4 v[4];
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int i = threadIdx.x + j * 256;
        if (i < vecs) {
            v[j] = xr[i];
            const uint32_t w[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float lo = __uint_as_float(w[c] << 16), hi = __uint_as_float(w[c] & 0xffff0000u);
                ss += lo * lo + hi * hi;
            }
        }
    }
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float r = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) * inv_d + eps);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int i = threadIdx.x + j * 256;
        if (i < vecs) {
            const uint4 gv = g[i];
            const uint32_t w[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
            const uint32_t gw[4] = {gv.x, gv.y, gv.z, gv.w};
            uint32_t o[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float lo = __uint_as_float(w[c] << 16) * r * __uint_as_float(gw[c] << 16);
                float hi = __uint_as_float(w[c] & 0xffff0000u) * r * __uint_as_float(gw[c] & 0xffff0000u);
                o[c] = (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
            }
            y[row * vecs + i] = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

void launch_rmsnorm(int dtype, const void* x, const void* g, void* y, int64_t rows, int d, float eps,
                    hipStream_t s) {
    if (rows <= 0) return;
    if (dtype == 0) {
        hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3((unsigned)rows), dim3(256), 0, s, (const float*)x,
                           (const float*)g, (float*)y, d, eps);
    } else if (d % 8 == 0 && d <= 8192) {
        hipLaunchKernelGGL(rmsnorm_bf16_vec_kernel, dim3((unsigned)rows), dim3(256), 0, s, (const uint4*)x,
                           (const uint4*)g, (uint4*)y, d / 8, eps, 1.0f / (float)d);
    } else {
        hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3((unsigned)rows), dim3(256), 0, s, (const bf16_t*)x,
                           (const bf16_t*)g, (bf16_t*)y, d, eps);
    }
}

// ------------------------------------------------------------------ rotary embedding
// Table: cos/sin of pos * theta^(-2i/hd), formed in fp64 so that position 131071 keeps
// full fp32 accuracy after rounding.
__global__ void __launch_bounds__(256) rope_table_kernel(float* __restrict__ cos_t, float* __restrict__ sin_t,
                                                         int64_t n, int half, double theta) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * half) return;
    const int64_t t = idx / half;
    const int i = (int)(idx % half);
    const double inv_freq = pow(theta, -(double)i / (double)half);   // theta^(-2i/hd)
    const double ang = (double)t * inv_freq;
    cos_t[idx] = (float)cos(ang);
    sin_t[idx] = (float)sin(ang);
}

void launch_rope_table(float* cos_t, float* sin_t, int64_t n, int hd, float theta, hipStream_t s) {
    const int half = hd / 2;
    const int64_t total = n * half;
    if (total <= 0) return;
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, cos_t, sin_t,
                       n, half, (double)theta);
}

// x[t, h, i], x[t, h, i+half] <- rotate by angle[t, i]   (rotate-half pairing)
template <typename T>
__global__ void __launch_bounds__(256) rope_kernel(T* __restrict__ x, int64_t ld, const float* __restrict__ cos_t,
                                                   const float* __restrict__ sin_t, int64_t n, int H, int half) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t per_row = (int64_t)H * half;
    if (idx >= n * per_row) return;
    const int64_t t = idx / per_row;
    const int rem = (int)(idx % per_row);
    const int h = rem / half, i = rem % half;
    T* p = x + t * ld + (int64_t)h * 2 * half + i;
    const float a = to_f32(p[0]), b = to_f32(p[half]);
    const float c = cos_t[t * half + i], sn = sin_t[t * half + i];
    p[0] = from_f32<T>(a * c - b * sn);
    p[half] = from_f32<T>(b * c + a * sn);
}

void launch_rope(int dtype, void* x, int64_t ld, const float* cos_t, const float* sin_t, int64_t n, int H,
                 int hd, hipStream_t s) {
    const int64_t total = n * H * (hd / 2);
    if (total <= 0) return;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (dtype == 0)
        hipLaunchKernelGGL(rope_kernel<float>, grid, dim3(256), 0, s, (float*)x, ld, cos_t, sin_t, n, H, hd / 2);
    else
        hipLaunchKernelGGL(rope_kernel<bf16_t>, grid, dim3(256), 0, s, (bf16_t*)x, ld, cos_t, sin_t, n, H, hd / 2);
}

// ------------------------------------------------------------------ plain tiled GEMM
// C[M,N] = A[M,K] W[N,K]^T (+bias) (+R); 64x64 tile, 16-deep K slices, 4x4 per thread,
// fp32 accumulation in one fixed order per output (independent of M tiling).
template <typename T>
__global__ void __launch_bounds__(256) gemm_basic_kernel(const T* __restrict__ A, int64_t lda,
                                                         const T* __restrict__ W, int64_t ldw, T* C,
                                                         int64_t ldc, const T* __restrict__ bias, const T* R,
                                                         int64_t ldr, int64_t M, int N, int K) {
    __shared__ float As[16][65];
    __shared__ float Ws[16][65];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t m0 = (int64_t)blockIdx.y * 64;
    const int n0 = blockIdx.x * 64;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = threadIdx.x + 256 * i;
            const int r = idx >> 4, c = idx & 15;
            const int64_t gm = m0 + r;
            const int gn = n0 + r;
            const int gk = k0 + c;
            As[c][r] = (gm < M && gk < K) ? to_f32(A[gm * lda + gk]) : 0.f;
            Ws[c][r] = (gn < N && gk < K) ? to_f32(W[(int64_t)gn * ldw + gk]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = Ws[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            float v = acc[i][j];
            if (bias) v += to_f32(bias[gn]);
            if (R) v += to_f32(R[gm * ldr + gn]);
            C[gm * ldc + gn] = from_f32<T>(v);
        }
    }
}

void launch_gemm_basic(int dtype, const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc,
                       const void* bias, const void* R, int64_t ldr, int64_t M, int N, int K, hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    // float32 operands that allow 16-byte loads: the float32 matrix-instruction kernel
    if (dtype == 0 && launch_gemm_f32_mfma((const float*)A, lda, (const float*)W, ldw, (float*)C, ldc, (const float*)bias,
                                           (const float*)R, ldr, M, N, K, s))
        return;
    const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
    if (dtype == 0)
        hipLaunchKernelGGL(gemm_basic_kernel<float>, grid, dim3(256), 0, s, (const float*)A, lda, (const float*)W,
                           ldw, (float*)C, ldc, (const float*)bias, (const float*)R, ldr, M, N, K);
    else
        hipLaunchKernelGGL(gemm_basic_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)A, lda,
                           (const bf16_t*)W, ldw, (bf16_t*)C, ldc, (const bf16_t*)bias, (const bf16_t*)R, ldr, M,
                           N, K);
}

// ------------------------------------------------------------------ SiLU * up
template <typename T>
__global__ void __launch_bounds__(256) silu_mul_kernel(const T* __restrict__ GU, T* __restrict__ H, int64_t M,
                                                       int F) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * F) return;
    const int64_t r = idx / F;
    const int f = (int)(idx % F);
    const float g = to_f32(GU[r * 2 * F + f]);
    const float u = to_f32(GU[r * 2 * F + F + f]);
    H[idx] = from_f32<T>(g / (1.0f + expf(-g)) * u);
}

void launch_silu_mul(int dtype, const void* GU, void* H, int64_t M, int F, hipStream_t s) {
    const int64_t total = M * F;
    if (total <= 0) return;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (dtype == 0)
        hipLaunchKernelGGL(silu_mul_kernel<float>, grid, dim3(256), 0, s, (const float*)GU, (float*)H, M, F);
    else
        hipLaunchKernelGGL(silu_mul_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)GU, (bf16_t*)H, M, F);
}

// ------------------------------------------------------------------ fp32-path attention
// One thread per (query row, head); 64 consecutive rows of one head per block; K/V tiles
// of 32 keys staged in LDS as fp32; online softmax in fp32.  o may alias q: a thread reads
// its whole q row before anything is written and no other thread reads that row.
template <typename T, int HD>
__global__ void __launch_bounds__(64) attention_basic_kernel(const T* q, const T* __restrict__ k,
                                                             const T* __restrict__ v, T* o, int64_t N, int Hq,
                                                             int Hkv, int64_t blk0) {
    __shared__ float Ks[32][HD];
    __shared__ float Vs[32][HD];
    const int h = blockIdx.y;
    const int c = h / (Hq / Hkv);
    const int64_t r0 = ((int64_t)blockIdx.x + blk0) * 64;
    const int64_t t = r0 + threadIdx.x;
    const bool live = t < N;
    float qv[HD], ov[HD];
    const float scale = 1.0f / sqrtf((float)HD);
#pragma unroll
    for (int i = 0; i < HD; ++i) {
        qv[i] = live ? to_f32(q[(t * Hq + h) * HD + i]) : 0.f;
        ov[i] = 0.f;
    }
    float m = -INFINITY, l = 0.f;
    const int64_t kv_end = (r0 + 64 < N) ? r0 + 64 : N;
    for (int64_t kv0 = 0; kv0 < kv_end; kv0 += 32) {
        for (int idx = threadIdx.x; idx < 32 * HD; idx += 64) {
            const int j = idx / HD, i = idx % HD;
            const int64_t sidx = kv0 + j;
            const bool ok = sidx < N;
            Ks[j][i] = ok ? to_f32(k[(sidx * Hkv + c) * HD + i]) : 0.f;
            Vs[j][i] = ok ? to_f32(v[(sidx * Hkv + c) * HD + i]) : 0.f;
        }
        __syncthreads();
        if (live) {
            for (int j = 0; j < 32; ++j) {
                if (kv0 + j > t) break;
                float dot = 0.f;
#pragma unroll
                for (int i = 0; i < HD; ++i) dot = fmaf(qv[i], Ks[j][i], dot);
                const float sc = dot * scale;
                const float mn = fmaxf(m, sc);
                const float a = expf(m - mn);      // exp(-inf) = 0 on the first key
                const float p = expf(sc - mn);
                l = l * a + p;
#pragma unroll
                for (int i = 0; i < HD; ++i) ov[i] = fmaf(p, Vs[j][i], ov[i] * a);
                m = mn;
            }
        }
        __syncthreads();
    }
    if (live) {
        const float inv = 1.0f / l;
#pragma unroll
        for (int i = 0; i < HD; ++i) o[(t * Hq + h) * HD + i] = from_f32<T>(ov[i] * inv);
    }
}

void launch_attention_basic(int dtype, const void* q, const void* k, const void* v, void* o, int64_t N, int Hq,
                            int Hkv, int hd, int64_t q_row0, hipStream_t s) {
    if (N <= 0) return;
    // float32 with a head dimension the matrix-instruction kernel covers: that one (same definition, ~10x faster)
    if (dtype == 0 && launch_attention_f32_mfma((const float*)q, (const float*)k, (const float*)v, (float*)o, N, Hq, Hkv, hd,
                                                q_row0, s))
        return;
    const int64_t blk0 = (q_row0 > 0 && q_row0 < N) ? q_row0 / 64 : 0;
    const dim3 grid((unsigned)((N + 63) / 64 - blk0), (unsigned)Hq);
#define PO_ATT(T, HDV)                                                                                       \
    hipLaunchKernelGGL((attention_basic_kernel<T, HDV>), grid, dim3(64), 0, s, (const T*)q, (const T*)k,    \
                       (const T*)v, (T*)o, N, Hq, Hkv, blk0)
    if (dtype == 0) {
        if (hd == 64) PO_ATT(float, 64);
        else if (hd == 128) PO_ATT(float, 128);
        else if (hd == 32) PO_ATT(float, 32);
    } else {
        if (hd == 64) PO_ATT(bf16_t, 64);
        else if (hd == 128) PO_ATT(bf16_t, 128);
        else if (hd == 32) PO_ATT(bf16_t, 32);
    }
#undef PO_ATT
}

// ------------------------------------------------------------------ last-row LM head
// logits[v] = sum_i x[i] W[v, i]; one wavefront per vocabulary row, 16-byte loads of W.
// rows: null = every vocabulary row; else the n_rows ids to compute (the acceptable output tokens, when nobody
// asked for the whole distribution): the same dot product per row, so those logits are the same bits either way
template <typename T>
__global__ void __launch_bounds__(256) lm_head_kernel(const T* __restrict__ x, const T* __restrict__ W,
                                                      float* __restrict__ logits, int V, int d,
                                                      const int32_t* __restrict__ rows, int n_rows) {
    constexpr int VEC = 16 / sizeof(T);
    const int lane = threadIdx.x & 63;
    const int idx = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (idx >= (rows ? n_rows : V)) return;
    const int row = rows ? rows[idx] : idx;
    const T* wr = W + (int64_t)row * d;
    float acc = 0.f;
    for (int i = lane * VEC; i < d; i += 64 * VEC) {
        const uint4 wv = *(const uint4*)(wr + i);
        const uint4 xv = *(const uint4*)(x + i);
        const T* wp = (const T*)&wv;
        const T* xp = (const T*)&xv;
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc = fmaf(to_f32(xp[c]), to_f32(wp[c]), acc);
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) logits[row] = acc;
}

void launch_lm_head(int dtype, const void* x, const void* W, float* logits, int V, int d, const int32_t* rows, int n_rows,
                    hipStream_t s) {
    const dim3 grid((unsigned)(((rows ? n_rows : V) + 3) / 4));
    if (dtype == 0)
        hipLaunchKernelGGL(lm_head_kernel<float>, grid, dim3(256), 0, s, (const float*)x, (const float*)W, logits,
                           V, d, rows, n_rows);
    else
        hipLaunchKernelGGL(lm_head_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)x, (const bf16_t*)W,
                           logits, V, d, rows, n_rows);
}

// ------------------------------------------------------------------ candidate log-probs
// lp_i = z[c_i] - logsumexp_j z[c_j]  (probabilities over the acceptable tokens sum to 1)
__global__ void __launch_bounds__(64) cand_logprob_kernel(const float* __restrict__ logits,
                                                          const int32_t* __restrict__ cand, int n,
                                                          float* __restrict__ lp) {
    float mx = -INFINITY;
    for (int i = threadIdx.x; i < n; i += 64) mx = fmaxf(mx, logits[cand[i]]);
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float sum = 0.f;
    for (int i = threadIdx.x; i < n; i += 64) sum += expf(logits[cand[i]] - mx);
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    const float lse = mx + logf(sum);
    for (int i = threadIdx.x; i < n; i += 64) lp[i] = logits[cand[i]] - lse;
}

void launch_cand_logprobs(const float* logits, const int32_t* cand, int n_cand, float* lp, hipStream_t s) {
    if (n_cand <= 0) return;
    hipLaunchKernelGGL(cand_logprob_kernel, dim3(1), dim3(64), 0, s, logits, cand, n_cand, lp);
}

// ------------------------------------------------------------------ gate/up packing
__global__ void __launch_bounds__(256) pack_gate_up_kernel(const uint4* __restrict__ wg, const uint4* __restrict__ wu,
                                                           uint4* __restrict__ dst, int F, int vec_per_row, int il) {
    const int r = blockIdx.x;            // 0 .. 2F-1, destination row
    const int blk = r / il, within = r % il;
    const int f = (blk >> 1) * il + within;
    const uint4* src = ((blk & 1) ? wu : wg) + (int64_t)f * vec_per_row;
    uint4* d = dst + (int64_t)r * vec_per_row;
    for (int i = threadIdx.x; i < vec_per_row; i += 256) d[i] = src[i];
}

void launch_pack_gate_up(int dtype, const void* wg, const void* wu, void* wgu, int F, int K, int il,
                         hipStream_t s) {
    const int esz = dtype == 0 ? 4 : 2;
    hipLaunchKernelGGL(pack_gate_up_kernel, dim3((unsigned)(2 * F)), dim3(256), 0, s, (const uint4*)wg,
                       (const uint4*)wu, (uint4*)wgu, F, K * esz / 16, il);
}

// ------------------------------------------------------------------ V transpose (bf16)
// Vt[c][t] = V[t][c] for t < n, 0 for n <= t < round_up(n, 64); 64x64 tiles through LDS.
__global__ void __launch_bounds__(256) v_transpose_kernel(const bf16_t* __restrict__ V, bf16_t* __restrict__ Vt,
                                                          int64_t n, int kv_dim, int64_t ldv) {
    __shared__ bf16_t tile[64][66];
    const int64_t t0 = (int64_t)blockIdx.x * 64;
    const int c0 = blockIdx.y * 64;
    for (int idx = threadIdx.x; idx < 64 * 64; idx += 256) {
        const int r = idx >> 6, c = idx & 63;          // r: token, c: channel
        const int64_t t = t0 + r;
        tile[r][c] = (t < n && c0 + c < kv_dim) ? V[t * kv_dim + c0 + c] : (bf16_t)0;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < 64 * 64; idx += 256) {
        const int c = idx >> 6, r = idx & 63;          // consecutive threads -> consecutive tokens
        if (c0 + c < kv_dim) Vt[(int64_t)(c0 + c) * ldv + t0 + r] = tile[r][c];
    }
}

void launch_v_transpose(const bf16_t* V, bf16_t* Vt, int64_t n, int kv_dim, int64_t ldv, hipStream_t s) {
    if (n <= 0) return;
    const dim3 grid((unsigned)((n + 63) / 64), (unsigned)((kv_dim + 63) / 64));
    hipLaunchKernelGGL(v_transpose_kernel, grid, dim3(256), 0, s, V, Vt, n, kv_dim, ldv);
}

// ------------------------------------------------------------------ rotary row packing (bf16)
// swap row blocks [32,64) and [64,96) of every 128-row head, in place
__global__ void __launch_bounds__(256) pack_rope_rows_kernel(bf16_t* W, int64_t row_elems) {
    const int head = blockIdx.y, r = blockIdx.x;       // r in [0, 32)
    bf16_t* a = W + ((int64_t)head * 128 + 32 + r) * row_elems;
    bf16_t* b = W + ((int64_t)head * 128 + 64 + r) * row_elems;
    for (int64_t i = threadIdx.x; i < row_elems; i += 256) {
        const bf16_t t = a[i];
        a[i] = b[i];
        b[i] = t;
    }
}

void launch_pack_rope_rows(bf16_t* W, int n_heads, int hd, int64_t row_elems, hipStream_t s) {
    if (hd != 128 || n_heads <= 0) return;
    hipLaunchKernelGGL(pack_rope_rows_kernel, dim3(32, (unsigned)n_heads), dim3(256), 0, s, W, row_elems);
}

__global__ void __launch_bounds__(64) vt_pad_zero_kernel(bf16_t* Vt, int64_t ldv, int64_t n, int pad) {
    if ((int)threadIdx.x < pad) Vt[(int64_t)blockIdx.x * ldv + n + threadIdx.x] = 0;
}

__global__ void __launch_bounds__(256) fill_zero32_kernel(uint32_t* dst, size_t n) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = 0u;
}

void launch_fill_zero32(void* dst, size_t n_words, hipStream_t s) {
    if (n_words == 0) return;
    hipLaunchKernelGGL(fill_zero32_kernel, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, s, (uint32_t*)dst, n_words);
}

// x[i] = float(bf16(x[i])), round to nearest even: what storing a float32 tensor as bf16 and reading it back does.
__global__ void __launch_bounds__(256) round_bf16_f32_kernel(float* x, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) x[i] = bf2f(f2bf(x[i]));
}

void launch_round_bf16_f32(float* x, int64_t n, hipStream_t s) {
    if (n <= 0) return;
    hipLaunchKernelGGL(round_bf16_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, x, n);
}

void launch_vt_pad_zero(bf16_t* Vt, int rows, int64_t ldv, int64_t n, hipStream_t s) {
    const int pad = (int)(round_up64(n, 64) - n);
    if (pad <= 0 || rows <= 0) return;
    hipLaunchKernelGGL(vt_pad_zero_kernel, dim3((unsigned)rows), dim3(64), 0, s, Vt, ldv, n, pad);
}

// Highest 32-bit word of an arena that differs from a fill pattern: per-thread strided scan,
// wavefront/workgroup maximum, one 64-bit atomic maximum per workgroup.  *out must start at 0 and
// receives (index of that word + 1), or stays 0 when nothing differs.
// K rows and V^T columns of a position range between the one-layer buffers and a prefix-cache entry, in one
// launch: workgroup row 0 copies the K rows (contiguous), workgroup row 1 + f copies row f of V^T (src and dst
// start at the same column, so they are misaligned alike).  16 bytes per thread where a 16-byte block lies
// wholly inside the range, single elements at its two ends.
__global__ void __launch_bounds__(256) kv_copy_kernel(unsigned char* dk, const unsigned char* sk, size_t k_bytes,
                                                      unsigned char* dv, size_t dpitch, const unsigned char* sv,
                                                      size_t spitch, size_t v_bytes, unsigned gk, unsigned gv) {
    unsigned char* d;
    const unsigned char* s;
    size_t n, first, stride;
    if (blockIdx.x < gk) {                      // workgroups [0, gk): the K rows, grid-stride
        d = dk; s = sk; n = k_bytes;
        first = (size_t)blockIdx.x * 256 + threadIdx.x;
        stride = (size_t)gk * 256;
    } else {                                    // then gv workgroups per V^T row
        const unsigned r = (blockIdx.x - gk) / gv, part = (blockIdx.x - gk) % gv;
        d = dv + (size_t)r * dpitch; s = sv + (size_t)r * spitch; n = v_bytes;
        first = (size_t)part * 256 + threadIdx.x;
        stride = (size_t)gv * 256;
    }
    // 16-byte blocks counted from the aligned address at or below the start (same misalignment on both sides)
    const size_t mis = (size_t)((uintptr_t)d & 15);
    const size_t nblk = n ? (mis + n + 15) >> 4 : 0;
    for (size_t b = first; b < nblk; b += stride) {
        const ptrdiff_t lo = (ptrdiff_t)(b << 4) - (ptrdiff_t)mis;            // byte offset of the block from d
        if (lo >= 0 && (size_t)lo + 16 <= n) {
            *(uint4*)(d + lo) = *(const uint4*)(s + lo);
        } else {
            for (int e = 0; e < 16; e += 2) {
                const ptrdiff_t o = lo + e;
                if (o >= 0 && (size_t)o + 2 <= n) *(uint16_t*)(d + o) = *(const uint16_t*)(s + o);
            }
        }
    }
}

void launch_kv_copy(void* dk, const void* sk, size_t k_bytes, void* dv, size_t dpitch, const void* sv, size_t spitch,
                    size_t v_bytes, int v_rows, hipStream_t s) {
    if (k_bytes == 0 && (v_bytes == 0 || v_rows <= 0)) return;
    size_t gk = (k_bytes / 16 + 255) / 256, gv = ((v_bytes + 30) / 16 + 255) / 256;
    if (gk > 2048) gk = 2048;
    if (gv > 8) gv = 8;
    if (gk == 0) gk = 1;
    if (gv == 0) gv = 1;
    hipLaunchKernelGGL(kv_copy_kernel, dim3((unsigned)(gk + gv * (size_t)v_rows)), dim3(256), 0, s, (unsigned char*)dk,
                       (const unsigned char*)sk, k_bytes, (unsigned char*)dv, dpitch, (const unsigned char*)sv, spitch,
                       v_bytes, (unsigned)gk, (unsigned)gv);
}

__global__ void __launch_bounds__(256) high_water_kernel(const uint32_t* ws, size_t n_words, uint32_t pattern,
                                                         unsigned long long* out) {
    __shared__ unsigned long long part[4];
    unsigned long long best = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_words; i += (size_t)gridDim.x * 256)
        if (ws[i] != pattern) best = i + 1;       // indices grow along the scan
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long o = __shfl_xor(best, off);
        best = o > best ? o : best;
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) best = part[w] > best ? part[w] : best;
        if (best) atomicMax(out, best);
    }
}

void launch_high_water(const void* ws, size_t bytes, uint32_t pattern, unsigned long long* out, hipStream_t s) {
    hipLaunchKernelGGL(high_water_kernel, dim3(2048), dim3(256), 0, s, (const uint32_t*)ws, bytes / 4, pattern, out);
}

}  // namespace po
