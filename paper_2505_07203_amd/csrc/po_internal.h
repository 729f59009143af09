// Internal declarations shared by the translation units of libpo (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>

namespace po {

typedef uint16_t bf16_t;   // bf16 bit pattern as stored in HBM

// ---- scalar conversions ---------------------------------------------------------------
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// fp32 -> bf16, round-to-nearest-even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ bf16_t f2bf(float f) {
    __bf16 h = (__bf16)f;
    return __builtin_bit_cast(bf16_t, h);
}
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return bf2f(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f2bf(v); }

static inline int64_t round_up64(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// ---- launchers: "basic" kernels, any dtype (dtype: 0 = fp32, 1 = bf16) ----------------
void launch_embed(int dtype, const int32_t* tok, const void* E, void* X, int64_t n, int d, hipStream_t s);
void launch_rmsnorm(int dtype, const void* x, const void* g, void* y, int64_t rows, int d, float eps,
                    hipStream_t s);
// cos/sin table [n, hd/2] each, angles formed in fp64
void launch_rope_table(float* cos_t, float* sin_t, int64_t n, int hd, float theta, hipStream_t s);
// in-place rotate-half RoPE on x[n, H, hd] (row stride ld elements)
void launch_rope(int dtype, void* x, int64_t ld, const float* cos_t, const float* sin_t, int64_t n,
                 int H, int hd, hipStream_t s);
// fp32-accumulating tiled GEMM  C[M,N] = A[M,K] W[N,K]^T (+bias[N]) (+R[M,N])
void launch_gemm_basic(int dtype, const void* A, int64_t lda, const void* W, int64_t ldw, void* C,
                       int64_t ldc, const void* bias, const void* R, int64_t ldr, int64_t M, int N,
                       int K, hipStream_t s);
// H[M,F] = silu(GU[:, :F]) * GU[:, F:]   (GU row stride 2F)
void launch_silu_mul(int dtype, const void* GU, void* H, int64_t M, int F, hipStream_t s);
// fp32-path attention (one thread per query row), o may alias q
// (q_row0: only the query-row blocks from the one that holds row q_row0 on are computed; 0 = all rows)
void launch_attention_basic(int dtype, const void* q, const void* k, const void* v, void* o, int64_t N,
                            int Hq, int Hkv, int hd, int64_t q_row0, hipStream_t s);
// logits[V] = x[d] . W[V,d]^T
// logits[r] = x . W[r] for every vocabulary row r, or (rows != null) only for r = rows[0 .. n_rows)
void launch_lm_head(int dtype, const void* x, const void* W, float* logits, int V, int d, const int32_t* rows, int n_rows,
                    hipStream_t s);
// lp[i] = logits[cand[i]] - logsumexp_j logits[cand[j]]
void launch_cand_logprobs(const float* logits, const int32_t* cand, int n_cand, float* lp, hipStream_t s);
// interleave gate/up rows in blocks of `il` rows: dst rows [2b*il, 2b*il+il) = Wg block b, next il = Wu block b
void launch_pack_gate_up(int dtype, const void* wg, const void* wu, void* wgu, int F, int K, int il,
                         hipStream_t s);

// ---- launchers: bf16 MFMA kernels ------------------------------------------------------
enum { EPI_STORE = 0, EPI_RESIDUAL = 1, EPI_SILU_MUL = 2, EPI_QKV_ROPE = 3, EPI_PARTIAL = 4 };
// C[M,N] = A[M,K] W[N,K]^T with bf16 MFMA, fp32 accumulation.
//   EPI_STORE    : C = acc (+ bias[N], bf16)
//   EPI_RESIDUAL : C = acc + R  (added in fp32; R may alias C)
//   EPI_SILU_MUL : W rows interleaved gate/up in blocks of 32; C[M, N/2] = silu(gate) * up
void launch_gemm_mfma(int epi, const bf16_t* A, int64_t lda, const bf16_t* W, int64_t ldw, bf16_t* C, int64_t ldc,
                      const bf16_t* bias, const bf16_t* R, int64_t ldr, int64_t M, int N, int K, hipStream_t s);
// Fused QKV projection: [Q|K|V] = A Wqkv^T (+bias), rotary embedding applied to Q and K in
// the fp32 epilogue, V written transposed.  Wqkv (and bias) rows must be in the packed order
// of launch_pack_rope_rows.  Q, K point at the first row of this call (row stride qd / kvd);
// Vt is the base of V^T [kvd][ldv] and the call writes columns pos0 .. pos0+M-1.  GEMM row r is
// rotated for sequence position row_pos[pos0 + r] (device array over buffer rows: several requests
// packed into one buffer), or pos0 + r when row_pos is null.
// q_scale: factor applied to the rotated Q values in fp32 before their one rounding to bf16 (1, or
// attention_q_scale(hd) when the attention that follows is launched with q_prescaled; K and V are never scaled).
void launch_gemm_qkv_rope(const bf16_t* A, int64_t lda, const bf16_t* Wqkv, int64_t ldw, const bf16_t* bias,
                          bf16_t* Q, bf16_t* K, bf16_t* Vt, int64_t ldv, const float* rope_cos,
                          const float* rope_sin, int64_t pos0, const int32_t* row_pos, int64_t M, int qd, int kvd,
                          int hd, int Kdim, float q_scale, hipStream_t s);
// the softmax scale in log2 units: p = exp2(q_scaled . k) = exp(q . k / sqrt(hd))
static inline float attention_q_scale(int hd) { return (float)(1.4426950408889634 / sqrt((double)hd)); }
// In place: within every head of `hd` rows (hd == 128 only; hd == 64 is already in order)
// swap row blocks [32,64) and [64,96), so that rotary partners i and i + hd/2 sit 32 rows
// apart inside one 64-row group.  row_elems = elements per row (1 for a bias vector).
void launch_pack_rope_rows(bf16_t* W, int n_heads, int hd, int64_t row_elems, hipStream_t s);
// zero columns [n, round_up(n,64)) of V^T [rows][ldv]
void launch_vt_pad_zero(bf16_t* Vt, int rows, int64_t ldv, int64_t n, hipStream_t s);
void launch_high_water(const void* ws, size_t bytes, uint32_t pattern, unsigned long long* out, hipStream_t s);
// Vt[Hkv*hd][ldv] = transpose of V[n, Hkv*hd]; columns n..round_up(n,64)-1 are zero-filled
// K rows (k_bytes contiguous bytes) and v_rows rows of V^T (v_bytes each, pitches in bytes) between the one-layer
// buffers and a prefix-cache entry; bf16 data, the V^T source and destination misaligned alike (same column)
void launch_kv_copy(void* dk, const void* sk, size_t k_bytes, void* dv, size_t dpitch, const void* sv, size_t spitch,
                    size_t v_bytes, int v_rows, hipStream_t s);
void launch_v_transpose(const bf16_t* V, bf16_t* Vt, int64_t n, int kv_dim, int64_t ldv, hipStream_t s);
// causal GQA flash attention; q [N,Hq,hd], k [N,Hkv,hd], vt [Hkv*hd][ldv]; o may alias q.
// redo: attention_mfma_redo_bytes(N, Hq) bytes of device memory, all zero on entry and left all zero (one word
// per 256-row query tile and head: the tiles whose scores leave the range of the fast kernel's fixed reference
// exponent are marked there and recomputed by the running-maximum kernel in a second launch)
size_t attention_mfma_redo_bytes(int64_t N, int Hq);
// q_prescaled: q holds the rotated queries times attention_q_scale(hd) (launch_gemm_qkv_rope's q_scale); the
// kernels then exponentiate K Q^T as it is.
void launch_attention_mfma(const bf16_t* q, const bf16_t* k, const bf16_t* vt, int64_t ldv, bf16_t* o,
                           int64_t N, int Hq, int Hkv, int hd, int64_t q_row0, int* redo, bool q_prescaled, hipStream_t s);
// n 32-bit words of zeros (a kernel, not a memset node, so that it can be captured into a graph)
void launch_fill_zero32(void* dst, size_t n_words, hipStream_t s);
void launch_round_bf16_f32(float* x, int64_t n, hipStream_t s);
// float32 GEMM on the float32 matrix instruction; false (nothing launched) when K, the leading dimensions or the
// pointers do not allow 16-byte loads
bool launch_gemm_f32_mfma(const float* A, int64_t lda, const float* W, int64_t ldw, float* C, int64_t ldc, const float* bias,
                          const float* R, int64_t ldr, int64_t M, int N, int K, hipStream_t s);
// float32 attention on the float32 matrix instruction; false (nothing launched) when hd is neither 64 nor 128
bool launch_attention_f32_mfma(const float* q, const float* k, const float* v, float* o, int64_t N, int Hq, int Hkv, int hd,
                               int64_t q_row0, hipStream_t s);
// The same for query rows [q_row0, N) when they are few and the keys many: the key tiles of a query tile are
// divided between workgroups (fp32 partial results in `scratch`, merged by a second kernel).  Sums are formed
// in a different order than in launch_attention_mfma: equal to rounding, not bit for bit.  Returns the
// number of key splits (0 or 1: not worth it or scratch too small, nothing launched); launch = false only asks.
// k2 / vt2 (pitch ldv2; may be null): a second K / V^T pair of the same layouts that holds the first n2 positions
// (n2 a multiple of 64) -- a prefix-cache entry read in place; positions from n2 on come from k / vt.
int launch_attention_mfma_split(const bf16_t* q, const bf16_t* k, const bf16_t* vt, int64_t ldv, bf16_t* o,
                                int64_t N, int Hq, int Hkv, int hd, int64_t q_row0, float* scratch,
                                size_t scratch_bytes, bool launch, const bf16_t* k2, const bf16_t* vt2, int64_t ldv2,
                                int64_t n2, bool q_prescaled, hipStream_t s);
bool gemm_mfma_supported(int N, int K);
// Time of one bf16 GEMM launch of M rows x N columns in units of (one 256 x 256 tile's K loop): rounds of tiles over
// the compute units with the tile height the launcher will pick.
double gemm_mfma_launch_cost(int64_t M, int N);
// C = A W^T + R for a GEMM with few rows, the reduction over K split between workgroups (a GEMM with few
// output tiles leaves most of the chip idle and every workgroup streaming a whole K range of both operands):
// split s of `splits` writes its fp32 partial tile sums to part[s][M][N], a second kernel adds them up in
// split order, adds R and rounds once.  The sum order differs from launch_gemm_mfma's (there one fp32
// accumulator runs over all of K), so the results agree to rounding, not bit for bit.  Returns the number
// of splits it would use for this shape and `part_bytes` of scratch memory; 0 or 1 = not worth it or does
// not fit (then nothing is launched).  With launch = false only that number is computed.
// launch_gemm_qkv_rope the same way (partials, then one kernel that sums them and applies bias, rotary
// embedding and the V^T store)
int launch_gemm_qkv_rope_splitk(const bf16_t* A, int64_t lda, const bf16_t* Wqkv, int64_t ldw, const bf16_t* bias,
                                bf16_t* Q, bf16_t* Kd, bf16_t* Vt, int64_t ldv, const float* rope_cos,
                                const float* rope_sin, int64_t pos0, const int32_t* row_pos, int64_t M, int qd,
                                int kvd, int hd, int K, float q_scale, float* part, size_t part_bytes, bool launch,
                                hipStream_t s);
// launch_gemm_mfma(EPI_SILU_MUL) the same way; part must not overlap H's rows [0, M)
int launch_gemm_mfma_splitk_silu(const bf16_t* A, int64_t lda, const bf16_t* W, int64_t ldw, bf16_t* H, int64_t ldh,
                                 int64_t M, int N, int K, float* part, size_t part_bytes, bool launch, hipStream_t s);
int launch_gemm_mfma_splitk_residual(const bf16_t* A, int64_t lda, const bf16_t* W, int64_t ldw, bf16_t* C,
                                     int64_t ldc, const bf16_t* R, int64_t ldr, int64_t M, int N, int K,
                                     float* part, size_t part_bytes, bool launch, hipStream_t s);

// ---- FP8-dynamic linear layers (OCP E4M3 codes + float32 scales) -----------------------------------
// rows of bf16 -> codes + one scale per row; source row r goes to destination row
// (r / blk) * dst_blk_stride + r % blk + dst_off (blk <= 0: rows stay in order); q may be x itself
bool quant_rows_supported(int K);
void launch_quant_rows(const bf16_t* x, int64_t ldx, unsigned char* q, int64_t ldq, float* scales, int64_t rows, int K,
                       int blk, int64_t dst_blk_stride, int64_t dst_off, hipStream_t s);
// C = (Qa Qw^T) * sa[row] * sw[col] with the epilogues of launch_gemm_mfma / launch_gemm_qkv_rope; codes one byte
// each, lda / ldw in bytes (K % 128 == 0)
bool gemm_fp8_supported(int N, int K);
void launch_gemm_fp8(int epi, const unsigned char* A, int64_t lda, const float* sa, const unsigned char* W, int64_t ldw,
                     const float* sw, bf16_t* C, int64_t ldc, const bf16_t* bias, const bf16_t* R, int64_t ldr, int64_t M,
                     int N, int K, hipStream_t s);
void launch_gemm_fp8_qkv_rope(const unsigned char* A, int64_t lda, const float* sa, const unsigned char* Wqkv, int64_t ldw,
                              const float* sw, const bf16_t* bias, bf16_t* Q, bf16_t* K, bf16_t* Vt, int64_t ldv,
                              const float* rope_cos, const float* rope_sin, int64_t pos0, const int32_t* row_pos,
                              int64_t M, int qd, int kvd, int hd, int Kdim, float q_scale, hipStream_t s);
// split-K forms of the two above for launches with few rows (see launch_gemm_mfma_splitk_residual): return the
// number of splits used, 0 = nothing launched (not worth it, or part_bytes of scratch too small)
int launch_gemm_fp8_splitk(int epi, const unsigned char* A, int64_t lda, const float* sa, const unsigned char* W,
                           int64_t ldw, const float* sw, bf16_t* C, int64_t ldc, const bf16_t* R, int64_t ldr, int64_t M,
                           int N, int K, float* part, size_t part_bytes, hipStream_t s);
int launch_gemm_fp8_qkv_rope_splitk(const unsigned char* A, int64_t lda, const float* sa, const unsigned char* Wqkv,
                                    int64_t ldw, const float* sw, const bf16_t* bias, bf16_t* Q, bf16_t* Kd, bf16_t* Vt,
                                    int64_t ldv, const float* rope_cos, const float* rope_sin, int64_t pos0,
                                    const int32_t* row_pos, int64_t M, int qd, int kvd, int hd, int K, float q_scale,
                                    float* part, size_t part_bytes, hipStream_t s);
// q, scales = quantise(bf16(rmsnorm(x; g)))   (d % 8 == 0, d <= 8192)
void launch_rmsnorm_quant(const bf16_t* x, const bf16_t* g, unsigned char* q, float* scales, int64_t rows, int d,
                          float eps, hipStream_t s);
bool attention_mfma_supported(int Hq, int Hkv, int hd);

// ---- micro-peaks (measurement only)
double launch_mfma_peak(int kind, int waves_per_simd, int iters, const void* operands, size_t operand_bytes, float* sink,
                        hipStream_t s);
void launch_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t s);

}  // namespace po
