// Host-side launchers of the libkvp kernels.  Every function only enqueues work on `s`.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "common.h"

namespace kvp {

// ---- kernels_generic.hip -------------------------------------------------------------------
void launch_rope_table(float2* tab, int max_pos, int half, double theta, hipStream_t s);
template <typename T, typename HT>
void launch_embed_rmsnorm(const int32_t* tokens, int tok_stride, int tok_offset, const T* E, int vocab,
                          const T* gain, float* x, HT* h, int n_tokens, int d, float eps, uint32_t* flags, hipStream_t s);
template <typename T, typename HT>
void launch_rmsnorm(const float* x, const T* gain, HT* h, int rows, int d, float eps, hipStream_t s);
template <typename T>
void launch_rope(T* x, int ld, int rows, int n_heads, int hd, int T_len, const float2* tab, hipStream_t s);
// In place on a dense [rows, n_heads * hd] matrix: per-head RMSNorm with gain [hd], then (rope) the rotary
// embedding at position row % T_len.
template <typename T, typename G>
void launch_head_norm(T* x, const G* gain, size_t rows, int n_heads, int hd, float eps, bool rope, int T_len,
                      const float2* tab, hipStream_t s);
template <typename T>
void launch_silu_mul(const T* gu, T* act, size_t rows, int f, hipStream_t s);
template <typename T>
void launch_gemm_store(const T* A, int lda, const T* W, int ldw, T* C, int ldc, int M, int N, int K, hipStream_t s);
template <typename T>
void launch_gemm_residual(const T* A, int lda, const T* W, int ldw, float* X, int ldx, int M, int N, int K, hipStream_t s);
template <typename T>
void launch_gemm_cache(const T* A, int lda, const T* W, int ldw, T* cache, int T_len, int64_t T_cap, int n_heads,
                       int hd, int M, int N, int K, hipStream_t s);
template <typename T>
void launch_attn_prefill_generic(const T* q, const T* k, const T* v, T* out, int B, int T_len, int n_q, int n_kv,
                                 int hd, hipStream_t s);

void launch_gather_last_rows(const float* x, float* y, int B, int T_len, int d, hipStream_t s);
// token-major [B*T][n_kv*hd] -> cache layout [B][n_kv][T_cap][hd]
template <typename T>
void launch_rows_to_cache(const T* src, T* dst, int B, int T_len, int64_t T_cap, int n_kv, int hd, hipStream_t s);

// ---- kernels_decode.hip --------------------------------------------------------------------
// Split partials of the single-query attention kernels: one row per (split, sequence, query head) of
// width + kPartPad floats -- `width` un-normalised sums, the running maximum, the normaliser, two unused
// (the padding keeps every row 16-byte aligned, so a consumer reads the sums with 16-byte loads).
constexpr int kPartPad = 4;
// mode 0: out = W x   1: out += W x   2: out = silu(W x) * (W2 x);  norm: x = rmsnorm(x; gain)
template <typename T>
void launch_gemv(int mode, bool norm, const T* W, const T* W2, const float* x, const T* gain, float* out, int B, int N,
                 int K, float eps, hipStream_t s);
int decode_attn_splits(int B, int n_kv, int T_len);
bool decode_attn_supported(int hd, int group);
// result goes to out (float32) or, if out_hi != NULL, to out_hi / out_lo as bf16 high / low halves;
// with neither, only the split partials are written (the consumer merges them)
template <typename T>
bool launch_decode_attn(const float* q, const T* kc, const T* vc, float* part, float* out, bf16* out_hi, bf16* out_lo,
                        int B, int T_len, int64_t T_cap, int n_q, int n_kv, int hd, int n_splits, const float2* rope_tab,
                        hipStream_t s);

// merge of split partials [n_splits][B][n_q][hd + kPartPad] -> out float [B][n_q][hd]
void launch_decode_combine(const float* part, float* out, int n_splits, int B, int n_q, int hd, hipStream_t s);

// ---- base step with the predictor absorbed into the attention (kernels_absorbed.hip) ----
// q~ = W_K^g^T rope(q) / sqrt(hd): q float [B][n_q][hd] -> out float [B][n_q][Ka]; wk [n_kv*hd][Ka]
template <typename T>
bool launch_absorb_q(const float* q, const T* wk, float* out, int B, int n_q, int n_kv, int hd, int Ka, int pos,
                     const float2* rope_tab, hipStream_t s);
// o = W_V^g r: r float [B][n_q][Ka] -> out float [B][n_q*hd] and / or bf16 high / low halves
template <typename T>
bool launch_absorb_o(const float* r, const T* wv, float* out, bf16* out_hi, bf16* out_lo, int B, int n_q, int n_kv, int hd,
                     int Ka, hipStream_t s);
// attention of all query heads over one auxiliary layer, token-major ka, va [B*T][Ka]; any element
// type, plain ALU (kernels_decode.hip).  part: [n_splits][B][n_q][Ka + kPartPad]; out float [B][n_q][Ka]
bool absorbed_attn_supported(int Ka);
template <typename T>
bool launch_absorbed_attn(const float* q, const T* ka, const T* va, float* part, float* out, int B, int T_len, int n_q,
                          int Ka, int n_splits, hipStream_t s);
// the same on the matrix cores: bf16, Ka 256 or 512, values transposed vT [B][Ka][T_pad]
bool absorbed_mfma_supported(int Ka);
int absorbed_mfma_splits(int B, int n_q, int T_len);
bool launch_absorbed_attn_mfma(const float* q, const bf16* ka, const bf16* vT, float* part, float* out, int B, int T_len,
                               int T_pad, int n_q, int Ka, hipStream_t s);

// k (rotated to position pos) and v of one new token per sequence -> slot pos of a cache layer
template <typename T>
void launch_kv_append(const float* k, const float* v, T* kc, T* vc, int B, int pos, int64_t T_cap, int n_kv, int hd,
                      const float2* rope_tab, hipStream_t s);

// ---- kernels_base_chain.hip (bf16 base step; activations travel as bf16 high / low halves) ----
int chain_ssq_parts(int N, int B);   // partial sums of squares a residual projection with N outputs emits per right-hand side
void launch_base_embed(const int32_t* tokens, int T_len, const bf16* E, int vocab, const bf16* gain, float* y, bf16* uh,
                       bf16* ul, float* ssq, int B, int d, uint32_t* flags, hipStream_t s);
// out = [rsqrt(mean + eps) *] W x         (ssq_in == NULL: no norm scale)
void launch_chain_project(const bf16* W, const bf16* xh, const bf16* xl, const float* ssq_in, int n_part_in, float eps,
                          float* out, int B, int N, int K, hipStream_t s);
// y += W x;  (yh, yl) = split(y * gain_next);  ssq_out = partial sums of y^2
void launch_chain_residual(const bf16* W, const bf16* xh, const bf16* xl, float* y, const bf16* gain_next, bf16* yh,
                           bf16* yl, float* ssq_out, int B, int N, int K, hipStream_t s);
// Same, but x = the merge of decode-attention split partials [n_splits][B][n_q][hd + kPartPad] (what
// launch_decode_attn leaves when it is given no destination), K = n_q * hd.  One or two
// right-hand sides only; returns false (nothing launched) for shapes it does not serve.
bool launch_chain_residual_merge(const bf16* W, const float* part, int n_splits, int n_q, int hd, float* y,
                                 const bf16* gain_next, bf16* yh, bf16* yl, float* ssq_out, int B, int N, int K,
                                 hipStream_t s);
// (ah, al) = split(silu(s Wg x) * (s Wu x)),  s = rsqrt(mean + eps)
void launch_chain_swiglu(const bf16* Wg, const bf16* Wu, const bf16* xh, const bf16* xl, const float* ssq_in,
                         int n_part_in, float eps, bf16* ah, bf16* al, int B, int N, int K, hipStream_t s);
void launch_argmax(const float* logits, int32_t* out, int B, int V, hipStream_t s);

}  // namespace kvp
