// Shape-generic kernels: the whole float32 path and the fall-back for bfloat16 shapes the
// MFMA kernels do not serve.  Element type T is the storage type (float or bf16); all
// arithmetic is float32.  Written for correctness on any shape (ragged tails everywhere).
#include "common.h"
#include "launch.h"

namespace kvp {

// ---------------------------------------------------------------------------------------
// Rotary table: tab[pos * half + d] = (cos, sin)(pos * theta^(-2d/head_dim)), built once per
// handle in double precision so the float32 kernels see correctly rounded factors.
// ---------------------------------------------------------------------------------------
__global__ void rope_table_kernel(float2* tab, int max_pos, int half, double theta) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= max_pos * half) return;
  int pos = idx / half, d = idx % half;
  double inv_freq = pow(theta, -(double)d / (double)half);   // theta^(-2d/hd), hd = 2*half
  double ang = (double)pos * inv_freq;
  tab[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

void launch_rope_table(float2* tab, int max_pos, int half, double theta, hipStream_t s) {
  int n = max_pos * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, tab, max_pos, half, theta);
}

// ---------------------------------------------------------------------------------------
// Embedding gather fused with the first RMSNorm:  x[n,:] = E[tok[n],:],  h = rmsnorm(x) * g.
// One wavefront per token.  Token ids are clamped into [0, vocab); a clamped id sets bit 0 of
// *flags (KVP_FLAG_TOKEN_CLAMPED), which kvp_check_flags reports.
// `tok_stride`/`tok_offset` pick token n as tokens[n * tok_stride + tok_offset] (the base step
// gathers the last token of each sequence: stride T, offset T-1).
// ---------------------------------------------------------------------------------------
template <typename T, typename HT>
__global__ void embed_rmsnorm_kernel(const int32_t* __restrict__ tokens, int tok_stride, int tok_offset,
                                     const T* __restrict__ E, int vocab, const T* __restrict__ gain,
                                     float* __restrict__ x, HT* __restrict__ h, int n_tokens, int d, float eps,
                                     uint32_t* __restrict__ flags) {
  int wave = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  int lane = threadIdx.x % kWave;
  if (wave >= n_tokens) return;
  int tok = tokens[(size_t)wave * tok_stride + tok_offset];
  if ((tok < 0 || tok >= vocab) && lane == 0) atomicOr(flags, 1u);
  tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
  const T* e = E + (size_t)tok * d;
  float* xr = x + (size_t)wave * d;
  float ss = 0.f;
  for (int i = lane; i < d; i += kWave) {
    float v = to_f32(e[i]);
    xr[i] = v;
    ss += v * v;
  }
  ss = wave_sum(ss);
  if (h == nullptr) return;
  float r = rsqrtf(ss / (float)d + eps);
  HT* hr = h + (size_t)wave * d;
  for (int i = lane; i < d; i += kWave) from_f32(hr[i], to_f32(e[i]) * r * to_f32(gain[i]));
}

// RMSNorm of the float32 residual stream: h = x * rsqrt(mean(x^2) + eps) * g.  One wave per row.
template <typename T, typename HT>
__global__ void rmsnorm_kernel(const float* __restrict__ x, const T* __restrict__ gain, HT* __restrict__ h,
                               int rows, int d, float eps) {
  int wave = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  int lane = threadIdx.x % kWave;
  if (wave >= rows) return;
  const float* xr = x + (size_t)wave * d;
  float ss = 0.f;
  for (int i = lane; i < d; i += kWave) { float v = xr[i]; ss += v * v; }
  ss = wave_sum(ss);
  float r = rsqrtf(ss / (float)d + eps);
  HT* hr = h + (size_t)wave * d;
  for (int i = lane; i < d; i += kWave) from_f32(hr[i], xr[i] * r * to_f32(gain[i]));
}

// In-place rotary embedding on a [rows, n_heads*hd] matrix; row n is position n % T.
template <typename T>
__global__ void rope_kernel(T* __restrict__ x, int ld, int rows, int n_heads, int hd, int T_len,
                            const float2* __restrict__ tab) {
  int half = hd / 2;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)rows * n_heads * half;
  if (idx >= total) return;
  int d = idx % half;
  int hh = (idx / half) % n_heads;
  size_t n = idx / ((size_t)half * n_heads);
  int pos = (int)(n % T_len);
  float2 cs = tab[(size_t)pos * half + d];
  T* p = x + n * ld + (size_t)hh * hd + d;
  float a = to_f32(p[0]), b = to_f32(p[half]);
  from_f32(p[0], a * cs.x - b * cs.y);
  from_f32(p[half], b * cs.x + a * cs.y);
}

// Query / key normalisation (optional OpenELM trait, the key norm of Sec. 7 "Analysis"): in place,
// x[row, head, :] <- x / sqrt(mean(x^2) + eps) * gain over the hd dims of every head, followed,
// with ROPE, by the rotary embedding at position row % T_len (the norm comes first).  One wave
// per (row, head); a lane owns the rotary pairs (p, p + hd/2), p = lane, lane + 64, ...
template <typename T, typename G, bool ROPE>
__global__ __launch_bounds__(256) void head_norm_kernel(T* __restrict__ x, const G* __restrict__ gain, size_t n_items,
                                                        int n_heads, int hd, float eps, int T_len,
                                                        const float2* __restrict__ tab) {
  const size_t item = (size_t)blockIdx.x * 4 + threadIdx.x / kWave;     // (row, head)
  if (item >= n_items) return;
  const int lane = threadIdx.x % kWave, half = hd / 2;
  T* p = x + item * hd;                         // rows are n_heads * hd wide: item * hd addresses (row, head)
  float ss = 0.f;
  for (int d = lane; d < half; d += kWave) {
    const float a = to_f32(p[d]), b = to_f32(p[d + half]);
    ss += a * a + b * b;
  }
  ss = wave_sum(ss);
  const float sc = rsqrtf(ss / (float)hd + eps);
  const int pos = ROPE ? (int)((item / n_heads) % T_len) : 0;
  for (int d = lane; d < half; d += kWave) {
    float a = to_f32(p[d]) * sc * to_f32(gain[d]), b = to_f32(p[d + half]) * sc * to_f32(gain[d + half]);
    if (ROPE) {
      const float2 cs = tab[(size_t)pos * half + d];
      const float ra = a * cs.x - b * cs.y, rb = b * cs.x + a * cs.y;
      a = ra; b = rb;
    }
    from_f32(p[d], a);
    from_f32(p[d + half], b);
  }
}

// act[n, j] = silu(gu[n, j]) * gu[n, f + j]
template <typename T>
__global__ void silu_mul_kernel(const T* __restrict__ gu, T* __restrict__ act, size_t rows, int f) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows * f) return;
  size_t n = idx / f; int j = idx % f;
  float g = to_f32(gu[n * 2 * f + j]), u = to_f32(gu[n * 2 * f + f + j]);
  from_f32(act[idx], g / (1.f + __expf(-g)) * u);
}

// ---------------------------------------------------------------------------------------
// C = A[M,K] * W[N,K]^T, 64x64 tile per 256-thread block, 4x4 outputs per thread, float32 FMA.
// The epilogue functor decides where an output element goes.
// ---------------------------------------------------------------------------------------
template <typename T>
struct EpiStore {
  T* C; int ldc;
  __device__ void operator()(int m, int n, float v) const { from_f32(C[(size_t)m * ldc + n], v); }
};
struct EpiResidual {   // X[m,n] += v  (float32 residual stream, each element owned by one thread)
  float* X; int ld;
  __device__ void operator()(int m, int n, float v) const { X[(size_t)m * ld + n] += v; }
};
template <typename T>
struct EpiCache {      // row m = b*T + t, column n = head*hd + dim  ->  cache[b][head][t][dim]
  T* cache; int T_len; int64_t T_cap; int n_heads, hd;
  __device__ void operator()(int m, int n, float v) const {
    int b = m / T_len, t = m % T_len, hh = n / hd, dd = n % hd;
    from_f32(cache[(((size_t)b * n_heads + hh) * T_cap + t) * hd + dd], v);
  }
};

template <typename T, typename Epi>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T* __restrict__ A, int lda,
                                                           const T* __restrict__ W, int ldw,
                                                           int M, int N, int K, Epi epi) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Ws[BK][BN + 4];
  int tid = threadIdx.x;
  int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  int lr = tid / 4, lk = (tid % 4) * 4;      // each thread stages 4 consecutive k of one row
  int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int k = k0 + lk + i;
      int am = m0 + lr, wn = n0 + lr;
      As[lk + i][lr] = (am < M && k < K) ? to_f32(A[(size_t)am * lda + k]) : 0.f;
      Ws[lk + i][lr] = (wn < N && k < K) ? to_f32(W[(size_t)wn * ldw + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][tm + i]; w[i] = Ws[k][tn + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * w[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int m = m0 + tm + i, n = n0 + tn + j;
      if (m < M && n < N) epi(m, n, acc[i][j]);
    }
}

template <typename T, typename Epi>
static void launch_gemm_generic(const T* A, int lda, const T* W, int ldw, int M, int N, int K, Epi epi, hipStream_t s) {
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  hipLaunchKernelGGL((gemm_generic_kernel<T, Epi>), grid, dim3(256), 0, s, A, lda, W, ldw, M, N, K, epi);
}

// ---------------------------------------------------------------------------------------
// Causal grouped-query attention, one wavefront per (query row, query head).
// q: [B*T, n_q*hd]; k, v: [B*T, n_kv*hd] (token-major); out: [B*T, n_q*hd].
// Keys are visited in blocks of 64 (one per lane) with an online softmax; the weighted sum
// over a block has lanes own output dims (hd <= 256).
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_prefill_generic_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                                   const T* __restrict__ v, T* __restrict__ out,
                                                                   int T_len, int n_q, int n_kv, int hd, float scale) {
  __shared__ float p_sh[4][kWave];
  __shared__ float q_sh[4][256];
  int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  int t = blockIdx.x * 4 + w;
  int hq = blockIdx.y, b = blockIdx.z;
  bool active = t < T_len;
  int hk = hq / (n_q / n_kv);
  size_t row = (size_t)b * T_len + (active ? t : 0);
  int ldq = n_q * hd, ldk = n_kv * hd;
  for (int d = lane; d < hd; d += kWave) q_sh[w][d] = to_f32(q[row * ldq + (size_t)hq * hd + d]) * scale;
  __syncthreads();
  float m_run = -INFINITY, l_run = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};            // dims lane, lane+64, lane+128, lane+192
  int n_keys = active ? t + 1 : 0;
  // all four waves of the block run the same number of block iterations (barriers inside)
  int max_keys = min(T_len, blockIdx.x * 4 + 4);
  for (int u0 = 0; u0 < max_keys; u0 += kWave) {
    int u = u0 + lane;
    float s = -INFINITY;
    if (u < n_keys) {
      const T* kr = k + ((size_t)b * T_len + u) * ldk + (size_t)hk * hd;
      float dsum = 0.f;
      for (int d = 0; d < hd; ++d) dsum += q_sh[w][d] * to_f32(kr[d]);
      s = dsum;
    }
    float m_blk = wave_max(s);
    float m_new = fmaxf(m_run, m_blk);
    float p = (u < n_keys) ? __expf(s - m_new) : 0.f;
    float corr = (m_new == -INFINITY) ? 1.f : __expf(m_run - m_new);
    l_run = l_run * corr + wave_sum(p);
    m_run = m_new;
    p_sh[w][lane] = p;
    __syncthreads();
    int cnt = min(kWave, n_keys - u0);
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] *= corr;
    for (int uu = 0; uu < cnt; ++uu) {
      float pu = p_sh[w][uu];
      const T* vr = v + ((size_t)b * T_len + u0 + uu) * ldk + (size_t)hk * hd;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int d = lane + j * kWave;
        if (d < hd) acc[j] += pu * to_f32(vr[d]);
      }
    }
    __syncthreads();
  }
  if (active) {
    float inv = 1.f / l_run;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int d = lane + j * kWave;
      if (d < hd) from_f32(out[row * ldq + (size_t)hq * hd + d], acc[j] * inv);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Helpers of the ordinary-inference reference runs (one model alone, Sec. 6.3 "Timing Experiments")
// ---------------------------------------------------------------------------------------
// y[b, :] = x[b * T + T - 1, :]: the residual stream of the last prompt position of every sequence
__global__ __launch_bounds__(256) void gather_last_rows_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                               int T_len, int d) {
  const float* src = x + ((size_t)blockIdx.x * T_len + T_len - 1) * d;
  for (int i = threadIdx.x; i < d; i += 256) y[(size_t)blockIdx.x * d + i] = src[i];
}
// Token-major keys or values [B*T][n_kv*hd] -> cache layout [B][n_kv][T_cap][hd], 16 bytes per thread
template <typename T>
__global__ __launch_bounds__(256) void rows_to_cache_kernel(const T* __restrict__ src, T* __restrict__ dst, int T_len,
                                                            int64_t T_cap, int n_kv, int hd, size_t n_chunks) {
  constexpr int E = 16 / (int)sizeof(T);
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= n_chunks) return;
  const int per_head = hd / E;
  const size_t row = c / ((size_t)n_kv * per_head);          // token index b * T + t
  const int rem = (int)(c % ((size_t)n_kv * per_head));
  const int head = rem / per_head, piece = rem % per_head;
  const size_t b = row / T_len, t = row % T_len;
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = *reinterpret_cast<const u32x4*>(src + (row * n_kv + head) * hd + piece * E);
  *reinterpret_cast<u32x4*>(dst + ((b * n_kv + head) * (size_t)T_cap + t) * hd + piece * E) = v;
}
void launch_gather_last_rows(const float* x, float* y, int B, int T_len, int d, hipStream_t s) {
  hipLaunchKernelGGL(gather_last_rows_kernel, dim3(B), dim3(256), 0, s, x, y, T_len, d);
}
template <typename T>
void launch_rows_to_cache(const T* src, T* dst, int B, int T_len, int64_t T_cap, int n_kv, int hd, hipStream_t s) {
  const size_t n_chunks = (size_t)B * T_len * n_kv * hd * sizeof(T) / 16;
  hipLaunchKernelGGL((rows_to_cache_kernel<T>), dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, s, src, dst, T_len,
                     T_cap, n_kv, hd, n_chunks);
}
template void launch_rows_to_cache<float>(const float*, float*, int, int, int64_t, int, int, hipStream_t);
template void launch_rows_to_cache<bf16>(const bf16*, bf16*, int, int, int64_t, int, int, hipStream_t);

// ---------------------------------------------------------------------------------------
// Host-side launchers (declared in launch.h)
// ---------------------------------------------------------------------------------------
template <typename T, typename HT>
void launch_embed_rmsnorm(const int32_t* tokens, int tok_stride, int tok_offset, const T* E, int vocab,
                          const T* gain, float* x, HT* h, int n_tokens, int d, float eps, uint32_t* flags, hipStream_t s) {
  int blocks = (n_tokens + 3) / 4;
  hipLaunchKernelGGL((embed_rmsnorm_kernel<T, HT>), dim3(blocks), dim3(256), 0, s, tokens, tok_stride, tok_offset,
                     E, vocab, gain, x, h, n_tokens, d, eps, flags);
}
__device__ __forceinline__ void load4(const float* p, float (&o)[4]) {
  f32x4 v = *reinterpret_cast<const f32x4*>(p);
  o[0] = v[0]; o[1] = v[1]; o[2] = v[2]; o[3] = v[3];
}
__device__ __forceinline__ void load4(const bf16* p, float (&o)[4]) {
  bf16x4 v = *reinterpret_cast<const bf16x4*>(p);
  o[0] = (float)v[0]; o[1] = (float)v[1]; o[2] = (float)v[2]; o[3] = (float)v[3];
}
__device__ __forceinline__ void store4(float* p, const float (&o)[4]) {
  *reinterpret_cast<f32x4*>(p) = f32x4{o[0], o[1], o[2], o[3]};
}
__device__ __forceinline__ void store4(bf16* p, const float (&o)[4]) {
  *reinterpret_cast<bf16x4*>(p) = bf16x4{(bf16)o[0], (bf16)o[1], (bf16)o[2], (bf16)o[3]};
}

// RMSNorm for rows of up to 8192 elements with d % 256 == 0: one wave per row, the row is read once
// with 16-byte loads and kept in registers between the sum of squares and the scaled write.
template <typename T, typename HT, int CH>   // CH = d / 256 float4 chunks per lane
__global__ __launch_bounds__(256) void rmsnorm_rows_kernel(const float* __restrict__ x, const T* __restrict__ gain,
                                                           HT* __restrict__ h, int rows, int d, float eps) {
  const int row = blockIdx.x * 4 + threadIdx.x / kWave, lane = threadIdx.x % kWave;
  if (row >= rows) return;
  const float* xr = x + (size_t)row * d;
  f32x4 v[CH];
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    v[c] = *reinterpret_cast<const f32x4*>(xr + (c * kWave + lane) * 4);
    ss += v[c][0] * v[c][0] + v[c][1] * v[c][1] + v[c][2] * v[c][2] + v[c][3] * v[c][3];
  }
  ss = wave_sum(ss);
  const float r = rsqrtf(ss / (float)d + eps);
  HT* hr = h + (size_t)row * d;
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    const int k = (c * kWave + lane) * 4;
    float gn[4], o[4];
    load4(gain + k, gn);
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = v[c][e] * r * gn[e];
    store4(hr + k, o);
  }
}

template <typename T, typename HT>
void launch_rmsnorm(const float* x, const T* gain, HT* h, int rows, int d, float eps, hipStream_t s) {
  dim3 grid((rows + 3) / 4), block(256);
  if (d % 256 == 0 && d <= 8192) {
    switch (d / 256) {
#define KVP_RN(C) case C: hipLaunchKernelGGL((rmsnorm_rows_kernel<T, HT, C>), grid, block, 0, s, x, gain, h, rows, d, eps); return;
      KVP_RN(1) KVP_RN(2) KVP_RN(3) KVP_RN(4) KVP_RN(5) KVP_RN(6) KVP_RN(7) KVP_RN(8) KVP_RN(12) KVP_RN(16) KVP_RN(20)
      KVP_RN(24) KVP_RN(28) KVP_RN(32)
#undef KVP_RN
      default: break;
    }
  }
  hipLaunchKernelGGL((rmsnorm_kernel<T, HT>), grid, block, 0, s, x, gain, h, rows, d, eps);
}
template <typename T>
void launch_rope(T* x, int ld, int rows, int n_heads, int hd, int T_len, const float2* tab, hipStream_t s) {
  size_t total = (size_t)rows * n_heads * (hd / 2);
  hipLaunchKernelGGL((rope_kernel<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, x, ld, rows, n_heads, hd, T_len, tab);
}
template <typename T, typename G>
void launch_head_norm(T* x, const G* gain, size_t rows, int n_heads, int hd, float eps, bool rope, int T_len,
                      const float2* tab, hipStream_t s) {
  const size_t items = rows * n_heads;
  dim3 grid((unsigned)((items + 3) / 4)), block(256);
  if (rope) hipLaunchKernelGGL((head_norm_kernel<T, G, true>), grid, block, 0, s, x, gain, items, n_heads, hd, eps, T_len, tab);
  else hipLaunchKernelGGL((head_norm_kernel<T, G, false>), grid, block, 0, s, x, gain, items, n_heads, hd, eps, 1, tab);
}
template void launch_head_norm<float, float>(float*, const float*, size_t, int, int, float, bool, int, const float2*, hipStream_t);
template void launch_head_norm<float, bf16>(float*, const bf16*, size_t, int, int, float, bool, int, const float2*, hipStream_t);
template void launch_head_norm<bf16, bf16>(bf16*, const bf16*, size_t, int, int, float, bool, int, const float2*, hipStream_t);

template <typename T>
void launch_silu_mul(const T* gu, T* act, size_t rows, int f, hipStream_t s) {
  size_t total = rows * f;
  hipLaunchKernelGGL((silu_mul_kernel<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, gu, act, rows, f);
}
template <typename T>
void launch_gemm_store(const T* A, int lda, const T* W, int ldw, T* C, int ldc, int M, int N, int K, hipStream_t s) {
  launch_gemm_generic<T>(A, lda, W, ldw, M, N, K, EpiStore<T>{C, ldc}, s);
}
template <typename T>
void launch_gemm_residual(const T* A, int lda, const T* W, int ldw, float* X, int ldx, int M, int N, int K, hipStream_t s) {
  launch_gemm_generic<T>(A, lda, W, ldw, M, N, K, EpiResidual{X, ldx}, s);
}
template <typename T>
void launch_gemm_cache(const T* A, int lda, const T* W, int ldw, T* cache, int T_len, int64_t T_cap, int n_heads,
                       int hd, int M, int N, int K, hipStream_t s) {
  launch_gemm_generic<T>(A, lda, W, ldw, M, N, K, EpiCache<T>{cache, T_len, T_cap, n_heads, hd}, s);
}
template <typename T>
void launch_attn_prefill_generic(const T* q, const T* k, const T* v, T* out, int B, int T_len, int n_q, int n_kv,
                                 int hd, hipStream_t s) {
  dim3 grid((T_len + 3) / 4, n_q, B);
  hipLaunchKernelGGL((attn_prefill_generic_kernel<T>), grid, dim3(256), 0, s, q, k, v, out, T_len, n_q, n_kv, hd,
                     1.0f / sqrtf((float)hd));
}

#define KVP_INST(T)                                                                                                   \
  template void launch_embed_rmsnorm<T, T>(const int32_t*, int, int, const T*, int, const T*, float*, T*, int, int,  \
                                           float, uint32_t*, hipStream_t);                                           \
  template void launch_rmsnorm<T, T>(const float*, const T*, T*, int, int, float, hipStream_t);                      \
  template void launch_rope<T>(T*, int, int, int, int, int, const float2*, hipStream_t);                             \
  template void launch_silu_mul<T>(const T*, T*, size_t, int, hipStream_t);                                          \
  template void launch_gemm_store<T>(const T*, int, const T*, int, T*, int, int, int, int, hipStream_t);             \
  template void launch_gemm_residual<T>(const T*, int, const T*, int, float*, int, int, int, int, hipStream_t);      \
  template void launch_gemm_cache<T>(const T*, int, const T*, int, T*, int, int64_t, int, int, int, int, int,        \
                                     hipStream_t);                                                                   \
  template void launch_attn_prefill_generic<T>(const T*, const T*, const T*, T*, int, int, int, int, int, hipStream_t);
KVP_INST(float)
KVP_INST(bf16)
template void launch_embed_rmsnorm<bf16, float>(const int32_t*, int, int, const bf16*, int, const bf16*, float*, float*,
                                                int, int, float, uint32_t*, hipStream_t);
template void launch_rmsnorm<bf16, float>(const float*, const bf16*, float*, int, int, float, hipStream_t);

}  // namespace kvp
