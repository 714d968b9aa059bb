// Base-model single-token step (Sec. 4.1 "Inference": b <- B(I[-1], KV^_B)): attention of one
// query per head over the predicted cache, split merge, argmax, and the plain-ALU GEMVs of the
// float32 path (the bf16 path's matrix-core GEMVs live in kernels_base_chain.hip).
// All of it is HBM-bound: every weight and every cache entry is read exactly once, with
// 16-byte loads and enough independent loads in flight per lane to cover memory latency.
#include <cstdlib>

#include "common.h"
#include "launch.h"

namespace kvp {

// ---------------------------------------------------------------------------------------
// GEMV for NB right-hand sides:  out[b, n] (op)= sum_k W[n, k] * x[b, k],  W row-major [N, K].
//   MODE 0: out = dot            MODE 1: out += dot (residual stream, in place)
//   MODE 2: out[b, n] = silu(Wg[n,:].x[b]) * (Wu[n,:].x[b])   (SwiGLU gate/up in one pass)
//   NORM: x is rmsnorm(xin; gain) computed on the fly (each block recomputes the row scales,
//         the input is tiny and L2-resident).
// A block stages x in LDS (chunks of KC floats per right-hand side); each wave owns R
// consecutive rows; each lane covers 8 consecutive k per 512-wide step.
// ---------------------------------------------------------------------------------------
constexpr int GEMV_LDS_FLOATS = 8192;

template <typename T, int NB, int R, int MODE, bool NORM>
__global__ __launch_bounds__(256) void gemv_kernel(const T* __restrict__ W, const T* __restrict__ W2,
                                                   const float* __restrict__ xin, const T* __restrict__ gain,
                                                   float* __restrict__ out, int N, int K, float eps) {
  constexpr int KC = (GEMV_LDS_FLOATS / NB) / 512 * 512;
  constexpr int NW = (MODE == 2) ? 2 : 1;
  __shared__ __attribute__((aligned(16))) float xs[NB][KC];
  __shared__ float red[4][NB];
  int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  int row0 = (blockIdx.x * 4 + wave) * R;

  float scale[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) scale[b] = 1.f;
  if (NORM) {
    float ss[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) ss[b] = 0.f;
    for (int k = threadIdx.x * 4; k < K; k += 256 * 4) {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        f32x4 v = *reinterpret_cast<const f32x4*>(xin + (size_t)b * K + k);
        ss[b] += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
      }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      float s = wave_sum(ss[b]);
      if (lane == 0) red[wave][b] = s;
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < NB; ++b) scale[b] = rsqrtf((red[0][b] + red[1][b] + red[2][b] + red[3][b]) / (float)K + eps);
  }

  float acc[NW][R][NB];
#pragma unroll
  for (int w = 0; w < NW; ++w)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int b = 0; b < NB; ++b) acc[w][r][b] = 0.f;

  for (int kc = 0; kc < K; kc += KC) {
    int klen = min(KC, K - kc);
    if (kc > 0) __syncthreads();
    for (int k = threadIdx.x * 4; k < klen; k += 256 * 4) {
      f32x4 g = {1.f, 1.f, 1.f, 1.f};
      if (NORM) {
#pragma unroll
        for (int i = 0; i < 4; ++i) g[i] = to_f32(gain[kc + k + i]);
      }
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        f32x4 v = *reinterpret_cast<const f32x4*>(xin + (size_t)b * K + kc + k);
        if (NORM) v = v * g * scale[b];
        *reinterpret_cast<f32x4*>(&xs[b][k]) = v;
      }
    }
    __syncthreads();
    for (int k = lane * 8; k < klen; k += 512) {
      float wv[NW][R][8];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        int row = min(row0 + r, N - 1);
        load8(W + (size_t)row * K + kc + k, wv[0][r]);
        if (MODE == 2) load8(W2 + (size_t)row * K + kc + k, wv[NW - 1][r]);
      }
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        f32x4 x0 = *reinterpret_cast<const f32x4*>(&xs[b][k]);
        f32x4 x1 = *reinterpret_cast<const f32x4*>(&xs[b][k + 4]);
#pragma unroll
        for (int w = 0; w < NW; ++w)
#pragma unroll
          for (int r = 0; r < R; ++r) {
            float a = acc[w][r][b];
#pragma unroll
            for (int i = 0; i < 4; ++i) a += wv[w][r][i] * x0[i];
#pragma unroll
            for (int i = 0; i < 4; ++i) a += wv[w][r][4 + i] * x1[i];
            acc[w][r][b] = a;
          }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      float d0 = wave_sum(acc[0][r][b]);
      float d1 = (MODE == 2) ? wave_sum(acc[NW - 1][r][b]) : 0.f;
      int row = row0 + r;
      if (lane == 0 && row < N) {
        float* o = out + (size_t)b * N + row;
        if (MODE == 0) *o = d0;
        else if (MODE == 1) *o += d0;
        else *o = d0 / (1.f + __expf(-d0)) * d1;
      }
    }
}

template <typename T, int NB, int MODE, bool NORM>
static void launch_gemv_r(const T* W, const T* W2, const float* x, const T* gain, float* out, int N, int K, float eps,
                          hipStream_t s) {
  // rows per wave: fewer rows -> more waves in flight for small matrices; more rows amortise
  // the LDS reads of x when several right-hand sides share a weight row.
  int R = (N >= 16384 || (NB >= 4 && N >= 4096)) ? 4 : ((N >= 8192 || NB >= 4) ? 2 : 1);
  if (MODE == 2 && R == 4) R = 2;
  auto grid = [&](int r) { return dim3((N + 4 * r - 1) / (4 * r)); };
  if (R == 4) hipLaunchKernelGGL((gemv_kernel<T, NB, 4, MODE, NORM>), grid(4), dim3(256), 0, s, W, W2, x, gain, out, N, K, eps);
  else if (R == 2) hipLaunchKernelGGL((gemv_kernel<T, NB, 2, MODE, NORM>), grid(2), dim3(256), 0, s, W, W2, x, gain, out, N, K, eps);
  else hipLaunchKernelGGL((gemv_kernel<T, NB, 1, MODE, NORM>), grid(1), dim3(256), 0, s, W, W2, x, gain, out, N, K, eps);
}

template <typename T, int MODE, bool NORM>
static void launch_gemv_b(const T* W, const T* W2, const float* x, const T* gain, float* out, int B, int N, int K,
                          float eps, hipStream_t s) {
  // Right-hand sides are processed in groups of at most 8 (weights are re-read per group).
  for (int b0 = 0; b0 < B; b0 += 8) {
    int nb = min(8, B - b0);
    const float* xb = x + (size_t)b0 * K;
    float* ob = out + (size_t)b0 * N;
    switch (nb) {
      case 1: launch_gemv_r<T, 1, MODE, NORM>(W, W2, xb, gain, ob, N, K, eps, s); break;
      case 2: launch_gemv_r<T, 2, MODE, NORM>(W, W2, xb, gain, ob, N, K, eps, s); break;
      case 3: launch_gemv_r<T, 3, MODE, NORM>(W, W2, xb, gain, ob, N, K, eps, s); break;
      case 4: launch_gemv_r<T, 4, MODE, NORM>(W, W2, xb, gain, ob, N, K, eps, s); break;
      case 5: launch_gemv_r<T, 5, MODE, NORM>(W, W2, xb, gain, ob, N, K, eps, s); break;
      case 6: launch_gemv_r<T, 6, MODE, NORM>(W, W2, xb, gain, ob, N, K, eps, s); break;
      case 7: launch_gemv_r<T, 7, MODE, NORM>(W, W2, xb, gain, ob, N, K, eps, s); break;
      default: launch_gemv_r<T, 8, MODE, NORM>(W, W2, xb, gain, ob, N, K, eps, s); break;
    }
  }
}

template <typename T>
void launch_gemv(int mode, bool norm, const T* W, const T* W2, const float* x, const T* gain, float* out, int B, int N,
                 int K, float eps, hipStream_t s) {
  if (mode == 0 && norm) launch_gemv_b<T, 0, true>(W, W2, x, gain, out, B, N, K, eps, s);
  else if (mode == 0) launch_gemv_b<T, 0, false>(W, W2, x, gain, out, B, N, K, eps, s);
  else if (mode == 1) launch_gemv_b<T, 1, false>(W, W2, x, gain, out, B, N, K, eps, s);
  else launch_gemv_b<T, 2, true>(W, W2, x, gain, out, B, N, K, eps, s);
}
template void launch_gemv<bf16>(int, bool, const bf16*, const bf16*, const float*, const bf16*, float*, int, int, int, float, hipStream_t);
template void launch_gemv<float>(int, bool, const float*, const float*, const float*, const float*, float*, int, int, int, float, hipStream_t);

// ---------------------------------------------------------------------------------------
// Decode attention, split over the cache length.  Grid (n_splits, n_kv, B); a block owns keys
// [split*chunk, min(T, (split+1)*chunk)) of one (sequence, kv head) and serves all G = n_q/n_kv
// query heads of that kv head, so each cache row is read once.
//   q      float [B, n_q*hd]  raw query projection; rotary (position T-1) and 1/sqrt(hd) are
//          applied here while staging q in LDS.
//   cache  T [B][n_kv][T_cap][hd] for this layer (keys post-rotary as predicted).
//   part   float [n_splits][B][n_q][hd + kPartPad]: un-normalised sum, running max, running denominator.
// A row of hd elements is covered by LPR = hd/8 lanes (16-byte loads); a wave reads 64/LPR rows
// per load instruction, U such instructions per tensor form one batch, and the next batch's
// loads are issued before the current batch is consumed.  Every lane group keeps its own
// online-softmax state; groups are merged by a lane butterfly, waves through LDS.
// ---------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_rot_add(float v) {   // v + (v rotated within its row of 16 lanes)
  int x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
  return v + __int_as_float(x);
}
template <int LPR>
__device__ __forceinline__ float group_sum(float d) {     // sum over the LPR lanes covering one cache row
  if (LPR == 16) {
    d = dpp_rot_add<0x128>(d);   // row_ror:8
    d = dpp_rot_add<0x124>(d);   // row_ror:4
    d = dpp_rot_add<0x122>(d);   // row_ror:2
    d = dpp_rot_add<0x121>(d);   // row_ror:1
    return d;
  }
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) d += __shfl_xor(d, o, 64);
  return d;
}

template <typename T> struct Raw8;
template <> struct Raw8<bf16> { typedef bf16x8 type; };
template <> struct Raw8<float> { struct type { f32x4 a, b; }; };
__device__ __forceinline__ bf16x8 load_raw8(const bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ Raw8<float>::type load_raw8(const float* p) {
  Raw8<float>::type r; r.a = *reinterpret_cast<const f32x4*>(p); r.b = *reinterpret_cast<const f32x4*>(p + 4); return r;
}
__device__ __forceinline__ void unpack8(const bf16x8& v, float (&o)[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (float)v[i];
}
__device__ __forceinline__ void unpack8(const Raw8<float>::type& v, float (&o)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) { o[i] = v.a[i]; o[4 + i] = v.b[i]; }
}

template <typename T, int HD, int G, bool SHARED = false>
__global__ __launch_bounds__(256) void decode_attn_split_kernel(const float* __restrict__ q, const T* __restrict__ kc,
                                                                const T* __restrict__ vc, float* __restrict__ part,
                                                                int T_len, int64_t T_cap, int n_kv, int chunk,
                                                                const float2* __restrict__ rope_tab, float sm_scale) {
  constexpr int LPR = HD / 8;           // lanes per cache row
  constexpr int RPW = kWave / LPR;      // rows per wave per load
  constexpr int NGRP = 4 * RPW;         // lane groups per block
  constexpr int U = 4;                  // load instructions per tensor and batch
  typedef typename Raw8<T>::type raw8;
  __shared__ float q_sh[G][HD];
  __shared__ float st_m[4][G], st_l[4][G];
  __shared__ float st_o[4][G][HD + 1];

  const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int B = gridDim.z, n_q = n_kv * G;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int grp = wave * RPW + lane / LPR;    // lane group id in the block
  const int sub = lane % LPR;                 // which 8 dims of the row
  const int c0 = split * chunk, c1 = min(T_len, c0 + chunk);
  // SHARED: every query head reads the one row set of its sequence (rows of width HD, T_cap per
  // sequence); grid row hk then only names which G query heads the block serves
  const size_t rows0 = SHARED ? (size_t)b : (size_t)b * n_kv + hk;
  const T* kbase = kc + rows0 * T_cap * HD + sub * 8;
  const T* vbase = vc + rows0 * T_cap * HD + sub * 8;

  raw8 kr[2][U], vr[2][U];
  auto issue = [&](int buf, int r0) {
#pragma unroll
    for (int j = 0; j < U; ++j) {
      int r = min(r0 + j * NGRP, max(c1 - 1, c0));   // clamped rows are masked when consumed
      r = min(r, T_len - 1);
      kr[buf][j] = load_raw8(kbase + (size_t)r * HD);
      vr[buf][j] = load_raw8(vbase + (size_t)r * HD);
    }
  };
  const int r_first = c0 + grp;
  issue(0, r_first);                    // the cache stream starts before q is staged

  // stage q with rotary at position T-1 (no table: q comes rotated) and the softmax scale
  for (int i = threadIdx.x; i < G * (HD / 2); i += 256) {
    int g = i / (HD / 2), d = i % (HD / 2);
    const float* qr = q + ((size_t)b * n_q + (size_t)hk * G + g) * HD;
    float2 cs = rope_tab ? rope_tab[(size_t)(T_len - 1) * (HD / 2) + d] : float2{1.f, 0.f};
    float a = qr[d], bb = qr[d + HD / 2];
    q_sh[g][d] = (a * cs.x - bb * cs.y) * sm_scale;
    q_sh[g][d + HD / 2] = (bb * cs.x + a * cs.y) * sm_scale;
  }
  __syncthreads();
  float qv[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int i = 0; i < 8; ++i) qv[g][i] = q_sh[g][sub * 8 + i];

  float m_run[G], l_run[G], acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m_run[g] = -INFINITY; l_run[g] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[g][i] = 0.f;
  }

  auto consume = [&](int buf, int r0) {
    float s[G][U];
    float vf[U][8];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      float kf[8];
      unpack8(kr[buf][j], kf);
      unpack8(vr[buf][j], vf[j]);
      const bool valid = r0 + j * NGRP < c1;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) d += qv[g][i] * kf[i];
        d = group_sum<LPR>(d);
        s[g][j] = valid ? d : -INFINITY;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mb = s[g][0];
#pragma unroll
      for (int j = 1; j < U; ++j) mb = fmaxf(mb, s[g][j]);
      float m_new = fmaxf(m_run[g], mb);             // finite: row r0 itself is valid
      float corr = __expf(m_run[g] - m_new);
      float lsum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[g][i] *= corr;
#pragma unroll
      for (int j = 0; j < U; ++j) {
        float p = __expf(s[g][j] - m_new);
        lsum += p;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[g][i] += p * vf[j][i];
      }
      l_run[g] = l_run[g] * corr + lsum;
      m_run[g] = m_new;
    }
  };

  // two-deep software pipeline over batches of U*NGRP rows (unrolled by two for static buffers)
  for (int r0 = r_first; r0 < c1; r0 += 2 * NGRP * U) {
    const int r1 = r0 + NGRP * U;
    if (r1 < c1) issue(1, r1);
    consume(0, r0);
    if (r1 >= c1) break;
    if (r1 + NGRP * U < c1) issue(0, r1 + NGRP * U);
    consume(1, r1);
  }

  // merge the lane groups of a wave with a butterfly over lane bits >= log2(LPR)
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mo = __shfl_xor(m_run[g], off, 64);
      float lo = __shfl_xor(l_run[g], off, 64);
      float m_new = fmaxf(m_run[g], mo);
      float w1 = (m_run[g] == -INFINITY) ? 0.f : __expf(m_run[g] - m_new);
      float w2 = (mo == -INFINITY) ? 0.f : __expf(mo - m_new);
      l_run[g] = l_run[g] * w1 + lo * w2;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float ao = __shfl_xor(acc[g][i], off, 64);
        acc[g][i] = acc[g][i] * w1 + ao * w2;
      }
      m_run[g] = m_new;
    }
  }
  // then the four waves through LDS
  if (lane < LPR) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      if (sub == 0) { st_m[wave][g] = m_run[g]; st_l[wave][g] = l_run[g]; }
#pragma unroll
      for (int i = 0; i < 8; ++i) st_o[wave][g][sub * 8 + i] = acc[g][i];
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < G * HD; i += 256) {
    int g = i / HD, d = i % HD;
    float m = -INFINITY;
    for (int p = 0; p < 4; ++p) m = fmaxf(m, st_m[p][g]);
    float l = 0.f, o = 0.f;
    for (int p = 0; p < 4; ++p) {
      float w = (st_m[p][g] == -INFINITY) ? 0.f : __expf(st_m[p][g] - m);
      l += st_l[p][g] * w;
      o += st_o[p][g][d] * w;
    }
    float* pr = part + (((size_t)split * B + b) * n_q + (size_t)hk * G + g) * (HD + kPartPad);
    pr[d] = o;
    if (d == 0) { pr[HD] = m; pr[HD + 1] = l; }
  }
}

// Merge the splits: out[b, hq, :] = sum_s o_s e^{m_s - m} / sum_s l_s e^{m_s - m}, summed in split
// order.  Grid (n_q, B), one thread per output dim; the loads of a batch of 8 splits are all
// issued before use.  (A separate launch on purpose: merging inside the split kernel needs a
// device-scope fence per block, which on this multi-die part costs far more than a launch.)
__global__ void decode_attn_combine_kernel(const float* __restrict__ part, float* __restrict__ out,
                                           bf16* __restrict__ out_hi, bf16* __restrict__ out_lo, int n_splits, int B,
                                           int n_q, int hd) {
  const int hq = blockIdx.x, b = blockIdx.y;
  const size_t stride = (size_t)B * n_q * (hd + kPartPad);
  const float* p0 = part + ((size_t)b * n_q + hq) * (hd + kPartPad);
  for (int d = threadIdx.x; d < hd; d += blockDim.x) {
    float m = -INFINITY, l = 0.f, o = 0.f;
    for (int s0 = 0; s0 < n_splits; s0 += 8) {
      float mv[8], lv[8], ov[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool ok = s0 + u < n_splits;
        const float* pr = p0 + (size_t)(ok ? s0 + u : 0) * stride;
        mv[u] = ok ? pr[hd] : -INFINITY;
        lv[u] = pr[hd + 1];
        ov[u] = pr[d];
      }
      float mb = m;
#pragma unroll
      for (int u = 0; u < 8; ++u) mb = fmaxf(mb, mv[u]);
      float corr = (m == -INFINITY) ? 0.f : __expf(m - mb);
      l *= corr; o *= corr;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        float w = (mv[u] == -INFINITY) ? 0.f : __expf(mv[u] - mb);
        l += lv[u] * w;
        o += ov[u] * w;
      }
      m = mb;
    }
    const size_t idx = ((size_t)b * n_q + hq) * hd + d;
    const float res = o / l;
    if (out_hi) {            // consumer is a matrix-core GEMV: hand over bf16 high / low halves
      bf16 hv = (bf16)res;
      out_hi[idx] = hv;
      out_lo[idx] = (bf16)(res - (float)hv);
    } else {
      out[idx] = res;
    }
  }
}

void launch_decode_combine(const float* part, float* out, int n_splits, int B, int n_q, int hd, hipStream_t s) {
  hipLaunchKernelGGL(decode_attn_combine_kernel, dim3(n_q, B), dim3(hd < 64 ? 64 : hd), 0, s, part, out, (bf16*)nullptr,
                     (bf16*)nullptr, n_splits, B, n_q, hd);
}

// ---------------------------------------------------------------------------------------
// Decode attention for bf16 caches with head_dim 128: scores on the matrix cores.
// Same grid, inputs and partial format as decode_attn_split_kernel.  The plain-ALU kernel
// above spends ~100 vector instructions per (K row, V row) pair and is ALU-bound well below
// HBM speed; here q.K^T runs as v_mfma_f32_16x16x32_bf16 with the key rows loaded straight
// from global memory in the MFMA "A" layout (lane (r = lane%16, g = lane/16) holds
// K[key r][32 s + 8 g .. + 7]) and q (bf16 high + low halves, G heads padded to 16 columns) as
// "B", which leaves only the P.V accumulation (V rows in 16-byte pieces, 16 lanes per row) and
// a few softmax operations per 16 keys on the vector ALUs.  Probabilities and rescale factors
// travel from the score lanes to the V lanes through a per-wave LDS tile.
// A wave consumes 32 keys per iteration; the K loads of iteration i+1 are issued as soon as
// the MFMAs of iteration i have consumed the registers, the V loads likewise after P.V.
// ---------------------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(256) void decode_attn_mfma_kernel(const float* __restrict__ q, const bf16* __restrict__ kc,
                                                               const bf16* __restrict__ vc, float* __restrict__ part,
                                                               int T_len, int64_t T_cap, int n_kv, int chunk,
                                                               const float2* __restrict__ rope_tab, float sm_scale) {
  constexpr int HD = 128;
  constexpr int KPI = 32;                         // keys per wave iteration (two MFMA row tiles)
  __shared__ float q_sh[G][HD];
  __shared__ __attribute__((aligned(16))) float p_sh[4][KPI][4 * ((G + 3) / 4)];   // [wave][key][head]
  __shared__ __attribute__((aligned(16))) float corr_sh[4][4 * ((G + 3) / 4)];
  __shared__ float st_m[4][G], st_l[4][G];
  __shared__ float st_o[4][G][HD + 1];
  constexpr int GP = 4 * ((G + 3) / 4);           // heads padded to a multiple of 4 for 16-byte LDS reads

  const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int B = gridDim.z, n_q = n_kv * G;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int r = lane % 16, g = lane / 16;         // score layout: r = key row (A) / head column (B, C)
  const int sub = lane % 16, rgrp = lane / 16;    // value layout: 8 dims sub*8.., key (4 j + rgrp) of a tile
  const int c0 = split * chunk, c1 = min(T_len, c0 + chunk);
  const bf16* kbase = kc + ((size_t)b * n_kv + hk) * T_cap * HD;
  const bf16* vbase = vc + ((size_t)b * n_kv + hk) * T_cap * HD;
  const int last_row = T_len - 1;

  bf16x8 kreg[2][4], vreg[8];
  auto issue_k = [&](int k0) {                    // rows k0 + 16 t + r, dims 32 s + 8 g
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const bf16* row = kbase + (size_t)min(k0 + 16 * t + r, last_row) * HD + g * 8;
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) kreg[t][s4] = load_stream8(row + 32 * s4);
    }
  };
  auto issue_v = [&](int k0) {                    // rows k0 + 4 j + rgrp, dims 8 sub
#pragma unroll
    for (int j = 0; j < 8; ++j)
      vreg[j] = load_stream8(vbase + (size_t)min(k0 + 4 * j + rgrp, last_row) * HD + sub * 8);
  };
  const int k_first = c0 + wave * KPI;
  if (k_first < c1) { issue_k(k_first); issue_v(k_first); }

  // stage q with rotary at position T-1 and the softmax scale (in the exp2 domain)
  const float qs = sm_scale * 1.4426950408889634f;
  for (int i = threadIdx.x; i < G * (HD / 2); i += 256) {
    int hh = i / (HD / 2), d = i % (HD / 2);
    const float* qr = q + ((size_t)b * n_q + (size_t)hk * G + hh) * HD;
    float2 cs = rope_tab[(size_t)(T_len - 1) * (HD / 2) + d];
    float a = qr[d], bb = qr[d + HD / 2];
    q_sh[hh][d] = (a * cs.x - bb * cs.y) * qs;
    q_sh[hh][d + HD / 2] = (bb * cs.x + a * cs.y) * qs;
  }
  __syncthreads();
  // B operand: lane (head r, g) holds q[r][32 s + 8 g .. + 7] as bf16 high / low halves; heads >= G are zero
  bf16x8 qh[4], ql[4];
#pragma unroll
  for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = (r < G) ? q_sh[r < G ? r : 0][32 * s4 + 8 * g + e] : 0.f;
      bf16 hv = (bf16)v;
      qh[s4][e] = hv;
      ql[s4][e] = (bf16)(v - (float)hv);
    }

  float m_run = -INFINITY, l_run = 0.f;           // per score lane: head r, partial over its keys
  float acc[G][8];
#pragma unroll
  for (int hh = 0; hh < G; ++hh)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[hh][i] = 0.f;

  for (int k0 = k_first; k0 < c1; k0 += 4 * KPI) {
    // ---- scores: S^T[key][head] for 32 keys ----
    f32x4 sc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      sc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[t][s4], qh[s4], sc[t], 0, 0, 0);
        sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[t][s4], ql[s4], sc[t], 0, 0, 0);
      }
    }
    const int k_next = k0 + 4 * KPI;
    if (k_next < c1) issue_k(k_next);
    // accumulator: lane (head r, g) holds keys k0 + 16 t + 4 g + i
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (k0 + 16 * t + 4 * g + i >= c1) sc[t][i] = -INFINITY;
        mx = fmaxf(mx, sc[t][i]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);          // finite: key k0 is valid
    const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
    float psum = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float p = __builtin_amdgcn_exp2f(sc[t][i] - m_new);
        psum += p;
        if (r < GP) p_sh[wave][16 * t + 4 * g + i][r] = (r < G) ? p : 0.f;
      }
    l_run = l_run * corr + psum;
    m_run = m_new;
    if (g == 0 && r < GP) corr_sh[wave][r] = (r < G) ? corr : 1.f;
    // The probabilities pass from the score lanes to the value lanes of the SAME wave through LDS
    // without a block barrier (LDS operations of one wave execute in program order); the
    // wavefront-scope fences emit no instruction, they only keep the compiler from moving a
    // lane's reads across the other lanes' writes.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    // ---- O += P V on the vector ALUs ----
    float cf[GP];
#pragma unroll
    for (int c4 = 0; c4 < GP / 4; ++c4) {
      f32x4 cv = *reinterpret_cast<const f32x4*>(&corr_sh[wave][4 * c4]);
#pragma unroll
      for (int e = 0; e < 4; ++e) cf[4 * c4 + e] = cv[e];
    }
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[hh][i] *= cf[hh];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float pv[GP];
#pragma unroll
      for (int c4 = 0; c4 < GP / 4; ++c4) {
        f32x4 t4 = *reinterpret_cast<const f32x4*>(&p_sh[wave][4 * j + rgrp][4 * c4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) pv[4 * c4 + e] = t4[e];
      }
      float vf[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) vf[i] = (float)vreg[j][i];
#pragma unroll
      for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[hh][i] += pv[hh] * vf[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the next iteration overwrites what was just read
    if (k_next < c1) issue_v(k_next);
  }

  // ---- merge inside the wave: the running max is wave-uniform per head, so partial sums just add ----
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
#pragma unroll
  for (int hh = 0; hh < G; ++hh)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float v = acc[hh][i];
      v += __shfl_xor(v, 16, 64);
      v += __shfl_xor(v, 32, 64);
      acc[hh][i] = v;
    }
  if (g == 0 && r < G) { st_m[wave][r] = m_run; st_l[wave][r] = l_run; }
  if (rgrp == 0) {
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
      for (int i = 0; i < 8; ++i) st_o[wave][hh][sub * 8 + i] = acc[hh][i];
  }
  __syncthreads();
  // ---- then the four waves; partials are stored with natural-log statistics ----
  for (int i = threadIdx.x; i < G * HD; i += 256) {
    int hh = i / HD, d = i % HD;
    float m = -INFINITY;
    for (int p = 0; p < 4; ++p) m = fmaxf(m, st_m[p][hh]);
    float l = 0.f, o = 0.f;
    for (int p = 0; p < 4; ++p) {
      float w = (st_m[p][hh] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st_m[p][hh] - m);
      l += st_l[p][hh] * w;
      o += st_o[p][hh][d] * w;
    }
    float* pr = part + (((size_t)split * B + b) * n_q + (size_t)hk * G + hh) * (HD + kPartPad);
    pr[d] = o;
    if (d == 0) { pr[HD] = m * 0.6931471805599453f; pr[HD + 1] = l; }   // the merge kernel works with e^x
  }
}

template <int HD>
static bool launch_decode_mfma(int G, dim3 grid, hipStream_t s, const float* q, const bf16* kc, const bf16* vc,
                               float* part, int T_len, int64_t T_cap, int n_kv, int chunk, const float2* tab, float scale) {
  if (HD != 128) return false;
#define KVP_DM(GG)                                                                                                 \
  case GG:                                                                                                         \
    hipLaunchKernelGGL((decode_attn_mfma_kernel<GG>), grid, dim3(256), 0, s, q, kc, vc, part, T_len, T_cap, n_kv,  \
                       chunk, tab, scale);                                                                         \
    return true;
  switch (G) {
    KVP_DM(1) KVP_DM(2) KVP_DM(3) KVP_DM(4) KVP_DM(6) KVP_DM(8)
    default: return false;
  }
#undef KVP_DM
}

template <typename T, int HD>
static bool launch_decode_hd(int G, dim3 grid, hipStream_t s, const float* q, const T* kc, const T* vc, float* part,
                             int T_len, int64_t T_cap, int n_kv, int chunk, const float2* tab, float scale) {
#define KVP_DA(GG)                                                                                                  \
  case GG:                                                                                                          \
    hipLaunchKernelGGL((decode_attn_split_kernel<T, HD, GG>), grid, dim3(256), 0, s, q, kc, vc, part, T_len, T_cap, \
                       n_kv, chunk, tab, scale);                                                                    \
    return true;
  switch (G) {
    KVP_DA(1) KVP_DA(2) KVP_DA(3) KVP_DA(4) KVP_DA(6) KVP_DA(8)
    default: return false;
  }
#undef KVP_DA
}

int decode_attn_splits(int B, int n_kv, int T_len) {
  // about two blocks per CU (measured best on the four benchmark shapes), at least 64 keys per block
  const int pairs = B * n_kv;
  int want = (512 + pairs - 1) / pairs;
  int max_by_len = (T_len + 63) / 64;
  int n = want < max_by_len ? want : max_by_len;
  // ... and blocks of 256 keys rather than shorter ones (a wave then runs two iterations and more, not one),
  // as long as that still leaves a block for every CU
  const int long_chunks = (T_len + 255) / 256, one_per_cu = (256 + pairs - 1) / pairs;
  if (n > long_chunks) {
    const int floor_n = n < one_per_cu ? n : one_per_cu;
    n = long_chunks > floor_n ? long_chunks : floor_n;
  }
  // one or two sequences: the output projection merges the partials in its prologue (one launch
  // fewer per layer on a latency-bound chain); keep that merge to one batch of eight
  if (B <= 2 && n > 8) n = 8;
  return n < 1 ? 1 : n;
}

bool decode_attn_supported(int hd, int G) {
  return (hd == 16 || hd == 32 || hd == 64 || hd == 128) && (G == 1 || G == 2 || G == 3 || G == 4 || G == 6 || G == 8);
}

template <typename T>
bool launch_decode_attn(const float* q, const T* kc, const T* vc, float* part, float* out, bf16* out_hi, bf16* out_lo,
                        int B, int T_len, int64_t T_cap, int n_q, int n_kv, int hd, int n_splits, const float2* rope_tab,
                        hipStream_t s) {
  int G = n_q / n_kv;
  int chunk = (T_len + n_splits - 1) / n_splits;
  dim3 grid(n_splits, n_kv, B);
  float scale = 1.0f / sqrtf((float)hd);
  bool ok = false;
  const char* alu = getenv("KVP_DECODE_ALU");     // "1": plain-ALU kernel even where the MFMA one applies (tests)
  if (sizeof(T) == 2 && hd == 128 && !(alu && alu[0] == '1'))
    ok = launch_decode_mfma<128>(G, grid, s, q, (const bf16*)kc, (const bf16*)vc, part, T_len, T_cap, n_kv, chunk,
                                 rope_tab, scale);
  if (!ok) switch (hd) {
    case 16: ok = launch_decode_hd<T, 16>(G, grid, s, q, kc, vc, part, T_len, T_cap, n_kv, chunk, rope_tab, scale); break;
    case 32: ok = launch_decode_hd<T, 32>(G, grid, s, q, kc, vc, part, T_len, T_cap, n_kv, chunk, rope_tab, scale); break;
    case 64: ok = launch_decode_hd<T, 64>(G, grid, s, q, kc, vc, part, T_len, T_cap, n_kv, chunk, rope_tab, scale); break;
    case 128: ok = launch_decode_hd<T, 128>(G, grid, s, q, kc, vc, part, T_len, T_cap, n_kv, chunk, rope_tab, scale); break;
    default: break;
  }
  if (!ok) return false;
  // no destination: the consumer merges the split partials itself (launch_chain_residual_merge)
  if (out || out_hi)
    hipLaunchKernelGGL(decode_attn_combine_kernel, dim3(n_q, B), dim3(hd < 64 ? 64 : hd), 0, s, part, out, out_hi, out_lo, n_splits, B, n_q, hd);
  return true;
}
template bool launch_decode_attn<float>(const float*, const float*, const float*, float*, float*, bf16*, bf16*, int, int, int64_t, int, int, int, int, const float2*, hipStream_t);
template bool launch_decode_attn<bf16>(const float*, const bf16*, const bf16*, float*, float*, bf16*, bf16*, int, int, int64_t, int, int, int, int, const float2*, hipStream_t);

// ---------------------------------------------------------------------------------------
// Attention of every query head over ONE shared set of rows per sequence: the base step with
// the predictor absorbed (Sec. 4.2 "Predictor Networks": the maps are linear, so
// q . (W_K k_A) = (W_K^T q) . k_A and sum_u p_u W_V v_A,u = W_V sum_u p_u v_A,u).  q: float
// [B][n_q][Ka], already rotated, mapped through W_K^T and scaled; ka, va: one auxiliary layer,
// token-major [B*T][Ka].  Plain-ALU kernel for any element type; out: float [B][n_q][Ka], the
// probability-weighted auxiliary values (still to be mapped through W_V).
// ---------------------------------------------------------------------------------------
template <typename T, int KA>
static bool launch_shared_ka(int G, dim3 grid, hipStream_t s, const float* q, const T* ka, const T* va, float* part,
                             int T_len, int chunk) {
#define KVP_DS(GG)                                                                                                     \
  case GG:                                                                                                             \
    hipLaunchKernelGGL((decode_attn_split_kernel<T, KA, GG, true>), grid, dim3(256), 0, s, q, ka, va, part, T_len,     \
                       (int64_t)T_len, (int)grid.y, chunk, (const float2*)nullptr, 1.0f);                              \
    return true;
  switch (G) {
    KVP_DS(1) KVP_DS(2) KVP_DS(4)
    default: return false;
  }
#undef KVP_DS
}
bool absorbed_attn_supported(int Ka) { return Ka == 16 || Ka == 32 || Ka == 64 || Ka == 128 || Ka == 256 || Ka == 512; }

template <typename T>
bool launch_absorbed_attn(const float* q, const T* ka, const T* va, float* part, float* out, int B, int T_len, int n_q,
                          int Ka, int n_splits, hipStream_t s) {
  const int G = (n_q % 4 == 0) ? 4 : (n_q % 2 == 0) ? 2 : 1;      // query heads per block
  const int chunk = (T_len + n_splits - 1) / n_splits;
  dim3 grid(n_splits, n_q / G, B);
  bool ok = false;
  switch (Ka) {
    case 16: ok = launch_shared_ka<T, 16>(G, grid, s, q, ka, va, part, T_len, chunk); break;
    case 32: ok = launch_shared_ka<T, 32>(G, grid, s, q, ka, va, part, T_len, chunk); break;
    case 64: ok = launch_shared_ka<T, 64>(G, grid, s, q, ka, va, part, T_len, chunk); break;
    case 128: ok = launch_shared_ka<T, 128>(G, grid, s, q, ka, va, part, T_len, chunk); break;
    case 256: ok = launch_shared_ka<T, 256>(G, grid, s, q, ka, va, part, T_len, chunk); break;
    case 512: ok = launch_shared_ka<T, 512>(G, grid, s, q, ka, va, part, T_len, chunk); break;
    default: break;
  }
  if (!ok) return false;
  hipLaunchKernelGGL(decode_attn_combine_kernel, dim3(n_q, B), dim3(Ka < 64 ? 64 : Ka), 0, s, part, out, (bf16*)nullptr,
                     (bf16*)nullptr, n_splits, B, n_q, Ka);
  return true;
}
template bool launch_absorbed_attn<float>(const float*, const float*, const float*, float*, float*, int, int, int, int, int, hipStream_t);
template bool launch_absorbed_attn<bf16>(const float*, const bf16*, const bf16*, float*, float*, int, int, int, int, int, hipStream_t);

// ---------------------------------------------------------------------------------------
// Generation loop (Sec. 4.1 "Inference", the loop after the first token): the base model's own
// key (rotated to position pos) and value of the token just fed go into slot pos of the cache.
// k, v: float [B][n_kv*hd];  cache layer: [B][n_kv][T_cap][hd].  One thread per rotary pair.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void kv_append_kernel(const float* __restrict__ k, const float* __restrict__ v,
                                                        T* __restrict__ kc, T* __restrict__ vc, int pos, int64_t T_cap,
                                                        int n_kv, int hd, const float2* __restrict__ rope_tab, int total) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int half = hd / 2;
  const int d = idx % half, head = (idx / half) % n_kv, b = idx / (half * n_kv);
  const float2 cs = rope_tab[(size_t)pos * half + d];
  const size_t src = ((size_t)b * n_kv + head) * hd + d;
  const size_t dst = (((size_t)b * n_kv + head) * (size_t)T_cap + pos) * hd + d;
  const float a = k[src], c = k[src + half];
  from_f32(kc[dst], a * cs.x - c * cs.y);
  from_f32(kc[dst + half], c * cs.x + a * cs.y);
  from_f32(vc[dst], v[src]);
  from_f32(vc[dst + half], v[src + half]);
}
template <typename T>
void launch_kv_append(const float* k, const float* v, T* kc, T* vc, int B, int pos, int64_t T_cap, int n_kv, int hd,
                      const float2* rope_tab, hipStream_t s) {
  const int total = B * n_kv * (hd / 2);
  hipLaunchKernelGGL((kv_append_kernel<T>), dim3((total + 255) / 256), dim3(256), 0, s, k, v, kc, vc, pos, T_cap, n_kv, hd,
                     rope_tab, total);
}
template void launch_kv_append<float>(const float*, const float*, float*, float*, int, int, int64_t, int, int, const float2*, hipStream_t);
template void launch_kv_append<bf16>(const float*, const float*, bf16*, bf16*, int, int, int64_t, int, int, const float2*, hipStream_t);

// ---------------------------------------------------------------------------------------
// Greedy first token: argmax over the vocabulary, lowest index among equal maxima; NaN never wins.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ logits, int32_t* __restrict__ out, int V) {
  __shared__ float bv[16];
  __shared__ int bi[16];
  const float* row = logits + (size_t)blockIdx.x * V;
  float best = -INFINITY; int idx = 0x7fffffff;
  auto take = [&](float v, int i) {            // (NaN fails both comparisons)
    if (v > best || (v == best && i < idx)) { best = v; idx = i; }
  };
  // 16-byte loads, eight in flight per thread (one pass over a 32k vocabulary), when the rows
  // stay 16-byte aligned; the remainder one element at a time
  constexpr int UN = 8;
  const int V4 = (V % 4 == 0) ? V / 4 : 0;
  const float4* row4 = reinterpret_cast<const float4*>(row);
  for (int c0 = threadIdx.x; c0 < V4; c0 += 1024 * UN) {
    float4 v[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) v[u] = row4[c0 + u * 1024 < V4 ? c0 + u * 1024 : 0];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int c = c0 + u * 1024;
      if (c < V4) { take(v[u].x, 4 * c); take(v[u].y, 4 * c + 1); take(v[u].z, 4 * c + 2); take(v[u].w, 4 * c + 3); }
    }
  }
  for (int i = V4 * 4 + threadIdx.x; i < V; i += 1024) take(row[i], i);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(best, o, 64); int oi = __shfl_xor(idx, o, 64);
    if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
  }
  int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  if (lane == 0) { bv[wave] = best; bi[wave] = idx; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < (int)(blockDim.x / kWave); ++w)
      if (bv[w] > best || (bv[w] == best && bi[w] < idx)) { best = bv[w]; idx = bi[w]; }
    out[blockIdx.x] = (idx == 0x7fffffff) ? 0 : idx;
  }
}

void launch_argmax(const float* logits, int32_t* out, int B, int V, hipStream_t s) {
  hipLaunchKernelGGL(argmax_kernel, dim3(B), dim3(1024), 0, s, logits, out, V);
}

}  // namespace kvp
