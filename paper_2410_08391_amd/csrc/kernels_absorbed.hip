// Base step with the predictor absorbed into the attention (gfx950).
//
// The predictor of base layer i is a pair of linear maps applied to the auxiliary layer j_i
// (Sec. 4.2 "Predictor Networks": K^_i = K_A W_K^T, V^_i = V_A W_V^T, W of shape [Kb, Ka]).
// Attention of query head h (key/value head g, W^g = rows [g hd, (g+1) hd) of W) over the
// predicted cache is therefore attention over the auxiliary cache itself:
//     q . K^_u        = (W_K^g^T q) . K_A,u
//     sum_u p_u V^_u  = W_V^g (sum_u p_u V_A,u)
// so the first token (Sec. 4.1 "Inference", b <- B(I[-1], KV^_B)) does not have to wait for the
// predicted cache to be written.  Three kernels per layer:
//     absorb_q   q~[b, h, :] = W_K^g^T rope(q[b, h, :]) / sqrt(hd)          [B][n_q][Ka]
//     attention  r[b, h, :]  = softmax_u(q~ . K_A,u) V_A                     [B][n_q][Ka]
//                (all query heads of a sequence share the auxiliary rows: on the matrix cores
//                 16 heads are the 16 columns of one MFMA tile)
//     absorb_o   o[b, h, :]  = W_V^g r[b, h, :]                              [B][n_q*hd]
#include "common.h"
#include "launch.h"

namespace kvp {

// Eight consecutive matrix elements as loaded (converted to float only where they are used, so that
// a load can be requested long before).
template <typename T> struct Raw8;
template <> struct Raw8<bf16> { bf16x8 v; };
template <> struct Raw8<float> { f32x4 a, b; };
__device__ __forceinline__ Raw8<bf16> raw8(const bf16* p) { return Raw8<bf16>{*reinterpret_cast<const bf16x8*>(p)}; }
__device__ __forceinline__ Raw8<float> raw8(const float* p) {
  return Raw8<float>{*reinterpret_cast<const f32x4*>(p), *reinterpret_cast<const f32x4*>(p + 4)};
}
__device__ __forceinline__ float elem(const Raw8<bf16>& r, int i) { return (float)r.v[i]; }
__device__ __forceinline__ float elem(const Raw8<float>& r, int i) { return i < 4 ? r.a[i] : r.b[i - 4]; }

constexpr int kAbsorbGMax = 8;

// ---------------------------------------------------------------------------------------
// absorb_q.  q: float [B][n_q][hd] (unrotated); wk: [n_kv*hd][Ka] row-major; out: float
// [B][n_q][Ka].  Grid (n_kv, ceil(Ka / 128), B), 256 threads: thread (rl = tid / 16, cp = tid % 16)
// sums rows rl, rl + 16, .. of W_K^g over its 8 columns for the G heads of the group; the 16
// partial sums meet through two shuffles and LDS.  The first eight rows of every thread (all of
// them up to head_dim 128) are requested before the queries are staged: one memory round trip.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void absorb_q_kernel(const float* __restrict__ q, const T* __restrict__ wk,
                                                       float* __restrict__ out, int n_q, int G, int hd, int Ka, int pos,
                                                       const float2* __restrict__ rope_tab, float scale) {
  __shared__ float q_sh[kAbsorbGMax][256];                 // hd <= 256
  __shared__ float red[4][kAbsorbGMax][128];
  const int g = blockIdx.x, cx = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, cp = tid % 16, rl = tid / 16, wave = tid / kWave;
  const int col = cx * 128 + cp * 8;
  const bool col_ok = col < Ka;
  const int half = hd / 2;
  const T* wbase = wk + (size_t)g * hd * Ka + (col_ok ? col : 0);
  Raw8<T> wr[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) wr[k] = raw8(wbase + (size_t)min(rl + 16 * k, hd - 1) * Ka);   // rows >= hd: unused
  for (int i = tid; i < G * half; i += 256) {
    const int hh = i / half, d = i % half;
    const float* qr = q + ((size_t)b * n_q + (size_t)g * G + hh) * hd;
    const float2 cs = rope_tab[(size_t)pos * half + d];
    const float a = qr[d], c = qr[d + half];
    q_sh[hh][d] = (a * cs.x - c * cs.y) * scale;
    q_sh[hh][d + half] = (c * cs.x + a * cs.y) * scale;
  }
  __syncthreads();
  float acc[kAbsorbGMax][8];
#pragma unroll
  for (int hh = 0; hh < kAbsorbGMax; ++hh)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[hh][i] = 0.f;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int d = rl + 16 * k;
    if (d < hd) {
#pragma unroll
      for (int hh = 0; hh < kAbsorbGMax; ++hh)
        if (hh < G) {
          const float qv = q_sh[hh][d];
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[hh][i] += qv * elem(wr[k], i);
        }
    }
  }
  for (int d = rl + 128; d < hd; d += 16) {                // head_dim above 128
    const Raw8<T> w = raw8(wbase + (size_t)d * Ka);
#pragma unroll
    for (int hh = 0; hh < kAbsorbGMax; ++hh)
      if (hh < G) {
        const float qv = q_sh[hh][d];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[hh][i] += qv * elem(w, i);
      }
  }
  // lanes l, l ^ 16, l ^ 32 hold other rows of the same columns
#pragma unroll
  for (int hh = 0; hh < kAbsorbGMax; ++hh)
    if (hh < G) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float v = acc[hh][i];
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        if (tid % kWave < 16) red[wave][hh][cp * 8 + i] = v;
      }
    }
  __syncthreads();
  for (int i = tid; i < G * 128; i += 256) {
    const int hh = i / 128, c = i % 128;
    if (cx * 128 + c < Ka)
      out[((size_t)b * n_q + (size_t)g * G + hh) * Ka + cx * 128 + c] =
          (red[0][hh][c] + red[1][hh][c]) + (red[2][hh][c] + red[3][hh][c]);
  }
}

template <typename T>
bool launch_absorb_q(const float* q, const T* wk, float* out, int B, int n_q, int n_kv, int hd, int Ka, int pos,
                     const float2* rope_tab, hipStream_t s) {
  const int G = n_q / n_kv;
  if (G > kAbsorbGMax || hd > 256 || hd % 2 || Ka % 8) return false;
  hipLaunchKernelGGL((absorb_q_kernel<T>), dim3(n_kv, (Ka + 127) / 128, B), dim3(256), 0, s, q, wk, out, n_q, G, hd, Ka, pos,
                     rope_tab, 1.0f / sqrtf((float)hd));
  return true;
}
template bool launch_absorb_q<float>(const float*, const float*, float*, int, int, int, int, int, int, const float2*, hipStream_t);
template bool launch_absorb_q<bf16>(const float*, const bf16*, float*, int, int, int, int, int, int, const float2*, hipStream_t);

// ---------------------------------------------------------------------------------------
// absorb_o.  r: float [B][n_q][Ka]; wv: [n_kv*hd][Ka] row-major; out[b][h*hd + d] =
// wv[g*hd + d, :] . r[b, h, :], as float and / or as bf16 high + low halves (for the matrix-core
// output projection).  Ka / 8 lanes per row of W_V^g (Ka a power of two between 16 and 512), each
// holding its 8 columns of r for the G heads; 256 / (Ka / 8) rows side by side, two such rounds
// per block: grid (n_kv, ceil(hd / rows per block), B).  Every load is requested before the
// first use; the sums over the lanes of a row use DPP inside 16 lanes.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float lanes_sum(float v, int lpr) {     // lpr consecutive lanes (a power of two), all get the sum
  if (lpr >= 2) v += row_dpp<0xB1>(v);
  if (lpr >= 4) v += row_dpp<0x4E>(v);
  if (lpr >= 8) v += row_dpp<0x141>(v);
  if (lpr >= 16) v += row_dpp<0x140>(v);
  if (lpr >= 32) v += __shfl_xor(v, 16, 64);
  if (lpr >= 64) v += __shfl_xor(v, 32, 64);
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void absorb_o_kernel(const float* __restrict__ r, const T* __restrict__ wv,
                                                       float* __restrict__ out, bf16* __restrict__ out_hi,
                                                       bf16* __restrict__ out_lo, int n_q, int G, int hd, int Ka) {
  const int g = blockIdx.x, b = blockIdx.z;
  const int lpr = Ka / 8, rows_par = 256 / lpr;
  const int sub = threadIdx.x % lpr, rgrp = threadIdx.x / lpr;
  const int d0 = blockIdx.y * 2 * rows_par + rgrp;
  const T* wbase = wv + (size_t)g * hd * Ka + sub * 8;
  Raw8<T> wr[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) wr[k] = raw8(wbase + (size_t)min(d0 + k * rows_par, hd - 1) * Ka);
  f32x4 rv[kAbsorbGMax][2];
#pragma unroll
  for (int hh = 0; hh < kAbsorbGMax; ++hh) {
    const float* rr = r + ((size_t)b * n_q + (size_t)g * G + (hh < G ? hh : 0)) * Ka + sub * 8;
    rv[hh][0] = *reinterpret_cast<const f32x4*>(rr);
    rv[hh][1] = *reinterpret_cast<const f32x4*>(rr + 4);
  }
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int d = d0 + k * rows_par;
#pragma unroll
    for (int hh = 0; hh < kAbsorbGMax; ++hh)
      if (hh < G) {
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) v += rv[hh][i / 4][i % 4] * elem(wr[k], i);
        v = lanes_sum(v, lpr);
        if (sub == 0 && d < hd) {
          const size_t idx = ((size_t)b * n_q + (size_t)g * G + hh) * hd + d;
          if (out) out[idx] = v;
          if (out_hi) {
            const bf16 hv = (bf16)v;
            out_hi[idx] = hv;
            out_lo[idx] = (bf16)(v - (float)hv);
          }
        }
      }
  }
}

template <typename T>
bool launch_absorb_o(const float* r, const T* wv, float* out, bf16* out_hi, bf16* out_lo, int B, int n_q, int n_kv, int hd,
                     int Ka, hipStream_t s) {
  const int G = n_q / n_kv;
  if (G > kAbsorbGMax || !absorbed_attn_supported(Ka)) return false;
  const int rows_per_block = 2 * (256 / (Ka / 8));
  hipLaunchKernelGGL((absorb_o_kernel<T>), dim3(n_kv, (hd + rows_per_block - 1) / rows_per_block, B), dim3(256), 0, s, r, wv,
                     out, out_hi, out_lo, n_q, G, hd, Ka);
  return true;
}
template bool launch_absorb_o<float>(const float*, const float*, float*, bf16*, bf16*, int, int, int, int, int, hipStream_t);
template bool launch_absorb_o<bf16>(const float*, const bf16*, float*, bf16*, bf16*, int, int, int, int, int, hipStream_t);

// ---------------------------------------------------------------------------------------
// The attention itself on the matrix cores, bf16 auxiliary cache, Ka = 256 or 512.
//   q    float [B][n_q][KA], rotated, mapped and scaled (natural-log domain)
//   ka   [B*T][KA] token-major keys of the auxiliary layer
//   vT   [B][KA][T_pad] its values transposed (column c of token t at [c][t]; T_pad a multiple
//        of 64, entries t >= T finite)
//   part [n_splits][B][n_q][KA + kPartPad]: unnormalised sums, running maximum (natural log), sum of
//        weights: the format decode_attn_combine_kernel merges.
// Grid (n_splits, ceil(n_q / 16), B), 4 waves; wave w takes the 32-key pieces w, w + 4, .. of the
// block's chunk.  Per piece:
//   scores  S^T[key][head] = K_A q~  : two 16-key tiles x KA/32 v_mfma_f32_16x16x32_bf16 (x 2: q~
//           as bf16 high + low halves, read from LDS in operand layout).  Tile t, row rho stands
//           for key 8 (rho / 4) + 4 t + rho % 4, so that the accumulator lane (head n, g) holds
//           keys 8 g .. 8 g + 7 of the piece: exactly the "B" operand of the next product.
//   softmax statistics per head = per lane column, two shuffles across g.
//   R^T[c][head] += V_A^T P : VC/16 tiles (a block owns VC of the KA value columns; KA / VC blocks
//           repeat the scores of a head tile), "A" = vT rows loaded straight from global memory
//           (lane (r, g): column c0 + r, keys 8 g .. 8 g + 7), "B" = the probabilities in
//           registers.  Nothing passes through LDS inside the loop except q~.
// ---------------------------------------------------------------------------------------
template <int KA, int VC>
__global__ __launch_bounds__(256) void absorbed_attn_mfma_kernel(const float* __restrict__ q, const bf16* __restrict__ ka,
                                                                 const bf16* __restrict__ vT, float* __restrict__ part,
                                                                 int T_len, int T_pad, int n_q, int chunk) {
  constexpr int KS = KA / 32;                    // k-steps of a score tile
  constexpr int NT = VC / 16;                    // column tiles of R^T this block owns
  constexpr int NVC = KA / VC;                   // blocks sharing a head tile, VC value columns each
  constexpr int OST = VC + 4;                    // row stride of the merge buffer (floats)
  constexpr int SMEM = 2 * KS * 1024 > 16 * OST * 4 ? 2 * KS * 1024 : 16 * OST * 4;
  __shared__ __attribute__((aligned(16))) char smem[SMEM];   // q~ fragments (2 * KS KB), later the merge buffer
  __shared__ float st_m[4][16], st_l[4][16];
  bf16x8* qh_sh = reinterpret_cast<bf16x8*>(smem);            // [KS][64]
  bf16x8* ql_sh = qh_sh + KS * 64;                            // [KS][64]
  float* o_sh = reinterpret_cast<float*>(smem);               // [16][OST]

  const int split = blockIdx.x, h0 = (blockIdx.y / NVC) * 16, vc0 = (blockIdx.y % NVC) * VC, b = blockIdx.z, B = gridDim.z;
  const int tid = threadIdx.x, lane = tid % kWave, wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int n = lane % 16, g = lane / 16;
  const int c0 = split * chunk, c1 = min(T_len, c0 + chunk);
  const bf16* kbase = ka + (size_t)b * T_len * KA + g * 8;
  const bf16* vbase = vT + ((size_t)b * KA + vc0 + n) * T_pad + g * 8;
  const int last_row = T_len - 1;
  const int krow = 8 * (n / 4) + n % 4;          // key of tile row n within the piece (+ 4 t)

  bf16x8 kreg[2][KS], vreg[NT];
  auto issue_k = [&](int k0) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const bf16* row = kbase + (size_t)min(k0 + krow + 4 * t, last_row) * KA;
#pragma unroll
      for (int s = 0; s < KS; ++s) kreg[t][s] = *reinterpret_cast<const bf16x8*>(row + 32 * s);
    }
  };
  auto issue_v = [&](int k0) {                   // k0 + 8 g + 7 < T_pad: k0 is a multiple of 32 below T_len
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) vreg[ct] = *reinterpret_cast<const bf16x8*>(vbase + (size_t)(16 * ct) * T_pad + k0);
  };
  const int k_first = c0 + 32 * wave;
  if (k_first < c1) { issue_k(k_first); issue_v(k_first); }

  // q~ into LDS in "B" operand layout: entry (s, lane (n, g)) = q~[h0 + n][32 s + 8 g .. + 7], exp2 domain
  for (int e = tid; e < KS * 64; e += 256) {
    const int s = e / 64, ln = e % 64, nn = ln % 16, gg = ln / 16;
    bf16x8 hi, lo;
    if (h0 + nn < n_q) {
      const float* src = q + ((size_t)b * n_q + h0 + nn) * KA + 32 * s + 8 * gg;
      const f32x4 a = *reinterpret_cast<const f32x4*>(src), c = *reinterpret_cast<const f32x4*>(src + 4);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float v = (i < 4 ? a[i] : c[i - 4]) * 1.4426950408889634f;
        const bf16 hv = (bf16)v;
        hi[i] = hv;
        lo[i] = (bf16)(v - (float)hv);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) { hi[i] = (bf16)0.f; lo[i] = (bf16)0.f; }
    }
    qh_sh[e] = hi;
    ql_sh[e] = lo;
  }
  __syncthreads();

  float m_run = -INFINITY, l_run = 0.f;          // head n; l is this lane's share (its 8 keys per piece)
  f32x4 acc[NT];
#pragma unroll
  for (int ct = 0; ct < NT; ++ct) acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int k0 = k_first; k0 < c1; k0 += 128) {
    f32x4 sc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    int qoff = lane;
    asm volatile("" : "+v"(qoff));               // the fragments are re-read every piece, not held in registers
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const bf16x8 qh = qh_sh[s * 64 + qoff], ql = ql_sh[s * 64 + qoff];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[t][s], qh, sc[t], 0, 0, 0);
        sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[t][s], ql, sc[t], 0, 0, 0);
      }
    }
    const int k_next = k0 + 128;
    if (k_next < c1) issue_k(k_next);
    // lane (head n, g): sc[t][i] is key k0 + 8 g + 4 t + i
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (k0 + 8 * g + 4 * t + i >= c1) sc[t][i] = -INFINITY;
        mx = fmaxf(mx, sc[t][i]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);        // finite: key k0 is valid
    const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
    float psum = 0.f;
    bf16x8 pb;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p = __builtin_amdgcn_exp2f(sc[t][i] - m_new);
        psum += p;
        pb[4 * t + i] = (bf16)p;
      }
    l_run = l_run * corr + psum;
    m_run = m_new;
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
      acc[ct] *= corr;
      acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vreg[ct], pb, acc[ct], 0, 0, 0);
    }
    if (k_next < c1) issue_v(k_next);
  }

  // ---- merge the four waves ----
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (g == 0) { st_m[wave][n] = m_run; st_l[wave][n] = l_run; }
  __syncthreads();                               // statistics visible; every wave is done with the q~ fragments
  float m_blk = fmaxf(fmaxf(st_m[0][n], st_m[1][n]), fmaxf(st_m[2][n], st_m[3][n]));   // wave 0 always has a key
  const float wgt = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run - m_blk);
  // lane (head n, g) holds columns 16 ct + 4 g + i of head n; the waves add in wave order
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int ct = 0; ct < NT; ++ct) {
        f32x4* dst = reinterpret_cast<f32x4*>(o_sh + n * OST + 16 * ct + 4 * g);
        f32x4 v = acc[ct] * wgt;
        if (w > 0) v += *dst;
        *dst = v;
      }
    }
    __syncthreads();
  }
  for (int i = tid; i < 16 * VC; i += 256) {
    const int hh = i / VC, c = i % VC;
    if (h0 + hh >= n_q) continue;
    float* pr = part + (((size_t)split * B + b) * n_q + h0 + hh) * (KA + kPartPad);
    pr[vc0 + c] = o_sh[hh * OST + c];
    if (c == 0 && vc0 == 0) {                      // (every column block computes the same statistics)
      const float mb = fmaxf(fmaxf(st_m[0][hh], st_m[1][hh]), fmaxf(st_m[2][hh], st_m[3][hh]));
      float l = 0.f;
      for (int w = 0; w < 4; ++w)
        l += (st_m[w][hh] == -INFINITY) ? 0.f : st_l[w][hh] * __builtin_amdgcn_exp2f(st_m[w][hh] - mb);
      pr[KA] = mb * 0.6931471805599453f;
      pr[KA + 1] = l;
    }
  }
}

int absorbed_mfma_chunk(int B, int n_q, int T_len) {
  // about two blocks per CU, chunks of whole 128-key rounds (four waves x 32 keys)
  const int tiles = (n_q + 15) / 16;
  int want = (512 + B * tiles - 1) / (B * tiles);
  int chunk = (T_len + want - 1) / want;
  chunk = ((chunk + 127) / 128) * 128;
  return chunk;
}
int absorbed_mfma_splits(int B, int n_q, int T_len) {
  const int chunk = absorbed_mfma_chunk(B, n_q, T_len);
  return (T_len + chunk - 1) / chunk;
}
bool absorbed_mfma_supported(int Ka) { return Ka == 256 || Ka == 512; }

bool launch_absorbed_attn_mfma(const float* q, const bf16* ka, const bf16* vT, float* part, float* out, int B, int T_len,
                               int T_pad, int n_q, int Ka, hipStream_t s) {
  const int chunk = absorbed_mfma_chunk(B, n_q, T_len);
  const int n_splits = (T_len + chunk - 1) / chunk;
  const int tiles = (n_q + 15) / 16;
  if (Ka == 256)
    hipLaunchKernelGGL((absorbed_attn_mfma_kernel<256, 256>), dim3(n_splits, tiles, B), dim3(256), 0, s, q, ka, vT, part,
                       T_len, T_pad, n_q, chunk);
  else if (Ka == 512)       // two blocks per head tile, 256 value columns each (registers)
    hipLaunchKernelGGL((absorbed_attn_mfma_kernel<512, 256>), dim3(n_splits, 2 * tiles, B), dim3(256), 0, s, q, ka, vT, part,
                       T_len, T_pad, n_q, chunk);
  else
    return false;
  launch_decode_combine(part, out, n_splits, B, n_q, Ka, s);
  return true;
}

}  // namespace kvp
