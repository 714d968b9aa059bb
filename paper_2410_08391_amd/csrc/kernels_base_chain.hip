// bf16 base-model step (Sec. 4.1 "Inference": b <- B(I[-1], KV^_B)) as a chain of GEMV kernels
// that hand activations to each other already split into bf16 high / low halves.
//
// Every projection of the single-token step is y = W x for a handful of right-hand sides, which
// is pure weight streaming, in a chain of ~6 dependent kernels per layer that run a few
// microseconds each.  Two things therefore decide the time: how well the weight stream is
// coalesced, and how many memory round trips lie on a wave's critical path.
//   * gemv_chain_kernel (3..16 right-hand sides, v_mfma_f32_16x16x32_bf16): a block owns 16*RT
//     consecutive weight rows and splits K over its waves.  Weights are read as 256-byte row
//     pieces and brought into the matrix-core "A" layout through a wave-private LDS region (or,
//     for odd shapes, loaded straight in that layout: lane (r = lane%16, g = lane/16) holds
//     W[row r][32 s + 8 g .. + 7], 16 rows x 64 bytes per wave load);
//   * gemv_rows_kernel (1 or 2 right-hand sides): plain ALU, a wave owns whole rows;
//   * the right-hand sides arrive as two bf16 arrays hi, lo with hi + lo == the float32
//     activation to ~2^-17, written by the producing kernel: two MFMAs per step, one per half
//     (the ALU kernel adds them back to float32);
//   * RMSNorm is folded in: the producer stores hi/lo of (y * gain_next) together with partial
//     sums of y^2; the consumer adds the partials (fixed order) and scales its result by
//     rsqrt(mean + eps), which commutes with the matrix product;
//   * a wave requests everything it will need (norm partials, the epilogue's old residual values
//     and gains, right-hand sides, a whole batch of weights) before it waits for anything;
//   * waves are merged through LDS in a fixed order, so results are bit-reproducible.
#include <cstdlib>
#include <type_traits>
#include "common.h"
#include "launch.h"

namespace kvp {

__device__ __forceinline__ void split_store(bf16* hi, bf16* lo, size_t idx, float v) {
  bf16 h = (bf16)v;
  hi[idx] = h;
  lo[idx] = (bf16)(v - (float)h);
}

// y[b,:] = E[last token of sequence b]; hi/lo = split(y * gain); ssq[b] = sum(y^2).  One block per b.
// A token id outside [0, vocab) is clamped and sets bit 0 of *flags.
__global__ __launch_bounds__(256) void base_embed_kernel(const int32_t* __restrict__ tokens, int T_len,
                                                         const bf16* __restrict__ E, int vocab,
                                                         const bf16* __restrict__ gain, float* __restrict__ y,
                                                         bf16* __restrict__ uh, bf16* __restrict__ ul,
                                                         float* __restrict__ ssq, int d, uint32_t* __restrict__ flags) {
  __shared__ float red[4];
  const int b = blockIdx.x;
  int tok = tokens[(size_t)b * T_len + T_len - 1];
  if ((tok < 0 || tok >= vocab) && threadIdx.x == 0) atomicOr(flags, 1u);
  tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
  const bf16* e = E + (size_t)tok * d;
  float ss = 0.f;
  for (int i0 = threadIdx.x; i0 < d; i0 += 256 * 8) {     // eight independent loads per trip: one round trip for d <= 2048
    bf16 ev[8], gv[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u * 256;
      ev[u] = e[i < d ? i : 0];
      gv[u] = gain[i < d ? i : 0];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u * 256;
      if (i < d) {
        const float v = (float)ev[u];
        y[(size_t)b * d + i] = v;
        ss += v * v;
        split_store(uh, ul, (size_t)b * d + i, v * (float)gv[u]);
      }
    }
  }
  ss = wave_sum(ss);
  if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = ss;
  __syncthreads();
  if (threadIdx.x == 0) ssq[b] = red[0] + red[1] + red[2] + red[3];
}

struct ChainArgs {
  const bf16* W;          // [N, K]
  const bf16* W2;         // MODE 2: second matrix [N, K]
  const bf16* xh;         // right-hand sides, high halves [B, K]
  const bf16* xl;         // low halves
  const float* ssq_in;    // NORM: [B, n_part_in] partial sums of squares of the un-gained input
  int n_part_in;
  float eps;
  float* out;             // MODE 0: [B, N] result;  MODE 1: [B, N] residual stream, updated in place
  const bf16* gain_next;  // MODE 1: gain of the norm that follows, [N]
  bf16* oh;               // MODE 1: split(y_new * gain_next);  MODE 2: split(silu(g) * u)    [B, N]
  bf16* ol;
  float* ssq_out;         // MODE 1: [B, gridDim.x] partial sums of y_new^2
  int B, N, K;
  // gemv_rows_kernel<.., MERGE>: the right-hand side is the merge of decode-attention split partials
  // [n_splits][B][n_q][hd + kPartPad] (hd un-normalised sums, running maximum, normaliser), K = n_q * hd
  const float* part = nullptr;
  int n_splits = 0, n_q = 0, hd = 0;
};

// Steps per batch of loads: as many as keep weights (4 registers per step and row tile) plus
// right-hand sides (8 per group of QG steps) within a budget out of the 128 registers a wave may
// hold when two 8-wave blocks share a CU (84, or 64 where the LDS route needs temporaries), at
// most 16 and at least one unit.
constexpr int chain_batch_steps(int rtnm, int qg, int unit, int budget) {
  int u = unit;                                // unit: a multiple of qg
  while (u + unit <= 16 && rtnm * (u + unit) * 4 + ((u + unit) / qg) * 8 <= budget) u += unit;
  return u;
}

// Lane i of each row of 16 lanes receives the value of lane i + SH of the same row (zero past the row's end).
template <int SH>
__device__ __forceinline__ bf16x8 row_shift_down(bf16x8 v) {
  if constexpr (SH == 0) {
    return v;
  } else {
    union { bf16x8 b; int i[4]; } in, out;
    in.b = v;
#pragma unroll
    for (int d = 0; d < 4; ++d) out.i[d] = __builtin_amdgcn_update_dpp(0, in.i[d], 0x100 + SH /* row_shl */, 0xf, 0xf, true);
    return out.b;
  }
}

// QG: matrix-core steps served by one load of the right-hand sides.  With at most 16 / QG
// right-hand sides the 16 lanes of a row are split into QG groups that fetch the operand of QG
// consecutive steps at once; a row shift then brings each group's data to the lanes the step
// reads (columns >= 16 / QG of the result hold sums of other steps' data and are never stored).
//
// LDSW: the weights take the coalesced route.  A wave load then covers 4 rows x 256 contiguous
// bytes (a quarter wave reads two whole cache lines instead of 16 bytes of each of 16 lines);
// four such loads are a unit of 16 rows x 128 k, which the wave writes to its own 4 KB of LDS
// and reads back in the matrix-core layout, four steps at a time (16-byte pieces of a row are
// stored at position piece ^ row, which keeps both the writes and the reads free of bank
// conflicts).  No barrier is involved: the region is private to the wave and LDS operations of
// a wave execute in order.  Needs K % 128 == 0 and N % 16 == 0.
//
// NW: waves per block, which split K among them.  The launcher uses 8: two such blocks fit a CU
// (registers and LDS), so one block's loads are in flight while the other reduces, stores and
// retires; 16-wave blocks, one per CU, streamed the weights 8-15 % slower, 4-wave blocks 4 % slower.
//
// STREAM: the weights are loaded with the non-temporal hint (read once per launch).  Off for more than 16
// right-hand sides, where the grid's rows share each weight tile through L2 and the hint costs 10 %.
template <int MODE, bool NORM, int NW, int RT, int QG, bool LDSW = false, bool STREAM = true>
__global__ __launch_bounds__(NW * 64) void gemv_chain_kernel(ChainArgs a) {
  // More than 16 right-hand sides: grid row y serves right-hand sides 16 y .. 16 y + 15.  The rows
  // of the grid run side by side, so a weight tile fetched for one of them is in L2 for the
  // others (same block column -> same XCD when the grid width is a multiple of 8).
  if (blockIdx.y > 0 || a.B > 16) {
    const int b0 = (int)blockIdx.y * 16;
    a.xh += (size_t)b0 * a.K; a.xl += (size_t)b0 * a.K;
    if (a.ssq_in) a.ssq_in += (size_t)b0 * a.n_part_in;
    if (a.out) a.out += (size_t)b0 * a.N;
    if (a.oh) { a.oh += (size_t)b0 * a.N; a.ol += (size_t)b0 * a.N; }
    if (a.ssq_out) a.ssq_out += (size_t)b0 * ((a.N + 15) / 16);
    a.B = min(16, a.B - b0);
  }
  constexpr int NM = (MODE == 2) ? 2 : 1;
  // steps whose loads are in flight together (a multiple of QG; LDSW: also of 4)
  constexpr int U = LDSW ? chain_batch_steps(RT * NM, QG, QG > 4 ? QG : 4, 64) : chain_batch_steps(RT * NM, QG, QG, 84);
  constexpr int NXG = U / QG;                                  // right-hand-side loads per batch
  constexpr int NPQ = 16 / QG;                                 // right-hand sides a row can serve
  static_assert(U % QG == 0, "a batch is a whole number of right-hand-side groups");
  constexpr int NBW = 16 / NW;                // right-hand sides whose norm a wave prepares (wave, wave + NW)
  constexpr int PU = 4;                       // norm partials per lane in the first round trip
  __shared__ float red[NW][RT * NM][16][17];
  __shared__ float scale_sh[16];
  __shared__ bf16x8 wst[LDSW ? NW : 1][LDSW ? 256 : 1];       // LDSW: one unit of 16 rows x 128 k per wave
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;   // (uniform: the slice bounds are scalars)
  const int r = lane % 16, g = lane / 16;
  const int B = a.B, N = a.N, K = a.K;
  const int n = min(r % NPQ, B - 1), xq = r / NPQ;   // this lane fetches right-hand side n for step (group start + xq)
  const int steps = (K + 31) / 32;
  // slice of K of this wave, in steps of 32 (LDSW: whole units of 4 steps)
  const int SG = LDSW ? 4 : 1;
  const int s0 = (int)((long)wave * (steps / SG) / NW) * SG, s1 = (int)((long)(wave + 1) * (steps / SG) / NW) * SG;

  // These kernels run a few microseconds each in a dependent chain, so a wave asks for everything
  // it will need before it waits for anything: norm partials, the epilogue's old residual values
  // and gains, then its first batch of weights (all of them for most shapes).  Loads are
  // unconditional with clamped addresses; scheduling fences keep the compiler from sinking them.
  float pn[NBW][PU], pn_more[NBW];
  if (NORM) {
#pragma unroll
    for (int t = 0; t < NBW; ++t) {
      const float* src = a.ssq_in + (size_t)min(wave + t * NW, B - 1) * a.n_part_in;
#pragma unroll
      for (int j = 0; j < PU; ++j) pn[t][j] = src[lane + j * kWave < a.n_part_in ? lane + j * kWave : 0];
      pn_more[t] = 0.f;                        // more than 64 PU partials (d_model > 4096): waited for here, one trip each
      for (int i = lane + PU * kWave; i < a.n_part_in; i += kWave) pn_more[t] += src[i];
    }
  }
  // epilogue operands of thread t < 256 RT: row i of row tile `tile`, right-hand side j
  const int e_tile = (int)threadIdx.x / 256, e_i = (int)threadIdx.x % 16, e_j = ((int)threadIdx.x % 256) / 16;
  const int e_row = ((int)blockIdx.x * RT + e_tile) * 16 + e_i;
  const size_t e_o = (size_t)min(e_j, B - 1) * N + min(e_row, N - 1);
  constexpr bool PRE = 256 * RT <= NW * 64;   // the epilogue is one trip: thread t finishes output t
  float y_old = 0.f;
  bf16 g_next = (bf16)0.f;
  if (MODE == 1 && PRE && threadIdx.x < 256 * RT) {
    y_old = a.out[e_o];
    g_next = a.gain_next[min(e_row, N - 1)];
  }
  __builtin_amdgcn_sched_barrier(0);

  const bf16* wrow[RT];
  const bf16* w2row[RT];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    // direct: row r of the tile;  LDSW: row lane/16 of the tile (+ 4 per load of a unit), 16-byte piece lane%16
    int row = LDSW ? min(((int)blockIdx.x * RT + t) * 16, N - 16) + g : min(((int)blockIdx.x * RT + t) * 16 + r, N - 1);
    wrow[t] = a.W + (size_t)row * K + (LDSW ? r * 8 : 0);
    w2row[t] = (MODE == 2) ? a.W2 + (size_t)row * K + (LDSW ? r * 8 : 0) : nullptr;
  }
  const bf16* xh = a.xh + (size_t)n * K;
  const bf16* xl = a.xl + (size_t)n * K;

  auto load_w = [](const bf16* p) { return STREAM ? load_stream8(p) : *reinterpret_cast<const bf16x8*>(p); };
  f32x4 acc[RT * NM];
#pragma unroll
  for (int m = 0; m < RT * NM; ++m) acc[m] = f32x4{0.f, 0.f, 0.f, 0.f};
  const bf16x8 zero8 = {(bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f};

  // (a wave without a slice of K, when there are fewer steps than waves, still makes one pass:
  //  all its loads are clamped and discarded, and it owes its share of the norm)
  for (int sb = s0; sb < s1 || sb == s0; sb += U) {
    bf16x8 wv[RT * NM][U], hi[NXG], lo[NXG];
    // Loads are unconditional (a straight run, so the waits can be counted); a step past the
    // slice, or lanes past the end of K, read the first 16 bytes of the array instead, all lanes
    // the same line, which costs next to nothing.
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (LDSW) {                    // load u % 4 of unit u / 4: rows 4 (u % 4) + lane / 16, all 128 k of the unit
        const bool ok = sb + u / 4 * 4 < s1;
        const size_t off = (size_t)(u % 4) * 4 * K + (size_t)(sb + u / 4 * 4) * 32;
#pragma unroll
        for (int t = 0; t < RT; ++t) {
          wv[t * NM][u] = load_w(ok ? wrow[t] + off : a.W);
          if (MODE == 2) wv[t * NM + NM - 1][u] = load_w(ok ? w2row[t] + off : a.W2);
        }
      } else {
        const int k = (sb + u) * 32 + g * 8;
        const bool ok = (sb + u < s1) && (k < K);
#pragma unroll
        for (int t = 0; t < RT; ++t) {
          wv[t * NM][u] = load_w(ok ? wrow[t] + k : a.W);
          if (MODE == 2) wv[t * NM + NM - 1][u] = load_w(ok ? w2row[t] + k : a.W2);
        }
      }
    }
#pragma unroll
    for (int x = 0; x < NXG; ++x) {
      const int k = (sb + x * QG + xq) * 32 + g * 8;
      const bool ok = (sb + x * QG + xq < s1) && (k < K);
      hi[x] = *reinterpret_cast<const bf16x8*>(ok ? xh + k : a.xh);
      lo[x] = *reinterpret_cast<const bf16x8*>(ok ? xl + k : a.xl);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (NORM && sb == s0) {                    // while the weights are on their way
#pragma unroll
      for (int t = 0; t < NBW; ++t) {
        const int b = wave + t * NW;
        if (b < B) {                           // partial sums in index order per lane, as they were written
          float v = 0.f;
#pragma unroll
          for (int j = 0; j < PU; ++j) {
            asm volatile("" : "+v"(pn[t][j]));   // keeps this use (and its wait) below the loads above; it would be hoisted out of the loop
            v += lane + j * kWave < a.n_part_in ? pn[t][j] : 0.f;
          }
          v = wave_sum(v + pn_more[t]);
          if (lane == 0) scale_sh[b] = rsqrtf(v / (float)K + a.eps);
        }
      }
    }
    if constexpr (LDSW) {                      // units through LDS into the matrix-core layout, in place in wv
#pragma unroll
      for (int ub = 0; ub < U / 4; ++ub) {
        if (sb + ub * 4 < s1) {                // (uniform)
#pragma unroll
          for (int m = 0; m < RT * NM; ++m) {
            // Lanes exchange data through the wave's LDS region without a block barrier: the LDS
            // operations of one wave execute in program order.  The wavefront-scope fences emit no
            // instruction; they keep the compiler from moving a lane's reads across the other
            // lanes' writes (which a single thread's view of memory would allow).
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
            for (int i = 0; i < 4; ++i) wst[wave][(4 * i + g) * 16 + (r ^ (4 * i + g))] = wv[m][ub * 4 + i];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) wv[m][ub * 4 + s4] = wst[wave][r * 16 + ((4 * s4 + g) ^ r)];
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          }
        }
      }
    }
#pragma unroll
    for (int x = 0; x < NXG; ++x) {
      const int k = (sb + x * QG + xq) * 32;
      const bool ok = (sb + x * QG + xq < s1) && (k + g * 8 < K);
      const bf16x8 hx = ok ? hi[x] : zero8;    // a zero right-hand side discards what a clamped load returned
      const bf16x8 lx = ok ? lo[x] : zero8;
      auto step = [&](auto qc) {
        constexpr int q = decltype(qc)::value;
        const int u = x * QG + q;
        if (sb + u >= s1) return;              // (uniform)
        const bf16x8 h8 = row_shift_down<q * NPQ>(hx), l8 = row_shift_down<q * NPQ>(lx);
#pragma unroll
        for (int m = 0; m < RT * NM; ++m) {
          acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[m][u], h8, acc[m], 0, 0, 0);
          acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[m][u], l8, acc[m], 0, 0, 0);
        }
      };
      step(std::integral_constant<int, 0>{});
      if constexpr (QG >= 2) step(std::integral_constant<int, 1>{});
      if constexpr (QG >= 4) { step(std::integral_constant<int, 2>{}); step(std::integral_constant<int, 3>{}); }
    }
  }
  // accumulator: lane (col = lane%16 = right-hand side, g) holds rows 4g .. 4g+3
#pragma unroll
  for (int m = 0; m < RT * NM; ++m)
#pragma unroll
    for (int i = 0; i < 4; ++i) red[wave][m][g * 4 + i][r] = acc[m][i];
  __syncthreads();

  for (int t = threadIdx.x; t < 256 * RT; t += NW * 64) {
    const int tile = t / 256, i = t % 16, j = (t % 256) / 16;   // row i of row tile `tile`, right-hand side j
    const int orow = ((int)blockIdx.x * RT + tile) * 16 + i;
    const bool live = j < B && orow < N;
    float v[NM];
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) s += red[w][tile * NM + m][i][j];
      v[m] = s;
    }
    if (NORM) {
      const float sc = scale_sh[min(j, B - 1)];
#pragma unroll
      for (int m = 0; m < NM; ++m) v[m] *= sc;
    }
    const size_t o = (size_t)min(j, B - 1) * N + min(orow, N - 1);
    if (MODE == 0) {
      if (live) a.out[o] = v[0];
    } else if (MODE == 1) {
      float yn = 0.f;
      if (live) {
        yn = (PRE ? y_old : a.out[o]) + v[0];
        a.out[o] = yn;
        split_store(a.oh, a.ol, o, yn * (float)(PRE ? g_next : a.gain_next[orow]));
      }
      // sum of y_new^2 over the 16 rows of this tile (the 16 lanes that share j), fixed order
      float sq = yn * yn;
      sq += __shfl_xor(sq, 1, 64);
      sq += __shfl_xor(sq, 2, 64);
      sq += __shfl_xor(sq, 4, 64);
      sq += __shfl_xor(sq, 8, 64);
      const int n_tiles = (N + 15) / 16, ti = (int)blockIdx.x * RT + tile;   // one partial per row tile, whatever RT is
      if (i == 0 && j < B && ti < n_tiles) a.ssq_out[(size_t)j * n_tiles + ti] = sq;
    } else {
      if (live) split_store(a.oh, a.ol, o, v[0] * v[NM - 1] * __builtin_amdgcn_rcpf(1.f + __expf(-v[0])));
    }
  }
}

// ---------------------------------------------------------------------------------------
// One or two right-hand sides: plain-ALU GEMV with fully coalesced weight reads.
// The matrix-core kernel above reads 16 rows x 64 B per wave instruction, which costs 40-60 %
// over a contiguous stream at these sizes; with one or two right-hand sides the arithmetic is
// trivial, so here a wave owns R whole rows and reads each as contiguous 1 KB pieces (lane l
// covers k = 512 c + 8 l .. + 7).  Same inputs, outputs and fused operations as
// gemv_chain_kernel.
//
// These kernels run a few microseconds each, one after another, with about one wave per SIMD,
// so what counts is the number of memory round trips on a wave's critical path, not occupancy.
// Everything a wave will need is therefore requested before anything is waited for: the
// right-hand side (rebuilt as float32 in LDS, once per block), the partial sums of the folded
// RMSNorm, the old residual values and next gains of the epilogue, and the weights of up to CG
// pieces per row (the whole row for every benchmark shape) -- one round trip in all.
// ---------------------------------------------------------------------------------------
template <int MODE, bool NORM, int NB, int R, bool MERGE, int CG>
__global__ __launch_bounds__(256) void gemv_rows_kernel(ChainArgs a) {
  constexpr int NM = (MODE == 2) ? 2 : 1;
  constexpr int WK = CG * 512;                // k-values per group (CG pieces per row)
  constexpr int XU = CG / 4;                  // 8-wide chunks of the right-hand side per thread and group
  constexpr int PU = 4;                       // norm partials per lane in the first round trip
  static_assert(CG % 4 == 0, "a group is a whole number of 2048-wide thread passes");
  __shared__ __attribute__((aligned(16))) float xs[NB][WK];
  __shared__ float sq_sh[4][NB];
  __shared__ float scale_sh[NB];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int N = a.N, K = a.K;
  const int row0 = ((int)blockIdx.x * 4 + wave) * R;
  const bf16x8 zero8 = {(bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f};

  // Loads are unconditional with clamped addresses, so that they form one straight run and the
  // waits can be counted; what a clamped load returned is discarded where it is used.
  bf16x8 wv[NM][R][CG];
  auto load_weights = [&](int k0) {
#pragma unroll
    for (int c = 0; c < CG; ++c) {
      const int k = k0 + c * 512 + lane * 8;
      const bool ok = k < K;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const size_t off = (size_t)min(row0 + r, N - 1) * K + (ok ? k : 0);
        wv[0][r][c] = load_stream8(a.W + off);
        if (MODE == 2) wv[NM - 1][r][c] = load_stream8(a.W2 + off);
      }
    }
  };
  bf16x8 xh[NB][XU], xl[NB][XU];
  auto load_rhs = [&](int k0) {
#pragma unroll
    for (int u = 0; u < XU; ++u) {
      const int k = k0 + ((int)threadIdx.x + u * 256) * 8;
      const int kc = k < K ? k : 0;
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        xh[b][u] = *reinterpret_cast<const bf16x8*>(a.xh + (size_t)b * K + kc);
        xl[b][u] = *reinterpret_cast<const bf16x8*>(a.xl + (size_t)b * K + kc);
      }
    }
  };
  // float32 right-hand side of group k0 into LDS (zeros beyond K)
  auto stage_rhs = [&](int k0) {
#pragma unroll
    for (int u = 0; u < XU; ++u) {
      const int kl = ((int)threadIdx.x + u * 256) * 8;
      const bool ok = k0 + kl < K;
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        float x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = ok ? (float)xh[b][u][i] + (float)xl[b][u][i] : 0.f;
        *reinterpret_cast<float4*>(&xs[b][kl]) = float4{x[0], x[1], x[2], x[3]};
        *reinterpret_cast<float4*>(&xs[b][kl + 4]) = float4{x[4], x[5], x[6], x[7]};
      }
    }
  };
  // The same from decode-attention split partials: thread t owns 8 consecutive dims of one head.
  // Same operations, in the same order per element, as decode_attn_combine_kernel (splits in
  // batches of eight).
  auto stage_merged = [&](int k0) {
    const size_t stride = (size_t)a.B * a.n_q * (a.hd + kPartPad);
#pragma unroll 1
    for (int u = 0; u < XU; ++u) {
      const int kl = ((int)threadIdx.x + u * 256) * 8;
      const int k8 = k0 + kl;
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = 0.f;
        float l = 1.f;
        if (k8 < K) {
          const int hq = k8 / a.hd, d = k8 % a.hd;
          const float* p0 = a.part + ((size_t)b * a.n_q + hq) * (a.hd + kPartPad);
          float m = -INFINITY;
          l = 0.f;
          for (int s0 = 0; s0 < a.n_splits; s0 += 8) {
            float mv[8], lv[8];
            float2 ov[8][4];
#pragma unroll
            for (int v = 0; v < 8; ++v) {
              const bool ok = s0 + v < a.n_splits;
              const float* pr = p0 + (size_t)(ok ? s0 + v : 0) * stride;
              mv[v] = ok ? pr[a.hd] : -INFINITY;
              lv[v] = pr[a.hd + 1];
#pragma unroll
              for (int i = 0; i < 4; ++i) ov[v][i] = *reinterpret_cast<const float2*>(pr + d + 2 * i);   // rows are 8-byte aligned only
            }
            float mb = m;
#pragma unroll
            for (int v = 0; v < 8; ++v) mb = fmaxf(mb, mv[v]);
            const float corr = (m == -INFINITY) ? 0.f : __expf(m - mb);
            l *= corr;
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] *= corr;
#pragma unroll
            for (int v = 0; v < 8; ++v) {
              const float w = (mv[v] == -INFINITY) ? 0.f : __expf(mv[v] - mb);
              l += lv[v] * w;
#pragma unroll
              for (int i = 0; i < 4; ++i) { o[2 * i] += ov[v][i].x * w; o[2 * i + 1] += ov[v][i].y * w; }
            }
            m = mb;
          }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) xs[b][kl + i] = o[i] / l;
      }
    }
  };

  // -- requests of the first group (scheduling fences keep them ahead of every use: the
  //    compiler would otherwise interleave loads and uses to save registers) -----------------
  if (!MERGE) load_rhs(0);
  __builtin_amdgcn_sched_barrier(0);
  float pn[PU];
  if (NORM) {                                  // every wave asks (for right-hand side wave % NB); waves < NB use it
    const float* src = a.ssq_in + (size_t)(wave % NB) * a.n_part_in;
#pragma unroll
    for (int j = 0; j < PU; ++j) {
      const int i = lane + j * kWave;
      pn[j] = src[i < a.n_part_in ? i : 0];
    }
  }
  // epilogue operands: lane l < R * NB finishes output (row l / NB, right-hand side l % NB)
  const int er = (lane % (R * NB)) / NB, eb = lane % NB;
  const int erow = row0 + er;
  const bool elive = lane < R * NB && erow < N;
  const size_t eo = (size_t)eb * N + min(erow, N - 1);
  float y_old = 0.f;
  bf16 g_next = (bf16)0.f;
  if (MODE == 1) {
    y_old = a.out[eo];
    g_next = a.gain_next[min(erow, N - 1)];
  }
  __builtin_amdgcn_sched_barrier(0);
  load_weights(0);
  __builtin_amdgcn_sched_barrier(0);

  float acc[NM][R][NB];
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int b = 0; b < NB; ++b) acc[m][r][b] = 0.f;

  for (int k0 = 0; k0 < K; k0 += WK) {
    if (k0 > 0) {                              // rows wider than CG pieces (no benchmark shape): one more round trip per group
      __syncthreads();
      if (!MERGE) load_rhs(k0);
      load_weights(k0);
    }
    if (MERGE) stage_merged(k0); else stage_rhs(k0);
    if (NORM && k0 == 0 && wave < NB) {        // partial sums in index order per lane, as they were written
      float v = 0.f;
#pragma unroll
      for (int j = 0; j < PU; ++j) v += lane + j * kWave < a.n_part_in ? pn[j] : 0.f;
      for (int i = lane + PU * kWave; i < a.n_part_in; i += kWave) v += a.ssq_in[(size_t)wave * a.n_part_in + i];
      v = wave_sum(v);
      if (lane == 0) scale_sh[wave] = rsqrtf(v / (float)K + a.eps);
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < CG; ++c) {
      if (k0 + c * 512 < K) {                  // (uniform) pieces beyond the row hold no data
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          const float4 x0 = *reinterpret_cast<const float4*>(&xs[b][c * 512 + lane * 8]);
          const float4 x1 = *reinterpret_cast<const float4*>(&xs[b][c * 512 + lane * 8 + 4]);
          const float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
          for (int m = 0; m < NM; ++m)
#pragma unroll
            for (int r = 0; r < R; ++r) {
              const bf16x8 w = k0 + c * 512 + lane * 8 < K ? wv[m][r][c] : zero8;
              float s = acc[m][r][b];
#pragma unroll
              for (int i = 0; i < 8; ++i) s += (float)w[i] * x[i];
              acc[m][r][b] = s;
            }
        }
      }
    }
  }
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int b = 0; b < NB; ++b) acc[m][r][b] = wave_sum(acc[m][r][b]);

  // -- epilogue: lane l < R * NB owns one output ---------------------------------------------
  float v0 = 0.f, v1 = 0.f;
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int b = 0; b < NB; ++b)
      if (er == r && eb == b) { v0 = acc[0][r][b]; v1 = acc[NM - 1][r][b]; }
  if (NORM) { const float sc = scale_sh[eb]; v0 *= sc; v1 *= sc; }
  float sq = 0.f;
  if (MODE == 0) {
    if (elive) a.out[eo] = v0;
  } else if (MODE == 1) {
    const float yn = y_old + v0;
    if (elive) {
      a.out[eo] = yn;
      split_store(a.oh, a.ol, eo, yn * (float)g_next);
      sq = yn * yn;
    }
  } else {
    if (elive) split_store(a.oh, a.ol, eo, v0 * v1 * __builtin_amdgcn_rcpf(1.f + __expf(-v0)));
  }
  if (MODE == 1) {                             // per-block partial sum of y_new^2, rows then waves in fixed order
    float tot = sq;
#pragma unroll
    for (int r = 1; r < R; ++r) tot += __shfl(sq, r * NB + eb, 64);
    if (lane < NB) sq_sh[wave][lane] = tot;
    __syncthreads();
    if (threadIdx.x < NB)
      a.ssq_out[(size_t)threadIdx.x * gridDim.x + blockIdx.x] =
          sq_sh[0][threadIdx.x] + sq_sh[1][threadIdx.x] + sq_sh[2][threadIdx.x] + sq_sh[3][threadIdx.x];
  }
}

constexpr int ROWS_R = 2;                      // rows per wave of gemv_rows_kernel (8 rows per block)

template <int MODE, bool NORM, int NB, bool MERGE>
static void launch_rows_nb(const ChainArgs& a, hipStream_t s) {
  dim3 grid((a.N + 4 * ROWS_R - 1) / (4 * ROWS_R)), block(256);
  const int pieces = (a.K + 511) / 512;
  // whole rows in flight when they fit the registers (two matrices: up to 8 pieces)
  if (pieces <= 4) hipLaunchKernelGGL((gemv_rows_kernel<MODE, NORM, NB, ROWS_R, MERGE, 4>), grid, block, 0, s, a);
  else if (pieces <= 8 || MODE == 2) hipLaunchKernelGGL((gemv_rows_kernel<MODE, NORM, NB, ROWS_R, MERGE, 8>), grid, block, 0, s, a);
  else if constexpr (MODE != 2) hipLaunchKernelGGL((gemv_rows_kernel<MODE, NORM, NB, ROWS_R, MERGE, 12>), grid, block, 0, s, a);
}

template <int MODE, bool NORM, bool MERGE = false>
static void launch_rows(const ChainArgs& a, hipStream_t s) {
  if (a.B == 1) launch_rows_nb<MODE, NORM, 1, MERGE>(a, s);
  else launch_rows_nb<MODE, NORM, 2, MERGE>(a, s);
}

// KVP_CHAIN_DIRECT=1 keeps the weights on the direct (matrix-core layout) loads, for comparison.
static bool chain_direct_loads() {
  static const bool v = [] { const char* e = getenv("KVP_CHAIN_DIRECT"); return e && e[0] == '1'; }();
  return v;
}

constexpr int CHAIN_NW = 8;                    // waves per block of gemv_chain_kernel

template <int MODE, bool NORM, int QG, bool STREAM = true>
static void launch_chain_qg(const ChainArgs& a, int rt, hipStream_t s) {
  // row tiles per block are capped so that weights and right-hand sides of a batch fit the registers
  constexpr int RT_MAX = (QG == 4 ? 4 : 2) / (MODE == 2 ? 2 : 1);
  constexpr int NW = CHAIN_NW;
  dim3 block(NW * 64);
  int tiles = (a.N + 15) / 16;
  const unsigned gy = (unsigned)((a.B + 15) / 16);     // groups of 16 right-hand sides
  if (rt > RT_MAX) rt = RT_MAX;
  // rows of 2048 and more elements: coalesced weights through LDS (at most 2 tiles x matrices)
  if (a.K >= 2048 && a.K % 128 == 0 && a.N % 16 == 0 && !chain_direct_loads()) {
    if constexpr (RT_MAX >= 2 && MODE != 2) {
      if (rt >= 2) { hipLaunchKernelGGL((gemv_chain_kernel<MODE, NORM, NW, 2, QG, true, STREAM>), dim3((tiles + 1) / 2, gy), block, 0, s, a); return; }
    }
    hipLaunchKernelGGL((gemv_chain_kernel<MODE, NORM, NW, 1, QG, true, STREAM>), dim3(tiles, gy), block, 0, s, a);
    return;
  }
  if constexpr (RT_MAX >= 4) {
    if (rt == 4) { hipLaunchKernelGGL((gemv_chain_kernel<MODE, NORM, NW, 4, QG, false, STREAM>), dim3((tiles + 3) / 4, gy), block, 0, s, a); return; }
  }
  if constexpr (RT_MAX >= 2) {
    if (rt >= 2) { hipLaunchKernelGGL((gemv_chain_kernel<MODE, NORM, NW, 2, QG, false, STREAM>), dim3((tiles + 1) / 2, gy), block, 0, s, a); return; }
  }
  hipLaunchKernelGGL((gemv_chain_kernel<MODE, NORM, NW, 1, QG, false, STREAM>), dim3(tiles, gy), block, 0, s, a);
}
template <int MODE, bool NORM>
static void launch_chain_rt(const ChainArgs& a, int rt, hipStream_t s) {
  if (a.B <= 4) launch_chain_qg<MODE, NORM, 4>(a, rt, s);
  else if (a.B <= 8) launch_chain_qg<MODE, NORM, 2>(a, rt, s);
  else if (a.B <= 16) launch_chain_qg<MODE, NORM, 1>(a, rt, s);
  else launch_chain_qg<MODE, NORM, 1, false>(a, rt, s);       // several grid rows share the weights through L2
}

// Row tiles per block: more of them for the tall matrices (the LM head), whose grids are many times the chip.
int chain_row_tiles(int N) {
  int tiles = (N + 15) / 16;
  if (tiles <= 256) return 1;
  if (tiles <= 512) return 2;
  return 4;
}
int chain_ssq_parts(int N, int B) {
  if (B <= 2) return (N + 4 * ROWS_R - 1) / (4 * ROWS_R);   // gemv_rows_kernel: one partial per block
  return (N + 15) / 16;                                      // gemv_chain_kernel: one partial per tile of 16 rows
}

template <int MODE, bool NORM>
static void launch_chain(ChainArgs a, hipStream_t s) {
  if (a.B <= 2) { launch_rows<MODE, NORM>(a, s); return; }
  launch_chain_rt<MODE, NORM>(a, chain_row_tiles(a.N), s);
}

void launch_base_embed(const int32_t* tokens, int T_len, const bf16* E, int vocab, const bf16* gain, float* y, bf16* uh,
                       bf16* ul, float* ssq, int B, int d, uint32_t* flags, hipStream_t s) {
  hipLaunchKernelGGL(base_embed_kernel, dim3(B), dim3(256), 0, s, tokens, T_len, E, vocab, gain, y, uh, ul, ssq, d, flags);
}
void launch_chain_project(const bf16* W, const bf16* xh, const bf16* xl, const float* ssq_in, int n_part_in, float eps,
                          float* out, int B, int N, int K, hipStream_t s) {
  ChainArgs a{W, nullptr, xh, xl, ssq_in, n_part_in, eps, out, nullptr, nullptr, nullptr, nullptr, B, N, K};
  if (ssq_in) launch_chain<0, true>(a, s); else launch_chain<0, false>(a, s);
}
void launch_chain_residual(const bf16* W, const bf16* xh, const bf16* xl, float* y, const bf16* gain_next, bf16* yh,
                           bf16* yl, float* ssq_out, int B, int N, int K, hipStream_t s) {
  ChainArgs a{W, nullptr, xh, xl, nullptr, 0, 0.f, y, gain_next, yh, yl, ssq_out, B, N, K};
  launch_chain<1, false>(a, s);
}
bool launch_chain_residual_merge(const bf16* W, const float* part, int n_splits, int n_q, int hd, float* y,
                                 const bf16* gain_next, bf16* yh, bf16* yl, float* ssq_out, int B, int N, int K,
                                 hipStream_t s) {
  if (B > 2 || K != n_q * hd || hd % 8 != 0) return false;
  ChainArgs a{W, nullptr, nullptr, nullptr, nullptr, 0, 0.f, y, gain_next, yh, yl, ssq_out, B, N, K};
  a.part = part; a.n_splits = n_splits; a.n_q = n_q; a.hd = hd;
  launch_rows<1, false, true>(a, s);
  return true;
}
void launch_chain_swiglu(const bf16* Wg, const bf16* Wu, const bf16* xh, const bf16* xl, const float* ssq_in,
                         int n_part_in, float eps, bf16* ah, bf16* al, int B, int N, int K, hipStream_t s) {
  ChainArgs a{Wg, Wu, xh, xl, ssq_in, n_part_in, eps, nullptr, nullptr, ah, al, nullptr, B, N, K};
  launch_chain<2, true>(a, s);
}

}  // namespace kvp
