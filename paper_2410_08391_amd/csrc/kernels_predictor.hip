// Streaming predictor kernel (gfx950 matrix cores).
//
// The predictor (Sec. 4.2 "Predictor Networks") maps every token's auxiliary key (value) vector of
// width Ka to the key (value) vector of width Kb of each base layer fed by that auxiliary layer:
// a GEMM with a very short inner dimension (Ka = 256..512) and a very wide output (all base
// layers of a run x Kb columns), whose output, the predicted cache, is the dominant memory
// traffic.  A tiled GEMM spends most of such a tile in its prologue and epilogue.  Here the
// token side is stationary instead:
//
//   * a block owns 256 tokens (8 waves x 32 tokens) of one auxiliary layer's keys or values; every
//     wave loads its tokens' whole Ka-wide rows ONCE, straight into registers in the MFMA operand
//     layout (Ka/16 fragments of 8 bf16);
//   * the weights of all head tiles of the block's chunk (a run of base layers sharing that
//     auxiliary layer x a group of kv heads; a head tile = the 128 weight rows of one head)
//     stream through a ring of four LDS stages of 128 rows x 64 k as ONE continuous pipeline of
//     direct global->LDS loads - there is no per-tile prologue, the loads of K step g+4 are
//     issued while step g computes, across head-tile boundaries;
//   * per K step a wave issues 16 MFMAs (4 tiles of 32 weight rows x 4 sub-steps of 16 k) against
//     16 LDS fragment reads; accumulators hold the wave's 32 tokens x 128 columns of one head;
//   * after Ka/64 K steps the head tile is complete: converted to bf16, transposed through a
//     wave-private LDS tile and stored as whole 256-byte rows of the cache layout
//     [B][n_kv_b][T_cap][hd] (hd = 128), while the pipeline keeps running.
//
// Waiting.  Direct-to-LDS loads and the cache stores are issued as inline assembly and tracked by
// hand: vector memory operations of a wave complete in issue order, so "at most X outstanding"
// (s_waitcnt vmcnt(X)) with X = the number of operations issued after the loads of the next K
// step means those loads have landed.  X counts the two younger K steps' loads (2 per wave and
// step) plus, in the three steps after a head tile's epilogue, that epilogue's 8 stores - hence
// stores are issued unconditionally (tokens past the end are clamped to the last token, whose
// row they rewrite with identical values), so the count never depends on the data.
#include "mfma.h"

#include <cstdlib>

#include "gemm_mfma.h"

namespace kvp {

namespace {

constexpr int PS_WAVES = 8;
constexpr int PS_TOK = 32 * PS_WAVES;          // tokens per block
constexpr int PS_NS = 4;                        // ring stages
constexpr int PS_STAGE = 128 * GEMM_BK;         // elements per stage (128 weight rows x 64 k)
constexpr int PS_ROW = 128 + 8;                 // staging row (elements): 272 B, spreads rows over the banks
constexpr int PS_MAX_TILES = 256;               // head tiles per block (LDS pointer table)
constexpr int PS_MAX_RUNS = 64;

struct PredRuns { uint8_t lo[PS_MAX_RUNS]; uint8_t hi[PS_MAX_RUNS]; };

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void store16(bf16* dst, u32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off nt" : : "v"(dst), "v"(v) : "memory");
}

constexpr int wait_imm(int x) { return (x & 15) | ((x >> 4) << 14) | 0x0070; }   // vmcnt(x), lgkmcnt(0)

template <int KT>
__global__ __launch_bounds__(64 * PS_WAVES) void predictor_stream_kernel(
    const bf16* const* __restrict__ w_tab, const int32_t* __restrict__ layer_map, const bf16* __restrict__ aux_k,
    const bf16* __restrict__ aux_v, size_t aux_block, bf16* __restrict__ k_cache, bf16* __restrict__ v_cache,
    size_t layer_elems, int N, int T_len, int64_t T_cap, int n_kv_b, int hs, int tiles_tok, PredRuns runs) {
  constexpr int Ka = KT * GEMM_BK;
  constexpr int NF = KT * 4;                    // activation fragments (16 k each) per token
  static_assert(KT >= 4, "the store accounting assumes at most one epilogue in any three K steps");
  __shared__ __attribute__((aligned(1024))) bf16 ring[PS_NS * PS_STAGE];
  __shared__ __attribute__((aligned(16))) bf16 stg[PS_WAVES * 32 * PS_ROW];
  __shared__ const bf16* wptr[PS_MAX_TILES];
  __shared__ int64_t rowoff[PS_WAVES * 32];

  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int l32 = lane % 32, g = lane / 32;
  const int bid = blockIdx.x;
  const int tt = bid % tiles_tok, chunk = bid / tiles_tok;
  const int s = chunk & 1, hg = (chunk >> 1) % hs, r = (chunk >> 1) / hs;
  const int lo = runs.lo[r], hi = runs.hi[r];
  const int hpg = n_kv_b / hs;                  // heads per group
  const int n_tiles = (hi - lo) * hpg;          // <= PS_MAX_TILES (checked by the host)
  const int tok0 = tt * PS_TOK + wave * 32;

  if (tid < n_tiles) {
    int i = lo + tid / hpg, h = hg * hpg + tid % hpg;
    wptr[tid] = w_tab[2 * i + s] + (size_t)h * 128 * Ka;
  }
  if (lane < 32) {
    int n = min(tok0 + lane, N - 1);
    int b = n / T_len, t = n % T_len;
    rowoff[wave * 32 + lane] = ((int64_t)b * n_kv_b * T_cap + t) * 128;
  }
  __syncthreads();

  // this wave's tokens, whole rows, in the MFMA "B" operand layout: token l32, k = 16 f + 8 g ..
  const bf16* A = (s ? aux_v : aux_k) + (size_t)layer_map[lo] * aux_block;
  bf16x8 act[NF];
  {
    const bf16* arow = A + (size_t)min(tok0 + l32, N - 1) * Ka + 8 * g;
#pragma unroll
    for (int f = 0; f < NF; ++f) act[f] = *reinterpret_cast<const bf16x8*>(arow + 16 * f);
  }

  // ring loads: one wave instruction fills 8 rows x 128 B; a wave issues two per K step
  int lane_off[2];
#pragma unroll
  for (int ld = 0; ld < 2; ++ld) {
    int row = (ld * PS_WAVES + wave) * 8 + lane / 8;
    int ch = (lane % 8) ^ swz_key(row);
    lane_off[ld] = row * Ka + ch * 8;
  }
  // loads of K step (tile u, position kt) into `stage`; tiles past the end re-load the last tile
  // (the data is never used; the operation count per step stays fixed)
  auto issue_one = [&](bf16* stage, int u, int kt, int ld) {
    const bf16* base = wptr[min(u, n_tiles - 1)] + kt * GEMM_BK;
    load_lds16(base + lane_off[ld], stage + (ld * PS_WAVES + wave) * 8 * GEMM_BK);
  };
#pragma unroll
  for (int st = 0; st < PS_NS; ++st) {
    issue_one(ring + st * PS_STAGE, st / KT, st % KT, 0);
    issue_one(ring + st * PS_STAGE, st / KT, st % KT, 1);
  }

  f32x16 acc[4];
  bf16x8 wf[2][4];
  auto read_frag = [&](const bf16* stage, int ks, int set, int ct) {
    wf[set][ct] = *reinterpret_cast<const bf16x8*>(stage + swz(ct * 32 + l32, ks * 2 + g));
  };

  // K step 0 has landed when at most the three younger steps' loads are outstanding
  __builtin_amdgcn_s_waitcnt(wait_imm((PS_NS - 1) * 2) | 0x0F00);
  __syncthreads();
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) read_frag(ring, 0, 0, ct);

  constexpr int X_STRICT = (PS_NS - 2) * 2;     // two younger K steps' loads
  constexpr int X_LAX = X_STRICT + 8;           // ... and one epilogue's stores among them
  bf16* wl = stg + wave * 32 * PS_ROW;
  int sidx = 0;
  for (int u = 0; u < n_tiles; ++u) {
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[ct][i] = 0.f;
    const bool after_epilogue = u > 0;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      bf16* cur = ring + sidx * PS_STAGE;
      const bf16* nxt = ring + ((sidx + 1) % PS_NS) * PS_STAGE;
      // the K step whose loads go into the stage this step frees: step g + NS
      const int u_ld = u + (kt + PS_NS) / KT, kt_ld = (kt + PS_NS) % KT;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int set = ks & 1;
        if (ks == 3) {
          // loads of the next K step have landed (in issue order: everything older than the X
          // youngest operations is complete) and this wave's reads of the current stage are done
          if (kt <= 2 && after_epilogue) __builtin_amdgcn_s_waitcnt(wait_imm(X_LAX));
          else __builtin_amdgcn_s_waitcnt(wait_imm(X_STRICT));
          __builtin_amdgcn_s_barrier();
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
          acc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[set][ct], act[kt * 4 + ks], acc[ct], 0, 0, 0);
          if (ks < 3) read_frag(cur, ks + 1, set ^ 1, ct);
          else read_frag(nxt, 0, set ^ 1, ct);
          if (ks == 3 && ct < 2) issue_one(cur, u_ld, kt_ld, ct);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      sidx = (sidx + 1) % PS_NS;
    }
    // head tile u complete: this wave's 32 tokens x 128 columns -> bf16 -> rows of the cache
    {
      const int i = lo + u / hpg, h = hg * hpg + u % hpg;
      bf16* obase = (s ? v_cache : k_cache) + (size_t)i * layer_elems + (size_t)h * T_cap * 128;
      // A lane holds, per group of four accumulator registers q, columns 8q + 4g .. + 3 of a 32-column tile.
      // Swapping the upper half-wave's group 2p with the lower half-wave's group 2p + 1 (v_permlane32_swap)
      // leaves every lane with 8 consecutive columns, 8 (2p + g) .. + 7: one 16-byte LDS write, bank-conflict free.
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int pq = 0; pq < 2; ++pq) {
          bf16x4 e4, o4;
#pragma unroll
          for (int e = 0; e < 4; ++e) { e4[e] = (bf16)acc[ct][(2 * pq) * 4 + e]; o4[e] = (bf16)acc[ct][(2 * pq + 1) * 4 + e]; }
          const u32x2 ev = __builtin_bit_cast(u32x2, e4), ov = __builtin_bit_cast(u32x2, o4);
          const u32x2 rx = __builtin_amdgcn_permlane32_swap(ev[0], ov[0], false, false);
          const u32x2 ry = __builtin_amdgcn_permlane32_swap(ev[1], ov[1], false, false);
          *reinterpret_cast<u32x4*>(wl + l32 * PS_ROW + ct * 32 + (2 * pq + g) * 8) = u32x4{rx[0], ry[0], rx[1], ry[1]};
        }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // wave-private tile: program order suffices
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int row = it * 4 + lane / 16, seg = lane % 16;
        u32x4 v = *reinterpret_cast<const u32x4*>(wl + row * PS_ROW + seg * 8);
        store16(obase + rowoff[wave * 32 + row] + seg * 8, v);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0070);   // the trailing (unused) ring loads must land before the LDS is released
}

}  // namespace

bool mfma_predictor_stream(const kvp_handle* h, void* tables, const bf16* aux_k, const bf16* aux_v, bf16* k_cache,
                           bf16* v_cache, int B, int T_len, int64_t T_cap, int layer0, int layer1, int Ka, int Kb,
                           int n_kv_b, size_t aux_block, size_t layer_elems, hipStream_t s) {
  const kvp_config& c = handle_cfg(h);
  const MfmaTables* t = static_cast<const MfmaTables*>(tables);
  const int N = B * T_len;
  const char* force = getenv("KVP_PRED_STREAM");      // "0": never, "1": whenever the shape allows (tests, tuning)
  if (force && force[0] == '0') return false;
  if (c.base.head_dim != 128 || Kb != n_kv_b * 128 || (Ka != 256 && Ka != 512)) return false;
  if (c.base.n_layers > 255 || layer1 <= layer0 || N < 1) return false;
  // The token side is stationary, so small prompts leave most of the chip idle: the tiled GEMM serves them
  if (!(force && force[0] == '1') && N < 4096) return false;
  const std::vector<int32_t>& lm = handle_layer_map(h);
  PredRuns runs;
  int n_runs = 0, longest = 0;
  for (int i = layer0; i < layer1;) {
    int e = i + 1;
    while (e < layer1 && lm[e] == lm[i]) ++e;
    if (n_runs == PS_MAX_RUNS) return false;
    runs.lo[n_runs] = (uint8_t)i; runs.hi[n_runs] = (uint8_t)e;
    ++n_runs;
    longest = e - i > longest ? e - i : longest;
    i = e;
  }
  const int tiles_tok = (N + PS_TOK - 1) / PS_TOK;
  // split the kv heads over blocks until the grid covers the chip (or a block is one head per layer)
  int hs = 1;
  while (hs < n_kv_b && (n_kv_b % (hs * 2) == 0) &&
         ((long)tiles_tok * 2 * n_runs * hs < 256 || longest * (n_kv_b / hs) > PS_MAX_TILES)) hs *= 2;
  if (longest * (n_kv_b / hs) > PS_MAX_TILES) return false;
  dim3 grid((unsigned)((long)tiles_tok * 2 * hs * n_runs));
  if (Ka == 256)
    hipLaunchKernelGGL(predictor_stream_kernel<4>, grid, dim3(64 * PS_WAVES), 0, s, t->w_tab, t->layer_map, aux_k, aux_v,
                       aux_block, k_cache, v_cache, layer_elems, N, T_len, T_cap, n_kv_b, hs, tiles_tok, runs);
  else
    hipLaunchKernelGGL(predictor_stream_kernel<8>, grid, dim3(64 * PS_WAVES), 0, s, t->w_tab, t->layer_map, aux_k, aux_v,
                       aux_block, k_cache, v_cache, layer_elems, N, T_len, T_cap, n_kv_b, hs, tiles_tok, runs);
  return true;
}

}  // namespace kvp
