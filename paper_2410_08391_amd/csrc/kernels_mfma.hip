// bf16 MFMA kernels for the auxiliary prefill and the predictor (gfx950 matrix cores):
// projection GEMMs with fused epilogues, causal grouped-query flash attention, and the
// predictor GEMMs that write the base cache layout directly.
#include "mfma.h"

#include <cstdlib>

#include "gemm_mfma.h"

namespace kvp {

// =========================================================================================
// GEMM operand sources and epilogues
// =========================================================================================

// Plain weight matrix W[N, K]: virtual column v of block tn is row tn*BN + v.
template <int BN>
struct BPlain {
  const bf16* W; int N, K;
  __device__ const bf16* a_base(const bf16* A, int) const { return A; }
  __device__ const bf16* row_ptr(int, int tn, int half, int r) const {
    int n = min(tn * BN + half * (BN / 2) + r, N - 1);
    return W + (size_t)n * K;
  }
};
// X[m, n] += v  on the float32 residual stream (N % 4 == 0: a run of 4 columns is all in or out)
template <int BN>
struct EpiResidualPair {
  typedef float out_t;
  static constexpr int HALVES = 2;
  typedef float vec4 __attribute__((ext_vector_type(4)));
  float* X; int N;
  __device__ void transform(int, int, int, const float (&v0)[4], const float (&v1)[4], vec4& o0, vec4& o1) const {
    o0 = vec4{v0[0], v0[1], v0[2], v0[3]};
    o1 = vec4{v1[0], v1[1], v1[2], v1[3]};
  }
  static constexpr bool PRELOAD = true;            // store() receives old contents + new value
  __device__ vec4 load(int, int m, int tn, int half, int p) const {
    int c = min(tn * BN + half * (BN / 2) + p, N - 4);   // N % 4 == 0; columns past N are never stored
    return *reinterpret_cast<const vec4*>(X + (size_t)m * N + c);
  }
  __device__ void store(int, int m, int tn, int half, int p, const vec4& v) const {
    int c = tn * BN + half * (BN / 2) + p;
    if (c >= N) return;
    *reinterpret_cast<vec4*>(X + (size_t)m * N + c) = v;
  }
};

// SwiGLU: half 0 = gate rows, half 1 = up rows of the same feed-forward units.
template <int BN>
struct BGateUp {
  const bf16* Wg; const bf16* Wu; int F, K;
  __device__ const bf16* a_base(const bf16* A, int) const { return A; }
  __device__ const bf16* row_ptr(int, int tn, int half, int r) const {
    int n = min(tn * (BN / 2) + r, F - 1);
    return (half ? Wu : Wg) + (size_t)n * K;
  }
};
template <int BN>
struct EpiSwiGLU {
  typedef bf16 out_t;
  static constexpr int HALVES = 1;                 // gate and up fold into one output
  static constexpr bool PRELOAD = false;
  bf16* act; int F;
  __device__ void transform(int, int, int, const float (&v0)[4], const float (&v1)[4], bf16x4& o0, bf16x4&) const {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float gte = v0[e];
      // silu(g) * u = g * u / (1 + 2^(-g log2 e)); hardware exp2 and reciprocal (1 ulp) suffice for bf16 output
      o0[e] = (bf16)(gte * v1[e] * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gte)));
    }
  }
  __device__ void store(int, int m, int tn, int, int p, const bf16x8& v) const {
    int c = tn * (BN / 2) + p;
    if (c >= F) return;                            // F % 8 == 0: a run of 8 is all in or out
    *reinterpret_cast<bf16x8*>(act + (size_t)m * F + c) = v;
  }
};

// Q, K, V projections of head_dim 128 heads.  A block covers BN/128 heads; half 0 holds
// dims 0..63 and half 1 dims 64..127 of each, i.e. the two members of every rotary pair.
// Heads are numbered q heads first, then k heads, then v heads; `head0` skips the q heads
// for the last auxiliary layer.
template <int BN>
struct BQKV {
  static constexpr int HB = BN / 128;
  const bf16* wq; const bf16* wk; const bf16* wv; int n_q, n_kv, head0, K;
  __device__ const bf16* a_base(const bf16* A, int) const { return A; }
  __device__ const bf16* row_ptr(int, int tn, int half, int r) const {
    int head = min(head0 + tn * HB + r / 64, n_q + 2 * n_kv - 1);
    int d = r % 64 + half * 64;
    const bf16* W; int hh;
    if (head < n_q) { W = wq; hh = head; }
    else if (head < n_q + n_kv) { W = wk; hh = head - n_q; }
    else { W = wv; hh = head - n_q - n_kv; }
    return W + ((size_t)hh * 128 + d) * K;
  }
};
template <int BN>
struct EpiQKVRope {
  typedef bf16 out_t;
  static constexpr int HALVES = 2;                 // half 0: dims 0..63 of a head, half 1: dims 64..127
  static constexpr bool PRELOAD = false;
  static constexpr int HB = BN / 128;
  bf16* q; bf16* k; bf16* v;
  int n_q, n_kv, head0, T_len;
  const float2* tab;    // [pos][64] (cos, sin)
  int rot_heads;        // heads below this index are rotated (n_q + n_kv; 0: rotation is left to a later kernel)
  __device__ void transform(int m, int tn, int p, const float (&v0)[4], const float (&v1)[4], bf16x4& o0, bf16x4& o1) const {
    int head = head0 + tn * HB + p / 64, d = p % 64;
    if (head < rot_heads) {
      const f32x4* cs = reinterpret_cast<const f32x4*>(tab + (size_t)(m % T_len) * 64 + d);
      f32x4 cs01 = cs[0], cs23 = cs[1];     // (cos, sin) of dims d, d+1 and d+2, d+3
      const float c[4] = {cs01[0], cs01[2], cs23[0], cs23[2]}, sn[4] = {cs01[1], cs01[3], cs23[1], cs23[3]};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o0[e] = (bf16)(v0[e] * c[e] - v1[e] * sn[e]);
        o1[e] = (bf16)(v1[e] * c[e] + v0[e] * sn[e]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) { o0[e] = (bf16)v0[e]; o1[e] = (bf16)v1[e]; }
    }
  }
  __device__ void store(int, int m, int tn, int half, int p, const bf16x8& val) const {
    int head = head0 + tn * HB + p / 64, d = p % 64 + half * 64;
    if (head >= n_q + 2 * n_kv) return;
    bf16* dst = (head < n_q)          ? q + (size_t)m * (n_q * 128) + head * 128 + d
                : (head < n_q + n_kv) ? k + (size_t)m * (n_kv * 128) + (head - n_q) * 128 + d
                                      : v + (size_t)m * (n_kv * 128) + (head - n_q - n_kv) * 128 + d;
    *reinterpret_cast<bf16x8*>(dst) = val;
  }
};

// Predictor (Sec. 4.2): problem `batch` = 2*i + s maps auxiliary layer j_i's keys (s = 0) or
// values (s = 1) with W_{K,i} / W_{V,i} into base layer i of the caller's cache.
template <int BN>
struct BPredictor {
  const bf16* const* w_tab;      // device [2 * L_B]
  const int32_t* layer_map;      // device [L_B]
  const bf16* aux_k; const bf16* aux_v;
  size_t aux_layer_elems;        // elements between the auxiliary layers' blocks (N * widest Ka)
  int Kb, Ka;
  int batch0;                    // first problem of this launch (2 * first base layer)
  __device__ const bf16* a_base(const bf16*, int batch) const {
    batch += batch0;
    int i = batch >> 1;
    return ((batch & 1) ? aux_v : aux_k) + (size_t)layer_map[i] * aux_layer_elems;
  }
  __device__ const bf16* row_ptr(int batch, int tn, int half, int r) const {
    int n = min(tn * BN + half * (BN / 2) + r, Kb - 1);
    return w_tab[batch + batch0] + (size_t)n * Ka;
  }
};
template <int BN>
struct EpiCachePair {
  typedef bf16 out_t;
  static constexpr int HALVES = 2;
  static constexpr bool PRELOAD = false;
  bf16* k_cache; bf16* v_cache;
  size_t layer_elems;            // B * n_kv_b * T_cap * hd
  int T_len; int64_t T_cap; int n_heads, hd, Kb;
  int batch0;
  __device__ void transform(int, int, int, const float (&v0)[4], const float (&v1)[4], bf16x4& o0, bf16x4& o1) const {
#pragma unroll
    for (int e = 0; e < 4; ++e) { o0[e] = (bf16)v0[e]; o1[e] = (bf16)v1[e]; }
  }
  __device__ void store(int batch, int m, int tn, int half, int p, const bf16x8& val) const {
    batch += batch0;
    int c = tn * BN + half * (BN / 2) + p;
    if (c >= Kb) return;           // Kb % 8 == 0 and hd % 8 == 0: a run of 8 stays inside one head
    bf16* cache = ((batch & 1) ? v_cache : k_cache) + (size_t)(batch >> 1) * layer_elems;
    int b = m / T_len, t = m % T_len;
    *reinterpret_cast<bf16x8*>(cache + (((size_t)b * n_heads + c / hd) * T_cap + t) * hd + c % hd) = val;
  }
};

template <class Tile, class BSrc, class Epi>
static void launch_gemm(const bf16* A, int lda, int M, int Nv, int K, int batches, BSrc bsrc, Epi epi, hipStream_t s) {
  auto kern = gemm_bf16_kernel<Tile, BSrc, Epi>;
  int tiles_m = (M + Tile::BM - 1) / Tile::BM, tiles_n = (Nv + Tile::BN - 1) / Tile::BN;
  int total = tiles_m * tiles_n;
  int grid_x = ((total + 7) / 8) * 8;
  // height (in row tiles) of the bands the tile walk proceeds in; 4 measured best (auxiliary stage -2.2 % at
  // 32768 x 2048-wide GEMMs against 8, 16 and 32 are 3-10 % worse): KVP_GROUP_M overrides for tuning
  static const int group_m = [] { const char* e = getenv("KVP_GROUP_M"); int v = e ? atoi(e) : 4; return v < 1 ? 1 : v; }();
  hipLaunchKernelGGL(kern, dim3(grid_x, batches), dim3(Tile::THREADS), 0, s, A, lda, M, K, tiles_m, tiles_n, group_m, bsrc, epi);
}

static int round_up(int v, int m) { return (v + m - 1) / m * m; }

typedef GemmTile<256, 256, 2, 4, 2> TileBig;     // 8 waves (two per SIMD), 128x64 per wave, 2 stages of 64 KB
typedef GemmTile<128, 128, 4, 2, 4> TileSmall;   // 8 waves, 32x64 per wave, 4 stages of 32 KB: one block per CU, deep pipeline
typedef GemmTile<128, 128, 4, 2, 2> TileSmall2;  // same tile, 2 stages: two blocks per CU, for grids larger than the chip
typedef GemmTile<128, 64, 4, 1, 3> TileNarrow;   // 4 waves, 32x64 per wave, 3 stages of 24 KB: two blocks per CU

// Tile choice: the biggest tile whose grid still fills the 256 CUs; small problems (few thousand
// tokens) are bound by how many K steps a block runs back to back, so they get smaller tiles,
// more blocks and a deeper load pipeline.
enum TileKind { TILE_BIG, TILE_SMALL, TILE_SMALL2, TILE_NARROW };
static TileKind pick_tile(int M, int Nv, bool narrow_ok, int batches = 1) {
  const char* force = getenv("KVP_GEMM_TILE");      // "big" / "small" / "narrow": for tests and tuning
  if (force && force[0] == 'b') return TILE_BIG;
  if (force && force[0] == 's') return (force[1] == '2') ? TILE_SMALL2 : TILE_SMALL;
  if (force && force[0] == 'n' && narrow_ok) return TILE_NARROW;
  long big = (long)((M + 255) / 256) * ((Nv + 255) / 256);
  if (big >= 384) return TILE_BIG;
  // Between half a round and one round of 256 x 256 tiles the big tile still wins: the four times as many
  // 128 x 128 tiles need two rounds of the chip's 512 slots, at a lower rate per CU, while the big tiles finish
  // in one (measured at 8192 tokens, d = 1536: O / down projections 101 -> 80 us per launch), and the CUs they
  // leave idle serve the base chain on the other stream.
  // The same holds between one and one and a half rounds (8192 tokens, 2560 virtual columns: the QKV projection of
  // a d = 1536 model): alone the big tile is 1 % slower there, but the CUs its short second round leaves idle take
  // the base chain's kernels, and the time to first token is 1.2 % shorter.
  const char* z = getenv("KVP_GEMM_ZONE");             // tuning: "0" 128 x 128 tiles below 1.5 rounds, "1" big tiles up to one round only
  const int zone = z ? z[0] - '0' : 2;
  if (zone >= 1 && big > 128 && big <= 256) return TILE_BIG;
  if (zone >= 2 && big > 256 && big < 384) return TILE_BIG;
  long small = (long)((M + 127) / 128) * ((Nv + 127) / 128);
  if (small * batches > 256) return TILE_SMALL2;
  if (small >= 200 || !narrow_ok) return TILE_SMALL;
  return TILE_NARROW;
}

void mfma_gemm_residual(const bf16* A, const bf16* W, float* X, int M, int N, int K, hipStream_t s) {
  switch (pick_tile(M, N, true)) {
    case TILE_BIG: launch_gemm<TileBig>(A, K, M, N, K, 1, BPlain<256>{W, N, K}, EpiResidualPair<256>{X, N}, s); break;
    case TILE_SMALL: launch_gemm<TileSmall>(A, K, M, N, K, 1, BPlain<128>{W, N, K}, EpiResidualPair<128>{X, N}, s); break;
    case TILE_SMALL2: launch_gemm<TileSmall2>(A, K, M, N, K, 1, BPlain<128>{W, N, K}, EpiResidualPair<128>{X, N}, s); break;
    default: launch_gemm<TileNarrow>(A, K, M, N, K, 1, BPlain<64>{W, N, K}, EpiResidualPair<64>{X, N}, s); break;
  }
}

void mfma_gemm_swiglu(const bf16* A, const bf16* Wg, const bf16* Wu, bf16* act, int M, int F, int K, hipStream_t s) {
  switch (pick_tile(M, 2 * F, true)) {
    case TILE_BIG: launch_gemm<TileBig>(A, K, M, 2 * F, K, 1, BGateUp<256>{Wg, Wu, F, K}, EpiSwiGLU<256>{act, F}, s); break;
    case TILE_SMALL: launch_gemm<TileSmall>(A, K, M, 2 * F, K, 1, BGateUp<128>{Wg, Wu, F, K}, EpiSwiGLU<128>{act, F}, s); break;
    case TILE_SMALL2: launch_gemm<TileSmall2>(A, K, M, 2 * F, K, 1, BGateUp<128>{Wg, Wu, F, K}, EpiSwiGLU<128>{act, F}, s); break;
    default: launch_gemm<TileNarrow>(A, K, M, 2 * F, K, 1, BGateUp<64>{Wg, Wu, F, K}, EpiSwiGLU<64>{act, F}, s); break;
  }
}

// vT[b][h][dim][t] = v[b*T + t][h*128 + dim]: 64 tokens x 128 dims per block through LDS, so that
// both the reads (256 B rows of v) and the writes (128 B runs along t) are coalesced.  Entries for
// t in [T, T_pad) are written as zero.
__global__ __launch_bounds__(256) void transpose_v_kernel(const bf16* __restrict__ v, bf16* __restrict__ vT, int T_len,
                                                          int T_pad, int n_kv) {
  __shared__ bf16 tile[64][128 + 2];
  const int t0 = blockIdx.x * 64, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  for (int c = tid; c < 64 * 16; c += 256) {
    int r = c / 16, ch = c % 16, t = t0 + r;
    bf16x8 val;
#pragma unroll
    for (int e = 0; e < 8; ++e) val[e] = (bf16)0.f;
    if (t < T_len) val = *reinterpret_cast<const bf16x8*>(v + ((size_t)b * T_len + t) * (n_kv * 128) + h * 128 + ch * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) tile[r][ch * 8 + e] = val[e];
  }
  __syncthreads();
  for (int c = tid; c < 128 * 8; c += 256) {
    int dim = c / 8, ch = c % 8;
    bf16x8 val;
#pragma unroll
    for (int e = 0; e < 8; ++e) val[e] = tile[ch * 8 + e][dim];
    *reinterpret_cast<bf16x8*>(vT + (((size_t)b * n_kv + h) * 128 + dim) * T_pad + t0 + ch * 8) = val;
  }
}

void mfma_qkv_rope(const bf16* hbuf, const bf16* wq, const bf16* wk, const bf16* wv, bf16* q, bf16* k, bf16* v, bf16* vT,
                   int N, int d, int n_q, int n_kv, int T_len, const float2* rope_tab, bool rotate, hipStream_t s) {
  int head0 = wq ? 0 : n_q;
  int heads = n_q + 2 * n_kv - head0;
  const int rot = rotate ? n_q + n_kv : 0;
  TileKind kind = pick_tile(N, heads * 128, false);
  if (kind == TILE_BIG && heads % 2 == 0)
    launch_gemm<TileBig>(hbuf, d, N, heads * 128, d, 1, BQKV<256>{wq, wk, wv, n_q, n_kv, head0, d},
                         EpiQKVRope<256>{q, k, v, n_q, n_kv, head0, T_len, rope_tab, rot}, s);
  else if (kind == TILE_SMALL2)
    launch_gemm<TileSmall2>(hbuf, d, N, heads * 128, d, 1, BQKV<128>{wq, wk, wv, n_q, n_kv, head0, d},
                            EpiQKVRope<128>{q, k, v, n_q, n_kv, head0, T_len, rope_tab, rot}, s);
  else
    launch_gemm<TileSmall>(hbuf, d, N, heads * 128, d, 1, BQKV<128>{wq, wk, wv, n_q, n_kv, head0, d},
                           EpiQKVRope<128>{q, k, v, n_q, n_kv, head0, T_len, rope_tab, rot}, s);
  if (vT) {
    int T_pad = round_up(T_len, 64), B = N / T_len;
    hipLaunchKernelGGL(transpose_v_kernel, dim3(T_pad / 64, n_kv, B), dim3(256), 0, s, v, vT, T_len, T_pad, n_kv);
  }
}

// =========================================================================================
// Causal grouped-query flash attention (head_dim 128), transposed-score formulation.
//
// A block owns one (sequence, kv head) and 32*SUB consecutive query positions for all G query
// heads of that kv head: wave w serves query head w % G and the 32-row query sub-tile w / G, so
// a K / V tile staged in LDS is shared by the whole group.  Eight (or six) waves per block put
// two waves on every SIMD: one wave's softmax arithmetic overlaps the other's MFMAs.
//
// Per 64-key tile a wave computes S^T = K Q^T (64 keys x 32 queries) so that a lane holds, for
// its query column, 32 of the 64 scores: the softmax row statistics need one cross-lane
// exchange only.  Then O^T += V^T P^T, where P^T goes from the score accumulators to the MFMA
// B operand without leaving registers: K rows are placed in LDS in an order (rows 4..7 and
// 8..11 of every 16 swapped) that makes the accumulator rows a lane holds exactly the 8
// consecutive keys the B operand wants.  V is read from a transposed copy ([dim][token]) so
// that its fragments are contiguous along keys.  Tiles go global -> LDS directly (no register
// staging), double buffered: tile j+1 is in flight while tile j is consumed.
// =========================================================================================
constexpr int FA_KT = 64;                          // keys per tile
constexpr int FA_STAGE = FA_KT * 128 * 2;          // elements per stage: K tile + V^T tile

// K tile: 64 rows of 256 B (16 chunks); V^T tile: 128 rows of 128 B (8 chunks).  64-bank LDS:
// 16 lanes of a 16-byte read are served per cycle, so 16 consecutive rows of one logical chunk
// must land in 16 distinct 16-byte units.
__device__ __forceinline__ int k_swz(int row, int chunk) { return row * 128 + ((chunk ^ (row & 15)) << 3); }
__device__ __forceinline__ int v_swz(int row, int chunk) { return row * 64 + ((chunk ^ ((row >> 1) & 7)) << 3); }
__device__ __forceinline__ int perm16(int r) {      // swap rows 4..7 with 8..11 inside each 16
  int q = (r >> 2) & 3;
  int nq = (q == 1) ? 2 : (q == 2 ? 1 : q);
  return (r & ~12) | (nq << 2);
}

template <int NW>
__global__ __launch_bounds__(NW * 64) void flash_prefill_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k,
                                                                const bf16* __restrict__ vT, bf16* __restrict__ out,
                                                                int T_len, int T_pad, int n_q, int n_kv, int G,
                                                                float c_log2, float guard) {
  __shared__ __attribute__((aligned(1024))) bf16 stage0[FA_STAGE];
  __shared__ __attribute__((aligned(1024))) bf16 stage1[FA_STAGE];

  const int SUB = NW / G;
  const int QB = 32 * SUB;
  const int n_qt = (T_len + QB - 1) / QB;
  // One-dimensional grid, (sequence, kv head) group fastest and query tiles from the last (most
  // key tiles) to the first: the long blocks of every group start first and the short ones fill
  // the tail (with the query tile fastest, the last group's long blocks start late and a fifth of
  // the chip idles at the end).
  const int n_groups = (int)gridDim.x / n_qt;         // = n_kv * batch
  const int grp = blockIdx.x % n_groups;
  const int qt = n_qt - 1 - blockIdx.x / n_groups;
  const int hk = grp % n_kv, b = grp / n_kv;
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int l32 = lane % 32, g = lane / 32;
  const int hq = hk * G + wave % G;
  const int q_lo = qt * QB + (wave / G) * 32;         // first query position of this wave
  const int q_block_hi = min(T_len, (qt + 1) * QB) - 1;
  const int n_tiles = q_block_hi / FA_KT + 1;
  const int ldq = n_q * 128, ldk = n_kv * 128;

  // Q^T fragments: lane holds query row (q_lo + l32), dims 16 ks + 8 g .. + 7
  bf16x8 qf[8];
  {
    int pos = min(q_lo + l32, T_len - 1);
    const bf16* qr = q + ((size_t)b * T_len + pos) * ldq + (size_t)hq * 128 + g * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qr + ks * 16);
  }

  f32x16 acc_o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc_o[dt][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const bf16* kbase = k + (size_t)b * T_len * ldk + (size_t)hk * 128;
  const bf16* vbase = vT + ((size_t)b * n_kv + hk) * 128 * (size_t)T_pad;

  // Direct-to-LDS staging.  One wave instruction fills 1024 contiguous bytes of a stage:
  //   K part: 4 LDS rows of 256 B; lane l -> LDS row rho = 4*i + l/16, physical chunk l%16; that
  //           slot holds key perm16(rho), logical chunk (l%16) ^ (rho & 15).
  //   V part: 8 LDS rows of 128 B; lane l -> dim row 8*i + l/8, physical chunk l%8, logical chunk
  //           (l%8) ^ ((row/2) & 7) = keys 8*chunk .. +7 of the tile.
  // The 16 K instructions and 16 V instructions of a tile are dealt round-robin to the waves.
  auto issue_tile = [&](bf16* st, int tile) {
    const int kv0 = tile * FA_KT;
    for (int i = wave; i < 32; i += NW) {
      if (i < 16) {
        int rho = 4 * i + lane / 16;
        int ch = (lane % 16) ^ (rho & 15);
        int key = min(kv0 + perm16(rho), T_len - 1);
        load_lds16(kbase + (size_t)key * ldk + ch * 8, st + i * 512);
      } else {
        int j = i - 16;
        int row = 8 * j + lane / 8;
        int ch = (lane % 8) ^ ((row >> 1) & 7);
        load_lds16(vbase + (size_t)row * T_pad + kv0 + ch * 8, st + FA_KT * 128 + j * 512);
      }
    }
  };

  issue_tile(stage0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  __syncthreads();

  for (int tile = 0; tile < n_tiles; ++tile) {
    const bf16* st = (tile & 1) ? stage1 : stage0;
    bf16* nst = (tile & 1) ? stage0 : stage1;
    if (tile + 1 < n_tiles) issue_tile(nst, tile + 1);
    const int kv0 = tile * FA_KT;
    if (kv0 <= q_lo + 31 && q_lo < T_len) {          // wave-uniform: tile has unmasked keys for this wave
      // ---- S^T = K Q^T ----  all 16 key fragments are fetched from LDS before the first MFMA so
      // the matrix core never waits on an LDS round trip in the middle of the chain
      f32x16 sacc[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[kt][i] = 0.f;
      // All 16 fragments of a chain are fetched before its first MFMA (FB < 16 fetches them in
      // batches: fewer registers, but measured slower even at three waves per SIMD).
      constexpr int FB = 16;
      bf16x8 fr[FB];
#pragma unroll
      for (int f0 = 0; f0 < 16; f0 += FB) {
#pragma unroll
        for (int f = 0; f < FB; ++f) {
          const int ks = (f0 + f) / 2, kt = (f0 + f) % 2;
          fr[f] = *reinterpret_cast<const bf16x8*>(st + k_swz(kt * 32 + l32, ks * 2 + g));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < FB; ++f) {
          const int ks = (f0 + f) / 2, kt = (f0 + f) % 2;
          sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[f], qf[ks], sacc[kt], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      // the first value fragments are fetched now and land while the softmax arithmetic runs
#pragma unroll
      for (int f = 0; f < FB; ++f) {
        const int kk = f / 4, dt = f % 4;
        fr[f] = *reinterpret_cast<const bf16x8*>(st + FA_KT * 128 + v_swz(dt * 32 + l32, kk * 2 + g));
      }
      __builtin_amdgcn_sched_barrier(0);
      // accumulator element i of key tile kt is key kv0 + 32 kt + 16 (i/8) + 8 g + i%8
      const int qpos = q_lo + l32;
      if (kv0 + FA_KT - 1 > q_lo) {                  // diagonal tile: some key may exceed some query
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            int key = kv0 + 32 * kt + 16 * (i / 8) + 8 * g + (i % 8);
            if (key > qpos) sacc[kt][i] = -INFINITY;
          }
      }
      // Softmax against a FIXED reference per query row.  exp(s - m) / sum exp(s - m) does not depend on m,
      // and in floating point a poor m costs no precision (bf16 and float32 share one exponent range, and
      // every product is scaled by the same factor), only range.  So the reference is the row maximum
      // of the FIRST key tile (finite: key 0 precedes every query), and later tiles skip the search
      // for their maximum -- a third of the softmax's vector instructions, which the matrix pipe does not
      // hide (measured: -7 % kernel time at 8192 tokens, -12 % at 2048).  Range is watched by a guard
      // instead: if a lane's sum of the tile's probabilities exceeds `guard` (2^20 by default; infinities
      // and NaNs fail the comparison too), the wave raises the reference of its rows to the tile's true
      // maximum, rescales what it has accumulated and recomputes the tile.  Scores far BELOW the reference
      // underflow to zero, which is what their weight is next to the key that set it.
      auto row_max = [&]() {
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 32; ++e) mx = fmaxf(mx, sacc[e / 16][e % 16]);
        return fmaxf(mx, __shfl_xor(mx, 32, 64));
      };
      auto move_reference = [&](float m_new) {       // m_new >= m_run: rescale what has been accumulated
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2);
        l_run *= alpha;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc_o[dt][i] *= alpha;
      };
      float psum;
      bf16x8 pf[4];
      auto exps = [&]() {
        const float mc = m_run * c_log2;
        psum = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int sgrp = 0; sgrp < 2; ++sgrp) {
            bf16x8 pk;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              float pv = __builtin_amdgcn_exp2f(sacc[kt][sgrp * 8 + e] * c_log2 - mc);
              psum += pv;
              pk[e] = (bf16)pv;
            }
            pf[kt * 2 + sgrp] = pk;
          }
      };
      if (tile == 0) move_reference(row_max());
      exps();
      if (tile > 0 && __builtin_amdgcn_ballot_w64(!(psum <= guard)) != 0) {   // wave-uniform, rare
        move_reference(fmaxf(m_run, row_max()));
        exps();
      }
      l_run += psum;
      // ---- O^T += V^T P^T ----
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int f0 = 0; f0 < 16; f0 += FB) {
        if (f0 > 0) {
#pragma unroll
          for (int f = 0; f < FB; ++f) {
            const int kk = (f0 + f) / 4, dt = (f0 + f) % 4;
            fr[f] = *reinterpret_cast<const bf16x8*>(st + FA_KT * 128 + v_swz(dt * 32 + l32, kk * 2 + g));
          }
        }
#pragma unroll
        for (int f = 0; f < FB; ++f) {
          const int kk = (f0 + f) / 4, dt = (f0 + f) % 4;
          acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[f], pf[kk], acc_o[dt], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's share of the next tile has landed
    __syncthreads();
  }

  // O^T accumulator element i of dim tile dt: dim 32 dt + 8 (i/4) + 4 g + i%4, query column l32
  const int qpos = q_lo + l32;
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qpos < T_len) {
    const float inv = 1.f / l_tot;
    bf16* orow = out + ((size_t)b * T_len + qpos) * ldq + (size_t)hq * 128;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int iq = 0; iq < 4; ++iq) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (bf16)(acc_o[dt][iq * 4 + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + dt * 32 + iq * 8 + g * 4) = o4;
      }
  }
}

}  // namespace kvp
#include "flash2.h"
namespace kvp {

// Overflow guard of the attention kernels' fixed-reference softmax (see flash_prefill_kernel): the largest sum
// of a tile's probabilities a lane accepts before its wave re-references the tile.  kvp_debug_flash_guard sets
// it for the process (tests force the re-referencing path with a tiny value); 0 restores the default.
static float g_flash_guard = 0.f;
void mfma_set_flash_guard(float limit) { g_flash_guard = limit; }
static float flash_guard() { return g_flash_guard > 0.f ? g_flash_guard : 1048576.f; }

static int flash_waves(int G) {
  switch (G) {
    case 1: case 2: case 4: case 8: return 8;
    case 3: case 6: return 6;
    default: return 0;
  }
}

template <int NW>
static void launch_flash(const bf16* q, const bf16* k, const bf16* vT, bf16* out, int B, int T_len, int n_q, int n_kv,
                         hipStream_t s) {
  int G = n_q / n_kv, QB = 32 * (NW / G);
  int n_qt = (T_len + QB - 1) / QB;
  float c_log2 = 1.4426950408889634f / sqrtf(128.f);
  hipLaunchKernelGGL(flash_prefill_kernel<NW>, dim3(n_qt * n_kv * B, 1, 1), dim3(NW * 64), 0, s, q, k, vT, out, T_len,
                     round_up(T_len, 64), n_q, n_kv, G, c_log2, flash_guard());
}

void mfma_flash_prefill(const bf16* q, const bf16* k, const bf16* vT, bf16* out, int B, int T_len, int n_q, int n_kv,
                        hipStream_t s) {
  const int G = n_q / n_kv;
  const char* v1 = getenv("KVP_FLASH_V1");           // "1": the unpipelined kernel for every group size
  if ((G == 3 || G == 4 || G == 6 || G == 8) && !(v1 && v1[0] == '1')) {
    int subs = (G <= 4) ? 2 : 1;
    // few blocks (short prompts, one or two sequences): the kernel's time is its longest block,
    // a chain of key tiles; 32-row blocks give every active wave a SIMD of its own
    if (subs == 2 && ((T_len + 63) / 64) * n_kv * B <= 256) subs = 1;   // (measured crossover: one block per CU)
    const char* fs = getenv("KVP_FLASH_SUBS");         // "1" / "2": tuning override (G = 3, 4 only)
    if (fs && G <= 4 && (fs[0] == '1' || fs[0] == '2')) subs = fs[0] - '0';
    const int QB = 32 * subs;
    const float c_log2 = 1.4426950408889634f / sqrtf(128.f);
    hipLaunchKernelGGL(flash_prefill2_kernel, dim3(((T_len + QB - 1) / QB) * n_kv * B, 1, 1), dim3(F2_WAVES * 64), 0, s,
                       q, k, vT, out, T_len, round_up(T_len, 64), n_q, n_kv, G, subs, c_log2, flash_guard());
    return;
  }
  switch (flash_waves(G)) {
    case 6: launch_flash<6>(q, k, vT, out, B, T_len, n_q, n_kv, s); break;
    case 8: launch_flash<8>(q, k, vT, out, B, T_len, n_q, n_kv, s); break;
    default: break;
  }
}

size_t mfma_vt_bytes_shape(const kvp_model_shape* m, int B, int T_len) {
  return (size_t)B * m->n_kv_heads * 128 * (size_t)round_up(T_len, 64) * sizeof(bf16);
}
size_t mfma_vt_bytes(const kvp_config* cfg, int B, int T_len) { return mfma_vt_bytes_shape(&cfg->aux, B, T_len); }

// =========================================================================================
// Support check, per-handle tables, predictor launch
// =========================================================================================
bool mfma_shape_supported(const kvp_model_shape* m) {
  if (m->head_dim != 128) return false;
  if (m->d_model % 64 || m->ffn_dim % 64) return false;
  if (flash_waves(m->n_q_heads / m->n_kv_heads) == 0) return false;
  return true;
}
bool mfma_supported(const kvp_config* cfg) { return mfma_shape_supported(&cfg->aux); }

int mfma_prepare(kvp_handle* h, void** tables_out) {
  *tables_out = nullptr;
  const kvp_config& c = handle_cfg(h);
  int L = c.base.n_layers;
  MfmaTables* t = new MfmaTables();
  std::vector<const void*> w(2 * L);
  for (int i = 0; i < L; ++i) { w[2 * i] = handle_pred_wk(h)[i]; w[2 * i + 1] = handle_pred_wv(h)[i]; }
  hipError_t e = hipMalloc((void**)&t->w_tab, 2 * L * sizeof(void*));
  if (e == hipSuccess) e = hipMalloc((void**)&t->layer_map, L * sizeof(int32_t));
  if (e == hipSuccess) e = hipMemcpy(t->w_tab, w.data(), 2 * L * sizeof(void*), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(t->layer_map, handle_layer_map(h).data(), L * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    mfma_release(t);
    return KVP_ERR_HIP;
  }
  *tables_out = t;
  return KVP_OK;
}

void mfma_release(void* tables) {
  MfmaTables* t = static_cast<MfmaTables*>(tables);
  if (!t) return;
  if (t->w_tab) (void)hipFree(t->w_tab);
  if (t->layer_map) (void)hipFree(t->layer_map);
  delete t;
}

bool mfma_predictor_supported(const kvp_config* cfg) {
  return cfg->dtype == KVP_DTYPE_BF16 && (cfg->aux.n_kv_heads * cfg->aux.head_dim) % 64 == 0;
}

int mfma_predictor(const kvp_handle* h, void* tables, const bf16* aux_k, const bf16* aux_v, bf16* k_cache, bf16* v_cache,
                   int B, int T_len, int64_t T_cap, int layer0, int layer1, int Ka, int Kb, int n_kv_b, size_t aux_block,
                   size_t layer_elems, hipStream_t s) {
  const kvp_config& c = handle_cfg(h);
  MfmaTables* t = static_cast<MfmaTables*>(tables);
  int N = B * T_len;
  const int batches = 2 * (layer1 - layer0), batch0 = 2 * layer0;
  if (batches <= 0) return KVP_OK;
  if (mfma_predictor_stream(h, tables, aux_k, aux_v, k_cache, v_cache, B, T_len, T_cap, layer0, layer1, Ka, Kb, n_kv_b,
                            aux_block, layer_elems, s))
    return KVP_OK;
  const char* ptile = getenv("KVP_PRED_TILE");   // "big" / "small" / "s2": tuning override
  // K = Ka is only 256..512 deep, so a tile is mostly prologue and epilogue (the cache write);
  // 128x128 tiles with two blocks per CU let one block's write overlap the other's MFMAs
  // (measured: 0.89 ms vs 1.09 ms for 256x256 tiles at B x T = 8 x 4096).
  int kind = 2;                                   // 0 big, 1 small (4 stages), 2 small (2 stages)
  if (ptile && ptile[0] == 'b') kind = 0;
  if (ptile && ptile[0] == 's') kind = (ptile[1] == '2') ? 2 : 1;
  if (kind == 0)
    launch_gemm<TileBig>(nullptr, Ka, N, Kb, Ka, batches,
                         BPredictor<256>{t->w_tab, t->layer_map, aux_k, aux_v, aux_block, Kb, Ka, batch0},
                         EpiCachePair<256>{k_cache, v_cache, layer_elems, T_len, T_cap, n_kv_b, c.base.head_dim, Kb, batch0}, s);
  else if (kind == 1)
    launch_gemm<TileSmall>(nullptr, Ka, N, Kb, Ka, batches,
                           BPredictor<128>{t->w_tab, t->layer_map, aux_k, aux_v, aux_block, Kb, Ka, batch0},
                           EpiCachePair<128>{k_cache, v_cache, layer_elems, T_len, T_cap, n_kv_b, c.base.head_dim, Kb, batch0}, s);
  else
    launch_gemm<TileSmall2>(nullptr, Ka, N, Kb, Ka, batches,
                            BPredictor<128>{t->w_tab, t->layer_map, aux_k, aux_v, aux_block, Kb, Ka, batch0},
                            EpiCachePair<128>{k_cache, v_cache, layer_elems, T_len, T_cap, n_kv_b, c.base.head_dim, Kb, batch0}, s);
  return KVP_OK;
}

}  // namespace kvp
