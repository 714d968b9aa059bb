// bf16 MFMA GEMM for gfx950:  C[M, Nv] = A[M, K] * Bv[Nv, K]^T  with float32 accumulation,
// where the "virtual" weight rows Bv and the destination of every output element are
// supplied by small functors, so one kernel serves the QKV (+rotary), O/down (+residual),
// gate/up (+SiLU*mul) and predictor (+cache scatter) projections.
//
// Tiling.  A block computes a BM x BN tile with WM x WN wavefronts; K advances in tiles of 64.
// Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4, no register
// staging) as rows of 64 bf16 (128 B) whose eight 16-byte chunks are XOR-swizzled with the row
// index so that the MFMA fragment reads are bank-conflict free.  NS stages form a ring: the
// prologue requests NS tiles, every K tile requests tile kt + NS into the stage it has just
// freed, and waits (explicit vmcnt) only for tile kt + 1.  Fragments are double buffered in
// registers, so the LDS reads of a sub-step ride behind the MFMAs of the one before.
//
// Column pairing.  The BN virtual columns of a block are two halves of BN/2; a wavefront
// owns the same column positions in both halves, so the epilogue sees, in one lane, output p
// of half 0 together with output p of half 1.  The rotary epilogue makes the halves the two
// halves of a head's dimensions, the SwiGLU epilogue makes them gate and up, plain epilogues
// just treat them as adjacent column ranges.
//
// MFMA: v_mfma_f32_32x32x16_bf16.  Fragment layout (64 lanes, g = lane / 32, r = lane % 32):
//   A fragment: row r,      k = 8g .. 8g+7        B fragment: column r, k = 8g .. 8g+7
//   C fragment: column r,   rows 8*(i/4) + 4g + i%4 for i = 0..15
// The kernel feeds weight rows as "A" and activation rows as "B", i.e. accumulates C^T.
#pragma once
#include <type_traits>

#include "common.h"

namespace kvp {

constexpr int GEMM_BK = 64;

template <int BM_, int BN_, int WM_, int WN_, int NS_>
struct GemmTile {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int NS = NS_;                 // LDS stages (K tiles resident or in flight)
  static constexpr int THREADS = 64 * WM * WN;
  static constexpr int RT = BM / WM / 32;        // 32-row tiles per wave
  static constexpr int CT = BN / WN / 32;        // 32-column tiles per wave (half from each column half)
  static constexpr int LA = BM * 8 / THREADS;    // 16-byte chunks of A staged per thread per step
  static constexpr int LB = BN * 8 / THREADS;
  static constexpr int STAGE_ELEMS = (BM + BN) * GEMM_BK;
  static_assert(CT % 2 == 0 && RT >= 1, "wave tile must hold column pairs");
  static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "staging must divide evenly");
  static_assert((BN / 2) % (THREADS / 8) == 0, "one staging pass must not straddle the column halves");
};

// LDS has 64 banks of 4 bytes: a 16-byte-per-lane read is served 16 lanes (256 B) per cycle.
// Rows are 128 B, so two consecutive rows span the banks once; XOR-ing the chunk index with
// (row / 2) % 8 makes any 16 consecutive rows of one logical chunk hit 16 distinct 16-byte units.
__device__ __forceinline__ int swz_key(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int swz(int row, int chunk) { return row * GEMM_BK + ((chunk ^ swz_key(row)) << 3); }

// XCD-aware tile order: consecutive blocks go to different XCDs (8 of them, each with its own
// L2), so give every XCD a contiguous range of the tile sequence, and walk that sequence in
// bands of GROUP_M row tiles so a band's A panels and the B panels stay L2 resident (the 32 tiles
// an XCD works on at a time then form a GROUP_M x 32 / GROUP_M patch; the launcher passes 4).
__device__ __forceinline__ bool tile_coords(int tiles_m, int tiles_n, int GROUP_M, int& tm, int& tn) {
  constexpr int XCD = 8;
  int total = tiles_m * tiles_n;
  int per = (total + XCD - 1) / XCD;
  int bid = blockIdx.x;
  int logical = (bid % XCD) * per + bid / XCD;
  if (logical >= total) return false;
  int band = GROUP_M * tiles_n;
  int first_m = (logical / band) * GROUP_M;
  int gsz = min(tiles_m - first_m, GROUP_M);
  int in_band = logical % band;
  tm = first_m + in_band % gsz;
  tn = in_band / gsz;
  return true;
}

// One wave-level direct global->LDS load: lane l's 16 bytes land at lds_base + 16*l (lds_base is
// wave-uniform).  Written as inline assembly on purpose.  Issued through the compiler builtin,
// the load is tracked as a store to LDS that later LDS reads may alias, and the compiler then
// makes fragment reads wait for ALL outstanding loads (vmcnt(0)), which serialises any pipeline
// deeper than two stages.  The kernels track completion themselves with explicit s_waitcnt.
__device__ __forceinline__ void load_lds16(const bf16* src, bf16* lds_base) {
  uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) bf16*)lds_base);
  asm volatile("" : "+s"(lds_addr));   // a register even when the address is a link-time constant
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(src) : "memory");
}

template <class Tile, class BSrc, class Epi>
__global__ __launch_bounds__(Tile::THREADS) void gemm_bf16_kernel(const bf16* __restrict__ A, int lda, int M, int K,
                                                                  int tiles_m, int tiles_n, int group_m, BSrc bsrc, Epi epi) {
  constexpr int BM = Tile::BM, BN = Tile::BN, RT = Tile::RT, CT = Tile::CT;
  constexpr int NWAVES = Tile::WM * Tile::WN;
  constexpr int GA = BM / 8 / NWAVES;     // 8-row groups of the A tile loaded by each wave per step
  constexpr int GB = BN / 8 / NWAVES;
  static_assert(BM % (8 * NWAVES) == 0 && BN % (8 * NWAVES) == 0, "row groups must divide among waves");
  static_assert((BN / 2) % 8 == 0, "a row group must not straddle the column halves");
  constexpr int NS = Tile::NS;
  __shared__ __attribute__((aligned(1024))) bf16 stages[NS * Tile::STAGE_ELEMS];

  int tm, tn;
  if (!tile_coords(tiles_m, tiles_n, group_m, tm, tn)) return;
  const int batch = blockIdx.y;
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int wm = wave / Tile::WN, wn = wave % Tile::WN;
  const int l32 = lane % 32, g = lane / 32;
  const int m0 = tm * BM;

  // Direct-to-LDS staging: one wave instruction fills 8 rows x 128 B of a stage; lane l supplies
  // row l/8, physical chunk l%8, i.e. the logical chunk (l%8) ^ swz_key(row) of that row.
  const bf16* a_src[GA];
  const bf16* b_src[GB];
  const bf16* Ab = bsrc.a_base(A, batch);
#pragma unroll
  for (int i = 0; i < GA; ++i) {
    int row = (i * NWAVES + wave) * 8 + lane / 8;
    int ch = (lane % 8) ^ swz_key(row);
    a_src[i] = Ab + (size_t)min(m0 + row, M - 1) * lda + ch * 8;
  }
#pragma unroll
  for (int i = 0; i < GB; ++i) {
    int row = (i * NWAVES + wave) * 8 + lane / 8;
    int ch = (lane % 8) ^ swz_key(row);
    b_src[i] = bsrc.row_ptr(batch, tn, row / (BN / 2), row % (BN / 2)) + ch * 8;
  }
  auto issue_loads = [&](bf16* st, int kt) {
    const int koff = kt * GEMM_BK;
#pragma unroll
    for (int i = 0; i < GA; ++i) load_lds16(a_src[i] + koff, st + (i * NWAVES + wave) * 8 * GEMM_BK);
#pragma unroll
    for (int i = 0; i < GB; ++i) load_lds16(b_src[i] + koff, st + BM * GEMM_BK + (i * NWAVES + wave) * 8 * GEMM_BK);
  };

  f32x16 acc[RT][CT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rt][ct][i] = 0.f;

  // fragment read rows inside a stage
  int a_row[RT], b_row[CT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) a_row[rt] = (wm * RT + rt) * 32 + l32;
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    int half = ct / (CT / 2), t = ct % (CT / 2);
    b_row[ct] = half * (BN / 2) + (wn * (CT / 2) + t) * 32 + l32;
  }

  // Software pipeline.  Fragments live in two register sets; while the MFMAs of sub-step ks run
  // from one set, the LDS reads of sub-step ks+1 fill the other, and the direct-to-LDS loads of
  // the next K tile are issued between the MFMAs of the first sub-steps.  The block barrier
  // sits between sub-steps 2 and 3: by then every wave has read its last fragments of the
  // current stage, so sub-step 3 (registers only) overlaps the next stage's first LDS reads.
  constexpr int KS = GEMM_BK / 16;
  constexpr int MF = RT * CT, RD = RT + CT;
  bf16x8 af[2][RT], bfr[2][CT];
  auto read_frag = [&](const bf16* st, int ks, int set, int i) {
    if (i < RT) af[set][i] = *reinterpret_cast<const bf16x8*>(st + swz(a_row[i], ks * 2 + g));
    else bfr[set][i - RT] = *reinterpret_cast<const bf16x8*>(st + BM * GEMM_BK + swz(b_row[i - RT], ks * 2 + g));
  };
  auto issue_one = [&](bf16* st, int koff, int i) {
    if (i < GA) load_lds16(a_src[i] + koff, st + (i * NWAVES + wave) * 8 * GEMM_BK);
    else load_lds16(b_src[i - GA] + koff, st + BM * GEMM_BK + ((i - GA) * NWAVES + wave) * 8 * GEMM_BK);
  };

  // vmcnt immediate for "at most X of this wave's loads still outstanding" (and lgkmcnt(0))
  constexpr int G_LOADS = GA + GB;                       // loads per wave per K tile
  constexpr int X_STEADY = (NS - 2) * G_LOADS;           // newer tiles that may still be in flight
  static_assert(X_STEADY <= 63, "vmcnt is a 6-bit counter");
  constexpr int WAIT_STEADY = (X_STEADY & 15) | ((X_STEADY >> 4) << 14) | 0x0070;
  constexpr int X_PRO = (NS - 1) * G_LOADS;
  static_assert(X_PRO <= 63, "vmcnt is a 6-bit counter");
  constexpr int WAIT_PRO = (X_PRO & 15) | ((X_PRO >> 4) << 14) | 0x0F70;

  const int KT = K / GEMM_BK;
#pragma unroll
  for (int t = 0; t < NS; ++t)
    if (t < KT) issue_loads(stages + t * Tile::STAGE_ELEMS, t);
  if (KT >= NS) __builtin_amdgcn_s_waitcnt(WAIT_PRO);    // tile 0 landed, tiles 1..NS-1 may be in flight
  else __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0)
  __syncthreads();
#pragma unroll
  for (int i = 0; i < RD; ++i) read_frag(stages, 0, 0, i);

  // K tile kt (stage kt % NS): sub-steps 0..KS-2 read their successors' fragments from the current
  // stage; then the barrier (tile kt+1 has landed for every wave, nobody reads the current stage
  // any more); the last sub-step runs from registers while the first fragments of tile kt+1 are
  // read and the loads of tile kt+NS are issued into the stage just freed.
  auto k_step = [&](int kt, auto next_c, auto load_c) {
    constexpr bool has_next = decltype(next_c)::value, has_load = decltype(load_c)::value;
    bf16* cur = stages + (kt % NS) * Tile::STAGE_ELEMS;
    const bf16* nxt = stages + ((kt + 1) % NS) * Tile::STAGE_ELEMS;
    const int koff = (kt + NS) * GEMM_BK;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int set = ks & 1;
      if (ks == KS - 1) {
        // tile kt+1 was issued NS-1 steps ago; in the steady state NS-2 younger tiles may still be in
        // flight, near the end of K fewer are, so wait for everything there
        // (both immediates also carry lgkmcnt(0): this wave's reads of the current stage are complete.
        // A bare barrier, not __syncthreads(): its fence would add a vmcnt(0) and drain the pipeline.)
        if (has_load || NS == 2) __builtin_amdgcn_s_waitcnt(WAIT_STEADY);
        else __builtin_amdgcn_s_waitcnt(0x0070);
        __builtin_amdgcn_s_barrier();
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < MF; ++j) {
        acc[j / CT][j % CT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][j % CT], af[set][j / CT], acc[j / CT][j % CT], 0, 0, 0);
        {
          constexpr int RPER = (RD + MF - 1) / MF;    // fragment reads riding behind each MFMA
#pragma unroll
          for (int u = 0; u < RPER; ++u) {
            const int fi = j * RPER + u;
            if (fi < RD) {
              if (ks + 1 < KS) read_frag(cur, ks + 1, set ^ 1, fi);
              else if (has_next) read_frag(nxt, 0, set ^ 1, fi);
            }
          }
        }
        if (has_load && ks == KS - 1) {
          constexpr int PER = (GA + GB + MF - 1) / MF;
#pragma unroll
          for (int u = 0; u < PER; ++u) {
            int idx = j * PER + u;
            if (idx < GA + GB) issue_one(cur, koff, idx);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  int kt = 0;
  for (; kt < KT - NS; ++kt) k_step(kt, std::true_type{}, std::true_type{});
  for (; kt < KT - 1; ++kt) k_step(kt, std::true_type{}, std::false_type{});
  k_step(KT - 1, std::false_type{}, std::false_type{});

  // Epilogue.  The weight fragment is the MFMA "A" operand and the activation fragment the "B"
  // operand, so an accumulator holds C^T: a lane owns ONE output row (lane%32 of a 32-row tile)
  // and, per group of four accumulator registers, FOUR CONSECUTIVE output columns, from column
  // half 0 and from the same position in half 1.  The functor first turns those into output
  // values (rotary, SiLU*mul, plain), which are staged in this wave's share of the - now idle -
  // operand LDS, one 32-row tile at a time; the tile is then read back row-contiguously so that
  // every lane hands the functor 16 contiguous output bytes of one row and a wave store
  // instruction covers whole cache lines.
  typedef typename Epi::out_t out_t;
  constexpr int HV = Epi::HALVES;                       // staged halves per position (SwiGLU folds two into one)
  constexpr int W = (CT / 2) * 32;                      // positions per half owned by this wave
  constexpr int VEC = 16 / (int)sizeof(out_t);          // outputs per 16-byte run
  constexpr int ROW_ELEMS = HV * W + VEC;               // + 16 bytes: spreads the 32 rows over the banks
  constexpr int WAVE_LDS_BYTES = NS * Tile::STAGE_ELEMS * (int)sizeof(bf16) / NWAVES;
  // rows staged at once: a whole 32-row tile if it fits the wave's LDS share, else two halves of 16
  constexpr int SROWS = (32 * ROW_ELEMS * (int)sizeof(out_t) <= WAVE_LDS_BYTES) ? 32 : 16;
  static_assert(SROWS * ROW_ELEMS * (int)sizeof(out_t) <= WAVE_LDS_BYTES, "staging tile must fit the wave's LDS share");
  __syncthreads();                                      // every wave is done with the operand stages
  out_t* wl = reinterpret_cast<out_t*>(reinterpret_cast<char*>(stages) + wave * WAVE_LDS_BYTES);
  typedef out_t vec4_t __attribute__((ext_vector_type(4)));
  typedef out_t vecr_t __attribute__((ext_vector_type(VEC)));
  constexpr int LPROW = HV * W / VEC;                   // lanes covering one staged row
  constexpr int ROWS_PER_IT = 64 / LPROW;
  static_assert(LPROW <= 64 && 64 % LPROW == 0 && SROWS % ROWS_PER_IT == 0, "a staged row must divide the wave");
  // An epilogue that adds into memory (Epi::PRELOAD) gets the old contents of the NEXT staged
  // unit requested before the current unit is transformed, staged and stored: otherwise every
  // 16-byte read-modify-write would wait a full memory round trip behind the store before it.
  constexpr int NPASS = 32 / SROWS, NIT = SROWS / ROWS_PER_IT, NUNIT = RT * NPASS;
  vecr_t xnext[NIT];
  auto preload = [&](int unit) {
    if constexpr (Epi::PRELOAD) {
      const int rt = unit / NPASS, pass = unit % NPASS;
      const int mrow0 = m0 + (wm * RT + rt) * 32;
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int row = it * ROWS_PER_IT + lane / LPROW;
        const int seg = lane % LPROW;
        const int half = seg / (W / VEC), pl = (seg % (W / VEC)) * VEC;
        const int mm = min(mrow0 + pass * SROWS + row, M - 1);
        xnext[it] = epi.load(batch, mm, tn, half, wn * W + pl);
      }
    }
  };
  preload(0);
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int mrow0 = m0 + (wm * RT + rt) * 32;
    const int m = min(mrow0 + l32, M - 1);              // rows past M are staged but never stored
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      vecr_t xcur[NIT];
      if constexpr (Epi::PRELOAD) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) xcur[it] = xnext[it];
        if (rt * NPASS + pass + 1 < NUNIT) preload(rt * NPASS + pass + 1);
      }
      const bool mine = (SROWS == 32) || (l32 / SROWS == pass);
      const int srow = l32 % SROWS;
#pragma unroll
      for (int t = 0; t < CT / 2; ++t)
#pragma unroll
        for (int iq = 0; iq < 4; ++iq) {
          const int pl = t * 32 + iq * 8 + g * 4;
          float v0[4], v1[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) { v0[e] = acc[rt][t][iq * 4 + e]; v1[e] = acc[rt][t + CT / 2][iq * 4 + e]; }
          if (mine) {
            vec4_t o0, o1;
            epi.transform(m, tn, wn * W + pl, v0, v1, o0, o1);
            *reinterpret_cast<vec4_t*>(wl + srow * ROW_ELEMS + pl) = o0;
            if (HV == 2) *reinterpret_cast<vec4_t*>(wl + srow * ROW_ELEMS + W + pl) = o1;
          }
        }
      // The staging region belongs to this wave alone and its LDS operations execute in program
      // order, so no block barrier is needed between the lanes' writes and the other lanes'
      // reads; the wavefront-scope fences (no instruction) keep the compiler from reordering them.
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int row = it * ROWS_PER_IT + lane / LPROW;
        const int seg = lane % LPROW;
        const int half = seg / (W / VEC), pl = (seg % (W / VEC)) * VEC;
        vecr_t v = *reinterpret_cast<const vecr_t*>(wl + row * ROW_ELEMS + half * W + pl);
        const int mm = mrow0 + pass * SROWS + row;
        if constexpr (Epi::PRELOAD) {
          if (mm < M) epi.store(batch, mm, tn, half, wn * W + pl, v + xcur[it]);
        } else {
          if (mm < M) epi.store(batch, mm, tn, half, wn * W + pl, v);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the next pass overwrites what was just read
    }
  }
}

}  // namespace kvp
