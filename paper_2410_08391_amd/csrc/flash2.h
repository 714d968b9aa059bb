// Causal grouped-query flash attention, head_dim 128, query groups of 3, 4, 6 or 8: the pipelined kernel.
//
// Same arithmetic (operation for operation), operand layouts and LDS tile formats as
// flash_prefill_kernel (see there): 8 waves, wave w serves query head w % G and the 32-row query
// sub-tile w / G (groups of 3 and 6 leave two of the eight waves without a tile: they only take
// part in the loads and barriers).  What differs is the schedule inside a wave.  On key tile j a wave has three
// dependent pieces of work: S(j) = QK(j), an MFMA chain; the softmax SM(j), vector arithmetic;
// O += PV(j), an MFMA chain.  Run in that order, with the block barrier keeping the two waves of
// a SIMD in step, the matrix core idles during both waves' softmax and the vector unit during
// both waves' chains: measured, the times simply add up.  Here a wave works on three tiles at
// once, and one phase is
//
//        MFMA:  PV(j-1), then QK(j+1)          VALU:  SM(j)
//
// written as 32 chunks of one MFMA, the LDS read of a later chunk's fragment and a slice of the
// softmax, pinned by a scheduling barrier after every chunk.  The exponentials run beside QK(j+1).
// The softmax reference of a query row is fixed by its first key tile and only an overflow guard
// watches the later ones (see flash_prefill_kernel: no row maximum in the steady state; the rare
// recomputation of a tile follows once PV(j-1) and the tile's exponentials are complete).  Scores are
// double buffered by tile parity.
//
// K and V tiles travel global -> LDS directly into two rings of four 16 KB slots.  At the top of
// phase j, after the barrier, the block requests K(j+3) and V(j+2): keys are needed one phase
// before the values of the same tile.  Every wave issues exactly four loads per phase (tile
// indices beyond the last are clamped, the data is never used), which makes the wait a constant
// vmcnt(6).  Only the last key tile of a block needs the causal mask (query blocks are 64 or 32
// rows, aligned): the masked softmax is a separate instantiation.
#pragma once
#include <type_traits>
#include <utility>

namespace kvp {

constexpr int F2_WAVES = 8;
constexpr int F2_SLOTS = 4;                  // ring slots per operand
constexpr int F2_TILE_BYTES = FA_KT * 128 * 2;   // one K tile or one V^T tile: 16 KB

__global__ __launch_bounds__(F2_WAVES * 64) void flash_prefill2_kernel(const bf16* __restrict__ q,
                                                                        const bf16* __restrict__ k,
                                                                        const bf16* __restrict__ vT,
                                                                        bf16* __restrict__ out, int T_len, int T_pad,
                                                                        int n_q, int n_kv, int G, int SUBS, float c_log2,
                                                                        float guard) {
  __shared__ __attribute__((aligned(1024))) bf16 kring[F2_SLOTS * FA_KT * 128];   // 64 KB
  __shared__ __attribute__((aligned(1024))) bf16 vring[F2_SLOTS * FA_KT * 128];   // 64 KB

  // SUBS: 32-row sub-tiles per block.  G = 6, 8 -> 1; G = 3, 4 -> 2, or 1 when the grid would
  // otherwise leave most of the chip idle (then half of the waves only load, and the active
  // ones have a SIMD each, which halves the time of the longest block).
  const int QB = 32 * SUBS;
  const int n_qt = (T_len + QB - 1) / QB;
  // One-dimensional grid, (sequence, kv head) group fastest and query tiles from the last (most
  // key tiles) to the first: the long blocks of every group start first and the short ones fill
  // the tail.  Blocks go to the XCDs round-robin, so a group's K / V stay within one XCD's L2
  // when the number of groups is a multiple of 8.
  const int n_groups = (int)gridDim.x / n_qt;         // = n_kv * batch
  const int grp = blockIdx.x % n_groups;
  const int qt = n_qt - 1 - blockIdx.x / n_groups;
  const int hk = grp % n_kv, b = grp / n_kv;
  const int tid = threadIdx.x, lane = tid % 64, wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int l32 = lane % 32, g = lane / 32;
  const bool active = wave < G * SUBS;                // this wave owns a (head, sub-tile)
  const int hq = hk * G + (active ? wave % G : 0);
  const int q_lo = qt * QB + (active ? wave / G : 0) * 32;
  const int q_block_hi = min(T_len, (qt + 1) * QB) - 1;
  const int n_tiles = q_block_hi / FA_KT + 1;
  const int ldq = n_q * 128, ldk = n_kv * 128;
  const int qpos = q_lo + l32;

  // Q^T fragments: lane holds query row qpos, dims 16 ks + 8 g .. + 7
  bf16x8 qf[8];
  {
    int pos = min(qpos, T_len - 1);
    const bf16* qr = q + ((size_t)b * T_len + pos) * ldq + (size_t)hq * 128 + g * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qr + ks * 16);
  }

  f32x16 acc_o[4], sacc[2][2];                        // sacc[tile parity][32-key half]
  bf16x8 pf[4];
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc_o[dt][i] = 0.f;

  const bf16* kbase = k + (size_t)b * T_len * ldk + (size_t)hk * 128;
  const bf16* vbase = vT + ((size_t)b * n_kv + hk) * 128 * (size_t)T_pad;

  // A tile is 16 wave-level loads (formats as in flash_prefill_kernel): two per wave.  The
  // requests are written as inline assembly on purpose: the compiler, seeing a direct-to-LDS load
  // it cannot tell apart from the LDS reads that follow, would make every fragment read wait for
  // ALL outstanding requests (vmcnt(0)) and so serialise the ring.  Completion is tracked by hand
  // with the constant vmcnt(6) at the top of each phase.
  const uint32_t kring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) bf16*)kring;
  const uint32_t vring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) bf16*)vring;
  auto dma16 = [&](const bf16* src, uint32_t lds_byte_addr) {   // lane l's 16 bytes land at lds_byte_addr + 16 l
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_byte_addr), "v"(src)
                 : "memory");
  };
  auto issue_k = [&](int tile) {
    const uint32_t st = kring_lds + (uint32_t)(tile % F2_SLOTS) * F2_TILE_BYTES;
    const int kv0 = min(tile, n_tiles - 1) * FA_KT;
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      const int i = wave * 2 + n;
      int rho = 4 * i + lane / 16;
      int ch = (lane % 16) ^ (rho & 15);
      int key = min(kv0 + perm16(rho), T_len - 1);
      dma16(kbase + (size_t)key * ldk + ch * 8, st + (uint32_t)i * 1024);
    }
  };
  auto issue_v = [&](int tile) {
    const uint32_t st = vring_lds + (uint32_t)(tile % F2_SLOTS) * F2_TILE_BYTES;
    const int kv0 = min(tile, n_tiles - 1) * FA_KT;
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      const int j = wave * 2 + n;
      int row = 8 * j + lane / 8;
      int ch = (lane % 8) ^ ((row >> 1) & 7);
      dma16(vbase + (size_t)row * T_pad + kv0 + ch * 8, st + (uint32_t)j * 1024);
    }
  };

  // Per-lane LDS byte addresses inside a slot (the swizzles of flash_prefill_kernel, rewritten so
  // that the fragment index enters as one XOR and the 32-row tile index as an immediate offset):
  //   K fragment (kt, ks):  kt * 8192 + (k_lane ^ (ks << 5))      = 2 * k_swz(kt*32 + l32, ks*2 + g)
  //   V fragment (dt, kk):  dt * 4096 + (v_lane ^ (kk << 5))      = 2 * v_swz(dt*32 + l32, kk*2 + g)
  const uint32_t k_lane = (uint32_t)(l32 * 256 + ((g ^ (l32 & 15)) << 4));
  const uint32_t v_lane = (uint32_t)(l32 * 128 + ((g ^ ((l32 >> 1) & 7)) << 4));
  // (byte offsets into the rings: the reads stay ordinary accesses of kring / vring)
  auto ld_k = [&](uint32_t off) { return *reinterpret_cast<const bf16x8*>(reinterpret_cast<const char*>(kring) + off); };
  auto ld_v = [&](uint32_t off) { return *reinterpret_cast<const bf16x8*>(reinterpret_cast<const char*>(vring) + off); };

  // One phase on tile j of parity C:  MFMA PV(j-1) [PV], MFMA QK(j+1) [QK], VALU SM(j) [SM, MASK].
  // FIRST: tile 0, whose row maximum becomes the reference of the row's exponentials.
  auto phase = [&](auto PVc, auto QKc, auto SMc, auto MASKc, auto FIRSTc, auto Cc, int j) {
    constexpr bool PV = decltype(PVc)::value, QK = decltype(QKc)::value, SM = decltype(SMc)::value;
    constexpr bool MASK = decltype(MASKc)::value, FIRST = decltype(FIRSTc)::value;
    static_assert(!FIRST || !PV, "the first tile has no predecessor");
    constexpr int C = decltype(Cc)::value;                   // parity of j: S(j) is sacc[C], S(j+1) goes to sacc[1-C]
    constexpr int NPV = PV ? 16 : 0, NM = NPV + (QK ? 16 : 0);
    constexpr int D = 3, R = 4;                               // fragment prefetch distance, ring size (deeper: spills, slower)
    const uint32_t vb = v_lane + (uint32_t)((j + F2_SLOTS - 1) % F2_SLOTS) * F2_TILE_BYTES;   // V(j-1)
    const uint32_t kb = k_lane + (uint32_t)((j + 1) % F2_SLOTS) * F2_TILE_BYTES;              // K(j+1)
    const int kv0 = j * FA_KT;
    bf16x8 fr[R];
    auto fetch = [&](auto Mc) {                               // fragment of MFMA number M of the phase
      constexpr int M = decltype(Mc)::value;
      if constexpr (M < NM) {
        if constexpr (M < NPV) fr[M % R] = ld_v((vb ^ ((M / 4) << 5)) + (M % 4) * 4096);
        else { constexpr int m = M - NPV; fr[M % R] = ld_k((kb ^ ((m / 2) << 5)) + (m % 2) * 8192); }
      }
    };
    auto mfma = [&](auto Mc) {
      constexpr int M = decltype(Mc)::value;
      if constexpr (M < NPV) {
        constexpr int kk = M / 4, dt = M % 4;
        acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[M % R], pf[kk], acc_o[dt], 0, 0, 0);
      } else if constexpr (M < NM) {
        constexpr int m = M - NPV;
        constexpr int ks = m / 2, kt = m % 2;
        if constexpr (ks == 0) {
          f32x16 zero;
#pragma unroll
          for (int i = 0; i < 16; ++i) zero[i] = 0.f;
          sacc[1 - C][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[M % R], qf[0], zero, 0, 0, 0);
        } else {
          sacc[1 - C][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[M % R], qf[ks], sacc[1 - C][kt], 0, 0, 0);
        }
      }
    };
    // Vector work: the causal mask (last tile only), then 16 pairs of exponentials spread over the QK
    // chunks (or after the chunks when there is no QK).  The first tile also searches its row maximum,
    // up front (it has no PV chain to hide behind), which becomes the row's reference.
    float mx = -INFINITY, mc = m_run * c_log2, psum = 0.f;
    auto mask_tile = [&]() {
      if constexpr (MASK) {
#pragma unroll
        for (int e = 0; e < 32; ++e) {
          const int kt = e / 16, i = e % 16;
          // accumulator element i of key tile kt is key kv0 + 32 kt + 16 (i/8) + 8 g + i%8
          int key = kv0 + 32 * kt + 16 * (i / 8) + 8 * g + (i % 8);
          if (key > qpos) sacc[C][kt][i] = -INFINITY;
        }
      }
    };
    auto row_max = [&]() {                                    // this lane's 32 scores, then the partner lane's
      mx = -INFINITY;
#pragma unroll
      for (int e = 0; e < 32; ++e) mx = fmaxf(mx, sacc[C][e / 16][e % 16]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    };
    auto exp_pair = [&](auto Uc) {
      constexpr int u = decltype(Uc)::value;
      constexpr int kt = u / 8, sgrp = (u / 4) % 2, e0 = 2 * (u % 4);
      float p0 = __builtin_amdgcn_exp2f(sacc[C][kt][sgrp * 8 + e0] * c_log2 - mc);
      float p1 = __builtin_amdgcn_exp2f(sacc[C][kt][sgrp * 8 + e0 + 1] * c_log2 - mc);
      psum += p0;
      psum += p1;
      pf[kt * 2 + sgrp][e0] = (bf16)p0;
      pf[kt * 2 + sgrp][e0 + 1] = (bf16)p1;
    };
    auto all_exps = [&]() {
      auto run = [&](auto self, auto Uc) -> void {
        exp_pair(Uc);
        if constexpr (decltype(Uc)::value + 1 < 16) self(self, std::integral_constant<int, decltype(Uc)::value + 1>{});
      };
      run(run, std::integral_constant<int, 0>{});
    };
    // new reference m_new >= m_run for the row: what has been accumulated so far is rescaled to it
    auto move_reference = [&](float m_new) {
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2);   // m_run = -inf (first tile): 0 * 0
      l_run *= alpha;
      m_run = m_new;
      mc = m_run * c_log2;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc_o[dt][i] *= alpha;
    };
    auto valu = [&](auto Mc) {
      constexpr int M = decltype(Mc)::value;
      if constexpr (SM && QK && M >= NPV) exp_pair(std::integral_constant<int, M - NPV>{});
    };
    auto chunk = [&](auto Mc) {
      constexpr int M = decltype(Mc)::value;
      fetch(std::integral_constant<int, M + D>{});
      mfma(Mc);
      valu(Mc);
      __builtin_amdgcn_sched_barrier(0);
    };
    auto chunks = [&](auto Lo, auto Hi) {
      constexpr int lo = decltype(Lo)::value, hi = decltype(Hi)::value;
      if constexpr (lo < hi) {
        auto run = [&](auto self, auto Ic) -> void {
          constexpr int I = decltype(Ic)::value;
          chunk(Ic);
          if constexpr (I + 1 < hi) self(self, std::integral_constant<int, I + 1>{});
        };
        run(run, Lo);
      }
    };
    {
      auto run = [&](auto self, auto Ic) -> void {
        fetch(Ic);
        if constexpr (decltype(Ic)::value + 1 < D) self(self, std::integral_constant<int, decltype(Ic)::value + 1>{});
      };
      run(run, std::integral_constant<int, 0>{});
    }
    if constexpr (SM) mask_tile();
    if constexpr (SM && FIRST) {                              // tile 0: its row maximum is the reference from here on
      row_max();
      move_reference(mx);
    }
    chunks(std::integral_constant<int, 0>{}, std::integral_constant<int, NPV>{});
    chunks(std::integral_constant<int, NPV>{}, std::integral_constant<int, NM>{});
    if constexpr (SM) {
      if constexpr (!QK) all_exps();
      if constexpr (!FIRST) {
        // Overflow guard (see flash_prefill_kernel).  PV(j-1) is complete here, so what has been accumulated
        // may be rescaled; the tile's probabilities are recomputed against the raised reference.
        if (__builtin_amdgcn_ballot_w64(!(psum <= guard)) != 0) {   // wave-uniform, rare
          row_max();
          move_reference(fmaxf(m_run, mx));
          psum = 0.f;
          all_exps();
        }
      }
      l_run += psum;
    }
  };
  using T_ = std::true_type;
  using F_ = std::false_type;
  using C0 = std::integral_constant<int, 0>;
  using C1 = std::integral_constant<int, 1>;
  // top of a phase: the block's shares of K(j+1) and V(j-1) have landed and every wave is done with
  // the slots the new requests overwrite
  auto top = [&](int j) {
    __builtin_amdgcn_s_waitcnt(0x0F76);   // vmcnt(6)
    __syncthreads();
    issue_k(j + 3);
    issue_v(j + 2);
  };

  // ---- prologue: K0 K1 V0 K2 V1 requested; S(0) = QK(0) ----
  issue_k(0); issue_k(1); issue_v(0); issue_k(2); issue_v(1);
  __builtin_amdgcn_s_waitcnt(0x0F78);     // vmcnt(8): K0 landed
  __syncthreads();
  if (!active) {                          // a wave without a tile: its share of the loads and the barriers only
    for (int jj = 0; jj <= n_tiles; ++jj) top(jj);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    return;
  }
  {
    // QK(0) alone: expressed as the QK part of a phase "-1" (K(j+1) with j = -1, parity 1 -> sacc[0])
    phase(F_{}, T_{}, F_{}, F_{}, F_{}, C1{}, -1);
  }
  // ---- phase 0: QK(1) beside SM(0) ----
  top(0);
  if (n_tiles == 1) phase(F_{}, F_{}, T_{}, T_{}, T_{}, C0{}, 0);
  else phase(F_{}, T_{}, T_{}, F_{}, T_{}, C0{}, 0);
  // ---- phases 1 .. n-2: PV(j-1), QK(j+1) beside SM(j), unmasked ----
  int j = 1;
  for (; j + 2 < n_tiles; j += 2) {
    top(j);
    phase(T_{}, T_{}, T_{}, F_{}, F_{}, C1{}, j);
    top(j + 1);
    phase(T_{}, T_{}, T_{}, F_{}, F_{}, C0{}, j + 1);
  }
  if (j + 1 < n_tiles) {                               // one more unmasked phase (odd j)
    top(j);
    phase(T_{}, T_{}, T_{}, F_{}, F_{}, C1{}, j);
    ++j;
  }
  // ---- phase n-1 (if n > 1): PV(n-2) beside the masked SM(n-1) ----
  if (n_tiles > 1) {
    top(j);
    if (j & 1) phase(T_{}, F_{}, T_{}, T_{}, F_{}, C1{}, j);
    else phase(T_{}, F_{}, T_{}, T_{}, F_{}, C0{}, j);
    ++j;
  }
  // ---- phase n: PV(n-1) ----
  top(j);
  phase(T_{}, F_{}, F_{}, F_{}, F_{}, C0{}, j);
  __builtin_amdgcn_s_waitcnt(0x0F70);     // drain the clamped tail requests before the block ends

  // O^T accumulator element i of dim tile dt: dim 32 dt + 8 (i/4) + 4 g + i%4, query column l32
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
