// bf16 MFMA GEMM for gfx950:  C[M, N] = A[M, K] * W[N, K]^T, fp32 accumulation.
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants: a lane feeds
// eight consecutive K elements of one row.  Tiles go global -> LDS directly (global_load_lds_dwordx4:
// no VGPR staging, no ds_write) through an NS-stage ring, so that loads run NS-1 K-steps ahead of
// the MFMAs; the wait for a stage is a manual s_waitcnt vmcnt(n) that leaves the younger stages in
// flight.  One such load writes 1 KB = 8 LDS rows, lane i at byte 16*i, so the XOR swizzle of the
// 128-byte rows is applied on the global side: lane i fetches chunk (i & 7) ^ key(r) of its row.
// The LDS of gfx950 sweeps 64 banks x 4 B = 256 B, i.e. two tile rows, so the key is (r >> 1) & 7:
// 16 consecutive rows then cover every bank exactly once per 16-byte read (measured: 1.5x the read
// rate of key r & 7, 5x that of unswizzled rows).  The fused epilogues are the ones the decoding
// step needs: rotary embedding + K / V^T store (QKV), SiLU(gate) * up (FFN), fp32 split-K partials
// that the next RMSNorm folds into the residual stream (O and down projections), and the LM head's
// per-tile (max, sum exp, argmax) reduction so that logits are never written.
//
// "Pair" epilogues need two columns in one lane (feature i and i + Dh/2 for the rotation, gate and
// up column for SwiGLU).  That is arranged by the order in which weight rows are placed in the LDS
// tile: fragment 2p of a wave holds side 0 and fragment 2p+1 side 1 of the same 32 columns.
#include "common.h"

#include <type_traits>

namespace l2pd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

enum { EPI_PARTIAL = 0, EPI_QKV = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3, EPI_QKV16 = 4, EPI_PARTIAL_SER = 5 };
// EPI_PARTIAL_SER is EPI_PARTIAL with GemmArgs::serial honoured (a kernel of its own: the second set of
// accumulators would cost the plain one registers).
// EPI_QKV and EPI_QKV16 compute the same Q/K/V projection with the same rotation arithmetic; they differ in
// how the weight rows are dealt to the MFMA column fragments.  EPI_QKV puts 32 first-half features of a head
// in one fragment and their rotation partners (feature + Dh/2) in the next, so a lane holds both members of
// a pair (needs an even number of fragments per wavefront).  EPI_QKV16 makes every fragment self-contained:
// columns 0..15 are 16 first-half features, columns 16..31 their partners, and a lane fetches its partner's
// value from the lane 16 further on; any number of fragments per wavefront then works (96-column tiles).

struct GemmArgs {
  const bf16* A;
  const bf16* B0;
  const bf16* B1;
  const bf16* B2;
  int M, N, K;          // N counts tile-space columns (for pair epilogues: both sides)
  int tiles_m, tiles_n, splits;
  Gate gate;
  // EPI_PARTIAL: K range z writes to parts + z * part_stride (fp32 [M, N])
  float* parts;
  size_t part_stride;
  int serial;           // > 1 (A-in-registers tile only, splits == 1): the workgroup walks `serial` K ranges one
                        // after the other, each into a fresh accumulator, and writes their sum, formed in
                        // ascending order: the bits that `serial` workgroups' partials give when the RMSNorm sums them
  int n_sub;            // > 0: the N rows are the rows of B0, B1, B2 stacked, n_sub rows each
  // EPI_SWIGLU
  bf16* act;
  int F;
  int act_quad_tiled;   // act in the quad-tiled layout (read into registers by the down projection) instead of row-major
  // EPI_QKV
  QkvEpilogue qkv;
  // EPI_LMHEAD
  LmHeadEpilogue lm;
};

// fp32 -> bf16, round to nearest even, two values per v_cvt_pk_bf16_f32; lo lands in bits 15:0
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ unsigned short f2bf(float f) { return (unsigned short)(pack_bf16(f, 0.f) & 0xffffu); }

// 4x4 transpose inside every aligned group of four lanes: on entry lane j of a group holds
// element (j, k) in w[k]; on return it holds element (k, j).  In the MFMA C layout a lane owns one
// column and four consecutive rows, so the transpose gives each lane four consecutive columns of
// one row, which it can store as one 8-byte piece instead of four 2-byte ones.
__device__ __forceinline__ void quad_transpose(unsigned (&w)[4], int lane) {
  const bool o1 = lane & 1, o2 = lane & 2;
  unsigned s0 = o1 ? w[0] : w[1], s1 = o1 ? w[2] : w[3];
  s0 = __shfl_xor(s0, 1, 64);
  s1 = __shfl_xor(s1, 1, 64);
  if (o1) { w[0] = s0; w[2] = s1; } else { w[1] = s0; w[3] = s1; }
  unsigned t0 = o2 ? w[0] : w[2], t1 = o2 ? w[1] : w[3];
  t0 = __shfl_xor(t0, 2, 64);
  t1 = __shfl_xor(t1, 2, 64);
  if (o2) { w[0] = t0; w[1] = t1; } else { w[2] = t0; w[3] = t1; }
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {   // s_waitcnt vmcnt(N) only (expcnt / lgkmcnt untouched)
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
// Workgroup barrier without the memory-model fence of __syncthreads(), which would wait for every
// outstanding global load (vmcnt(0)) and so drain the prefetch ring.  LDS visibility is ordered by
// the explicit waits around it; the empty asm statements keep the compiler from moving LDS
// accesses across the barrier.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// 16 bytes per lane, global -> LDS without passing through VGPRs.  The LDS destination of the whole
// wavefront is M0 + 16 * lane.  Written as inline asm on purpose: the compiler's wait-count pass
// falls back to lgkmcnt(0) before every LDS read while a direct-to-LDS load it knows of is in
// flight, which would serialise the fragment prefetch; completion is tracked by hand with
// wait_vmcnt<>().  (Untracked extra loads can only make the compiler's own vmcnt waits stricter,
// because vmcnt retires in order.)
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(gptr), "s"(lds_addr)
               : "memory", "m0");
}

// AREG (tiles whose wavefronts all sit side by side in M, WN == 1): a wavefront's A rows are read by that
// wavefront alone, so staging them in LDS buys no reuse and costs LDS bandwidth twice (the write of the
// direct-to-LDS load and the fragment read), and LDS bandwidth is what bounds the loop (taking A's LDS
// traffic out of the 256 x 192 gate/up loop, A not loaded at all, moves it from 1.04 to 1.22 PFLOP/s).
// With AREG the A fragments go global -> registers directly, in the MFMA operand layout (lane (row, half)
// loads the 16 bytes it feeds to a K-step), through a ring of four register sets, the stage they are
// for being NS-1 stages ahead like the LDS ring of B; only B is staged in LDS.  The K loop is unrolled
// four times so that the register sets are addressed statically.  A must be quad-tiled in memory (see
// gemm_qkv_a_quad_tiled in common.h): the operand layout puts consecutive lanes on consecutive rows, and from a row-major A
// every lane's 16 bytes would lie in a cache line of their own (64 tag look-ups per wavefront load; measured
// 131 us against 107 for the gate/up GEMM); quad-tiled, one wavefront load is eight whole lines.
template <int BM, int BN, int BK, int WM, int WN, int NS, int EPI, bool AREG = false>
__global__ void __launch_bounds__(WM* WN * 64) k_gemm_bf16(GemmArgs a) {
  constexpr int NT = WM * WN * 64;
  constexpr int NW = WM * WN;
  constexpr int FM = BM / WM / 32, FN = BN / WN / 32;
  constexpr bool PAIR = (EPI == EPI_QKV || EPI == EPI_SWIGLU);
  static_assert(!PAIR || (FN % 2 == 0), "pair epilogues need an even number of column fragments");
  static_assert(BK == 32 || BK == 64, "LDS tile rows hold 32 or 64 K elements");
  static_assert(!AREG || (WN == 1 && NS == 4), "A in registers: wavefronts side by side in M, four register sets");
  constexpr int CPR = BK / 8;               // 16-byte chunks per LDS row
  constexpr int RPD = 64 / CPR;             // rows filled by one direct-to-LDS wave load (1 KB)
  constexpr int KEY_SHIFT = BK == 64 ? 1 : 2;   // rows per 256-byte bank sweep = 1 << KEY_SHIFT
  constexpr int KS = BK / 16;               // MFMA K-steps per stage
  constexpr int LROWS = AREG ? BN : BM + BN;    // tile rows staged in LDS
  constexpr int LPS = LROWS / RPD / NW;     // direct-to-LDS loads per thread per stage
  constexpr int LPSW = LPS + (AREG ? FM * KS : 0);   // vector memory loads per thread per stage (what vmcnt counts)
  static_assert(LPS * NW * RPD == LROWS, "tile/threads mismatch");
  static_assert(NS >= 3 && (NS - 2) * LPSW < 64, "ring depth: at least 3 stages, vmcnt is 6 bits");

  if (gate_skip(a.gate)) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // [stage][A: BM rows (unless AREG) | B: BN rows][BK bf16]
  constexpr int STAGE_BYTES = LROWS * BK * 2;
  constexpr int BROW0 = AREG ? 0 : BM;      // first LDS row of the B tile

  // ---- tile assignment: consecutive ids on one XCD share a weight panel ----
  const int total = a.tiles_m * a.tiles_n * a.splits;
  const int per_xcd = (total + 7) / 8;
  const int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (v >= total) return;
  const int per_split = a.tiles_m * a.tiles_n;
  const int z = v / per_split;
  int rem = v % per_split;
  constexpr int GM = 8;
  const int chunk = rem / (GM * a.tiles_n);
  rem -= chunk * GM * a.tiles_n;
  const int gmc = min(GM, a.tiles_m - chunk * GM);
  const int tile_n = rem / gmc;
  const int tile_m = chunk * GM + rem % gmc;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int hf = lane >> 5, lj = lane & 31;

  const int k_len = a.K / a.splits;
  const int k_begin = z * k_len;
  const int nk = k_len / BK;

  // ---- per-thread source pointers of the direct-to-LDS loads (fixed over the K loop) ----
  // Load q of a stage (q = wave + i*NW) fills combined tile rows RPD*q .. RPD*q+RPD-1 (A rows first, then B).
  const bf16* src[LPS];
#pragma unroll
  for (int i = 0; i < LPS; ++i) {
    const int q = wave + i * NW;
    const int rr = q * RPD + lane / CPR;         // row in the combined [A; B] tile
    const int c = (lane % CPR) ^ ((rr >> KEY_SHIFT) & (CPR - 1));   // global chunk that belongs at this lane's slot
    if (rr < BROW0) {
      int gr = min(m0 + rr, a.M - 1);
      src[i] = a.A + (size_t)gr * a.K + k_begin + c * 8;
    } else {
      const int r = rr - BROW0;
      const bf16* base;
      size_t grow;
      if constexpr (EPI == EPI_QKV16) {
        const int half = a.qkv.Dh / 2, gpq = half / 16;
        const int Gq = tile_n * (BN / 32) + (r >> 5), j = r & 31;
        const int hg = Gq / gpq, gi = Gq % gpq;
        const int mat = min(hg / a.qkv.H, 2), head = hg % a.qkv.H;
        base = mat == 0 ? a.B0 : (mat == 1 ? a.B1 : a.B2);
        grow = (size_t)(head * a.qkv.Dh + gi * 16 + (j & 15) + (j >> 4) * half);
      } else if constexpr (!PAIR) {
        int gn = min(n0 + r, a.N - 1);
        base = a.B0;
        if (a.n_sub > 0) {
          const int mat = gn / a.n_sub;
          gn -= mat * a.n_sub;
          base = mat == 0 ? a.B0 : (mat == 1 ? a.B1 : a.B2);
        }
        grow = (size_t)gn;
      } else {
        int rw = r / (32 * FN), f = (r >> 5) % FN, j = r & 31;
        int G = tile_n * (BN / 64) + rw * (FN / 2) + (f >> 1), side = f & 1;
        if constexpr (EPI == EPI_SWIGLU) {
          base = side ? a.B1 : a.B0;
          grow = (size_t)min(G * 32 + j, a.F - 1);
        } else {
          const int half = a.qkv.Dh / 2, gph = half / 32;
          int hg = G / gph, gi = G % gph;
          int mat = hg / a.qkv.H, head = hg % a.qkv.H;
          mat = min(mat, 2);
          base = mat == 0 ? a.B0 : (mat == 1 ? a.B1 : a.B2);
          grow = (size_t)(head * a.qkv.Dh + side * half + gi * 32 + j);
        }
      }
      src[i] = base + grow * a.K + k_begin + c * 8;
    }
  }
  // LDS byte address of this wave's first slot in stage 0 (wave-uniform, goes to M0)
  const unsigned lds0 = __builtin_amdgcn_readfirstlane(
      (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)(smem + wave * 1024));
  // AREG: this lane's 16 bytes of fragment i at K-step 0 of stage 0
  const bf16* pa[FM];
#pragma unroll
  for (int i = 0; i < FM; ++i)
  {
    // quad-tiled A (see gemm_qkv_a_quad_tiled in common.h): chunk c of row r at ((r / 4) * (K / 8) + c) * 32 + (r % 4) * 8
    const int r = min(m0 + wm * (BM / WM) + i * 32 + lj, a.M - 1);
    pa[i] = a.A + ((size_t)(r >> 2) * (a.K / 8) + k_begin / 8 + hf) * 32 + (r & 3) * 8;
  }
  bf16x8_t ra[AREG ? 4 : 1][FM][KS];
  // Loads of one stage are issued in KS parts (load i belongs to part i % KS), one part per K-step,
  // so that they trickle into the texture-address queue behind MFMAs instead of arriving as a burst
  // from every wave right after the barrier (a burst stalls instruction issue until the queue drains).
  // kt < 0: nothing left to stage in LDS.  The A register loads (AREG) are issued all the same, from the
  // last stage's address when stage kt_a lies behind the end of K: the compiler counts the loads it knows
  // of to place its own waits, and a count that depended on a branch would make it wait for every load.
  auto issue_part = [&](auto setc, int kt, int kt_a, int part) {
    constexpr int SET = decltype(setc)::value;    // AREG: register set of stage kt_a (kt_a % 4, known statically)
    if (kt >= 0) {
      const unsigned dst = lds0 + (kt % NS) * STAGE_BYTES;
#pragma unroll
      for (int i = 0; i < LPS; ++i)
        if (i % KS == part) dma16(src[i] + kt * BK, dst + i * NW * 1024);
    }
    if constexpr (AREG) {
      // plain loads; the direct-to-LDS loads around them are volatile asm with a memory clobber, so all of
      // them stay where they are in the instruction stream and vmcnt counts LPSW loads per stage
      const int kc = min(kt_a, nk - 1);
#pragma unroll
      for (int pp = 0; pp < KS; ++pp)
        if (pp == part) {
#pragma unroll
          for (int i = 0; i < FM; ++i)
            ra[SET][i][pp] = *reinterpret_cast<const bf16x8_t*>(pa[i] + (kc * (BK / 8) + pp * 2) * 32);
        }
    }
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragment row byte offsets inside a stage (row * 128) and the row's swizzle key
  int offA[FM], offB[FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) offA[i] = (wm * (BM / WM) + i * 32 + lj) * (BK * 2);
#pragma unroll
  for (int j = 0; j < FN; ++j) offB[j] = BROW0 * (BK * 2) + (wn * (BN / WN) + j * 32 + lj) * (BK * 2);
  const int key = (lj >> KEY_SHIFT) & (CPR - 1);   // row's swizzle key (fragment bases are multiples of 32)

  // Software pipeline.  Fragments are double-buffered in registers: the ds_reads of K-step kk+1 are
  // issued before the MFMAs of step kk, and the first fragments of the next stage are read during
  // the last step of the current one.  The ring advances (wait for stage kt+1, barrier, refill the
  // buffer of stage kt-1 with stage kt+NS-1) right before that last step, so a wave that waits at
  // the barrier leaves a full step of MFMAs queued behind it.
  bf16x8_t fa[2][FM], fb[2][FN];
  auto read_frags = [&](int buf, const unsigned char* base, int kk) {
    const int sw = ((kk * 2 + hf) ^ key) << 4;
    if constexpr (!AREG) {
#pragma unroll
      for (int i = 0; i < FM; ++i) fa[buf][i] = *reinterpret_cast<const bf16x8_t*>(base + offA[i] + sw);
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) fb[buf][j] = *reinterpret_cast<const bf16x8_t*>(base + offB[j] + sw);
  };
  // One K-step: the FM*FN MFMAs on fragment set `cur`, with the ds_reads that fetch set `cur ^ 1`
  // (K-step kk_next of the stage at `nbase`) slotted in between them, one read after each of the
  // first MFMAs, so that every read is issued while an MFMA occupies the matrix pipe.  (AREG: the A
  // fragments of the step are register set SET's, and only the FN reads of B are slotted in.)
  constexpr int NR = AREG ? FN : FM + FN;
  auto step = [&](auto setc, auto dsetc, int kk, const unsigned char* nbase, int kk_next, int dma_kt, int dma_kt_a,
                  int dma_part) {
    const int cur = kk & 1;   // fragment set of K-step kk
    constexpr int SET = decltype(setc)::value;
    const int sw = ((kk_next * 2 + hf) ^ key) << 4;
    const int nxt = cur ^ 1;
#pragma unroll
    for (int idx = 0; idx < FM * FN; ++idx) {
      const int i = idx / FN, j = idx % FN;
      if constexpr (AREG) {
        // every call site passes a constant kk (the K loop over a stage is fully unrolled), so the register
        // set is addressed statically
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ra[SET][i][kk], fb[cur][j], acc[i][j], 0, 0, 0);
      } else {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < NR; ++r) {
        if ((r < FM * FN ? r : FM * FN - 1) != idx) continue;   // read r goes after MFMA min(r, last)
        if constexpr (AREG) {
          fb[nxt][r] = *reinterpret_cast<const bf16x8_t*>(nbase + offB[r] + sw);
        } else {
          if (r < FM) fa[nxt][r] = *reinterpret_cast<const bf16x8_t*>(nbase + offA[r] + sw);
          else fb[nxt][r - FM] = *reinterpret_cast<const bf16x8_t*>(nbase + offB[r - FM] + sw);
        }
      }
      if (idx == 0 && (AREG || dma_kt >= 0)) issue_part(dsetc, dma_kt, dma_kt_a, dma_part);   // stays in program order
    }
#pragma unroll
    for (int idx = 0; idx < FM * FN; ++idx) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA, then the LDS reads of its slot
#pragma unroll
      for (int r = 0; r < NR; ++r)
        if ((r < FM * FN ? r : FM * FN - 1) == idx) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // Prologue.  Without AREG: stages 0 .. NS-2 in full.  With AREG: stages 0 .. NS-3 in full and part 0 of stage
  // NS-2; its other parts go out with the K-steps of stage 0, like those of every later stage.  (If the prologue
  // loaded them too, stage 0 would load the same registers again, the compiler would drop the prologue's loads
  // as dead, and the count below would no longer be the number of loads in flight.)  The wait counts loads,
  // so nothing may move across it: scheduling barriers on both sides.
  constexpr int P0 = (LPS + KS - 1) / KS + (AREG ? FM : 0);   // loads of part 0 of a stage
  {
    auto pro = [&](auto setc) {
      constexpr int ST = decltype(setc)::value;
      if (ST < NS - 1 && (AREG || ST < nk)) {   // AREG: nk is a multiple of four
#pragma unroll
        for (int part = 0; part < KS; ++part)
          if (!AREG || ST < NS - 2 || part == 0) issue_part(setc, ST, ST, part);
      }
    };
    pro(std::integral_constant<int, 0>{});
    pro(std::integral_constant<int, 1>{});
    pro(std::integral_constant<int, 2>{});
    static_assert(NS - 1 <= 5, "prologue covers up to five stages");
    if constexpr (NS - 1 > 3) pro(std::integral_constant<int, 3>{});
    if constexpr (NS - 1 > 4) pro(std::integral_constant<int, 4>{});
  }
  __builtin_amdgcn_sched_barrier(0);
  if constexpr (AREG) {
    wait_vmcnt<(NS - 3) * LPSW + P0>();   // stage 0 has landed: only the later stages' loads are outstanding
  } else {
    if (nk >= NS - 1) wait_vmcnt<(NS - 2) * LPSW>();
    else wait_vmcnt<0>();
  }
  __builtin_amdgcn_sched_barrier(0);
  lds_barrier();
  // Drain scalar loads here, so that only in-order LDS reads are pending when the loop is entered
  // and the compiler can wait for "all but the newest reads" instead of lgkmcnt(0) at its head.
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
  read_frags(0, smem, 0);
  __builtin_amdgcn_sched_barrier(0);
  // One stage of the K loop; SET = kt % 4 names the register sets statically (ignored without AREG).
  auto stage = [&](auto setc, int kt) {
    constexpr int SET = decltype(setc)::value;
    const unsigned char* base = smem + (kt % NS) * STAGE_BYTES;
    // parts 1 .. KS-1 of stage kt+NS-2 (its part 0 went out with the last K-step of iteration kt-1)
    // (without AREG the prologue has issued all of stage NS-2 already)
    const int dma_a = ((AREG || kt >= 1) && kt + NS - 2 < nk) ? kt + NS - 2 : -1;
#pragma unroll
    for (int kk = 0; kk < KS - 1; ++kk)
      step(setc, std::integral_constant<int, (SET + NS - 2) % 4>{}, kk, base, kk + 1, dma_a, kt + NS - 2, kk + 1);
    if (kt + 1 < nk) {
      // stage kt+1 has landed once at most the loads of the NS-3 younger stages are outstanding
      if (kt + NS - 2 < nk) wait_vmcnt<(NS - 3) * LPSW>();
      else wait_vmcnt<0>();
      lds_barrier();   // stage kt+1 visible to all; every wave is past its reads of stage kt-1
    }
    __builtin_amdgcn_sched_barrier(0);
    // The reads of the next stage's first fragments are unconditional (after the last stage they
    // fetch stale but valid LDS that nobody uses): a branch around them would make the compiler's
    // LDS wait counts conservative at the join.  The buffer of stage kt-1 is free from here on:
    // start refilling it with stage kt+NS-1.
    step(setc, std::integral_constant<int, (SET + NS - 1) % 4>{}, KS - 1, smem + ((kt + 1) % NS) * STAGE_BYTES, 0,
         (kt + NS - 1 < nk) ? kt + NS - 1 : -1, kt + NS - 1, 0);
  };
  constexpr bool SERIAL = AREG && EPI == EPI_PARTIAL_SER;
  f32x16 tot[SERIAL ? FM : 1][SERIAL ? FN : 1];   // sum of the finished K ranges
  const int seg = SERIAL ? nk / max(a.serial, 1) : 0;   // stages per K range (a multiple of four)
  if constexpr (AREG) {
    for (int kt = 0; kt < nk; kt += 4) {   // the launcher guarantees nk % 4 == 0
      stage(std::integral_constant<int, 0>{}, kt);
      stage(std::integral_constant<int, 1>{}, kt + 1);
      stage(std::integral_constant<int, 2>{}, kt + 2);
      stage(std::integral_constant<int, 3>{}, kt + 3);
      if constexpr (SERIAL) {
        if (a.serial > 1 && (kt + 4) % seg == 0) {   // a K range ends here: bank it and start the next from zero
          const bool first = kt + 4 == seg;
#pragma unroll
          for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                tot[i][j][r] = first ? acc[i][j][r] : tot[i][j][r] + acc[i][j][r];
                acc[i][j][r] = 0.f;
              }
        }
      }
    }
    if constexpr (SERIAL) {
      if (a.serial > 1) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j) acc[i][j] = tot[i][j];
      }
    }
  } else {
    for (int kt = 0; kt < nk; ++kt) stage(std::integral_constant<int, 0>{}, kt);
  }
  lds_barrier();

  // ------------------------------------------------------------------------------------------
  // C layout of the 32x32 MFMA: register r of a lane is row (r/4)*8 + hf*4 + r%4, column lj.
  const int row_base = m0 + wm * (BM / WM);
  if constexpr (EPI == EPI_PARTIAL || EPI == EPI_PARTIAL_SER) {
    float* out = a.parts + (size_t)z * a.part_stride;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        int col = n0 + wn * (BN / WN) + j * 32 + lj;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int row = row_base + i * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
          if (row < a.M && col < a.N) out[(size_t)row * a.N + col] = acc[i][j][r];
        }
      }
  } else if constexpr (EPI == EPI_SWIGLU) {
    const int lr = lj & 3, c4 = lj & ~3;   // after the transpose: row within the group, first of 4 columns
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int p = 0; p < FN / 2; ++p) {
        const int G = tile_n * (BN / 64) + wn * (FN / 2) + p;
        const int col = G * 32 + c4;
#pragma unroll
        for (int rq = 0; rq < 4; rq += 2) {   // two row groups share one transpose: low / high half words
          unsigned w[4];
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            const float g0 = acc[i][2 * p][rq * 4 + rr], u0 = acc[i][2 * p + 1][rq * 4 + rr];
            const float g1 = acc[i][2 * p][rq * 4 + 4 + rr], u1 = acc[i][2 * p + 1][rq * 4 + 4 + rr];
            // SiLU(g) * u with the hardware reciprocal (1 ulp) instead of an exact division; the
            // operations are spelled out so that every tile configuration rounds alike
            const float s0 = __fmul_rn(__fmul_rn(g0, __builtin_amdgcn_rcpf(__fadd_rn(1.f, __expf(-g0)))), u0);
            const float s1 = __fmul_rn(__fmul_rn(g1, __builtin_amdgcn_rcpf(__fadd_rn(1.f, __expf(-g1)))), u1);
            w[rr] = pack_bf16(s0, s1);
          }
          quad_transpose(w, lane);
#pragma unroll
          for (int h2 = 0; h2 < 2; ++h2) {
            const int row = row_base + i * 32 + (rq + h2) * 8 + hf * 4 + lr;
            uint2 o;
            o.x = h2 ? (w[0] >> 16) | (w[1] & 0xffff0000u) : (w[0] & 0xffffu) | (w[1] << 16);
            o.y = h2 ? (w[2] >> 16) | (w[3] & 0xffff0000u) : (w[2] & 0xffffu) | (w[3] << 16);
            if (row < a.M && col < a.F) {   // F is a multiple of 4, so a group of 4 columns is in or out as a whole
              const size_t at = a.act_quad_tiled
                                    ? ((size_t)(row >> 2) * (a.F / 8) + (col >> 3)) * 32 + (row & 3) * 8 + (col & 7)
                                    : (size_t)row * a.F + col;
              *reinterpret_cast<uint2*>(reinterpret_cast<unsigned short*>(a.act) + at) = o;
            }
          }
        }
      }
  } else if constexpr (EPI == EPI_QKV) {
    const QkvEpilogue& e = a.qkv;
    const int half = e.Dh / 2, gph = half / 32;
    const bool vec4 = (e.Tq % 4 == 0) && (e.pos0 % 4 == 0) && (e.Tpad % 4 == 0) && (!e.seq_gb || e.pos_per_gb % 4 == 0);
    const int lr = lj & 3;
    // which matrix / head / 32-feature group each of the wavefront's fragment pairs belongs to (uniform)
    int p_mat[FN / 2], p_head[FN / 2], p_gi[FN / 2];
#pragma unroll
    for (int p = 0; p < FN / 2; ++p) {
      const int G = tile_n * (BN / 64) + wn * (FN / 2) + p;
      const int hg = G / gph;
      p_gi[p] = G % gph;
      p_mat[p] = hg / e.H;
      p_head[p] = hg % e.H;
    }
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      // Sequence and position of this lane's 16 rows (register r: row (r/4)*8 + hf*4 + r%4 of the fragment), worked
      // out once per row fragment and shared by all fragment pairs.
      int seq_r[16], pos_r[16];
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int row0 = row_base + i * 32 + rq * 8 + hf * 4;
        int t = row0 % e.Tq, bq = row0 / e.Tq;
        int off = (e.seq_gb && row0 < a.M) ? e.seq_gb[bq] * e.pos_per_gb : 0;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          seq_r[rq * 4 + rr] = bq;
          pos_r[rq * 4 + rr] = e.pos0 + off + t;
          if (++t == e.Tq) {   // next sequence of the batch
            t = 0;
            ++bq;
            off = (e.seq_gb && row0 + rr + 1 < a.M) ? e.seq_gb[bq] * e.pos_per_gb : 0;
          }
        }
      }
      // after the transposes a lane stores row `lr` of each group of four
      int seq_st[4], pos_st[4];
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        seq_st[rq] = lr == 0 ? seq_r[rq * 4] : (lr == 1 ? seq_r[rq * 4 + 1] : (lr == 2 ? seq_r[rq * 4 + 2] : seq_r[rq * 4 + 3]));
        pos_st[rq] = lr == 0 ? pos_r[rq * 4] : (lr == 1 ? pos_r[rq * 4 + 1] : (lr == 2 ? pos_r[rq * 4 + 2] : pos_r[rq * 4 + 3]));
      }
#pragma unroll
      for (int p = 0; p < FN / 2; ++p) {
        const int mat = p_mat[p], head = p_head[p], gi = p_gi[p];
        if (mat > 2) continue;                               // uniform over the wavefront
        const int dim = gi * 32 + lj;   // first-half feature index; partner is dim + half
        if (mat == 2) {
          // V is stored transposed ([B, H, Dh, Tpad]) so that attention reads keys contiguously
          unsigned short* vt = reinterpret_cast<unsigned short*>(e.vtstore);
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const int row0 = row_base + i * 32 + rq * 8 + hf * 4;
            if (vec4 && row0 + 3 < a.M) {
              const size_t o = ((size_t)(seq_r[rq * 4] * e.H + head) * e.Dh + dim) * e.Tpad + pos_r[rq * 4];
              uint2 lo4, hi4;
              lo4.x = pack_bf16(acc[i][2 * p][rq * 4 + 0], acc[i][2 * p][rq * 4 + 1]);
              lo4.y = pack_bf16(acc[i][2 * p][rq * 4 + 2], acc[i][2 * p][rq * 4 + 3]);
              hi4.x = pack_bf16(acc[i][2 * p + 1][rq * 4 + 0], acc[i][2 * p + 1][rq * 4 + 1]);
              hi4.y = pack_bf16(acc[i][2 * p + 1][rq * 4 + 2], acc[i][2 * p + 1][rq * 4 + 3]);
              *reinterpret_cast<uint2*>(vt + o) = lo4;
              *reinterpret_cast<uint2*>(vt + o + (size_t)half * e.Tpad) = hi4;
            } else {
#pragma unroll
              for (int rr = 0; rr < 4; ++rr) {
                if (row0 + rr >= a.M) continue;
                const size_t o = ((size_t)(seq_r[rq * 4 + rr] * e.H + head) * e.Dh + dim) * e.Tpad + pos_r[rq * 4 + rr];
                vt[o] = f2bf(acc[i][2 * p][rq * 4 + rr]);
                vt[o + (size_t)half * e.Tpad] = f2bf(acc[i][2 * p + 1][rq * 4 + rr]);
              }
            }
          }
        } else {
          // Rotation of Q and K.  All table reads of the fragment pair are issued before its first
          // store: the compiler cannot move a load above a store that might alias it, so an
          // interleaved order would pay one memory round trip per element.
          unsigned short* dst = reinterpret_cast<unsigned short*>(mat == 0 ? e.q : e.kstore);
          float cs[16], sn[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const bool live = row_base + i * 32 + (r >> 2) * 8 + hf * 4 + (r & 3) < a.M;
            const unsigned ti = (unsigned)pos_r[r] * (unsigned)half + (unsigned)dim;   // < 2^31 by construction
            cs[r] = live ? e.cos_t[ti] : 0.f;
            sn[r] = live ? e.sin_t[ti] : 0.f;
          }
          // rotate, round, and turn "one column, four rows" per lane into "four columns, one row"
          const int c4 = gi * 32 + (lj & ~3);
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            unsigned w[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
              const int r = rq * 4 + rr;
              const float x1 = acc[i][2 * p][r], x2 = acc[i][2 * p + 1][r];
              // explicit roundings: every tile configuration must produce the same bits, whatever
              // contraction into fused multiply-adds the compiler would pick for each of them
              const float o1 = __fmaf_rn(x1, cs[r], -__fmul_rn(x2, sn[r]));
              const float o2 = __fmaf_rn(x2, cs[r], __fmul_rn(x1, sn[r]));
              w[rr] = pack_bf16(o1, o2);
            }
            quad_transpose(w, lane);
            const int row = row_base + i * 32 + rq * 8 + hf * 4 + lr;
            if (row >= a.M) continue;
            const size_t o = mat == 0 ? (size_t)row * e.d + head * e.Dh + c4
                                      : ((size_t)seq_st[rq] * e.Tpad + pos_st[rq]) * e.d + head * e.Dh + c4;
            uint2 lo, hi;   // feature c4..c4+3 and its partner c4+half..c4+half+3
            lo.x = (w[0] & 0xffffu) | (w[1] << 16);
            lo.y = (w[2] & 0xffffu) | (w[3] << 16);
            hi.x = (w[0] >> 16) | (w[1] & 0xffff0000u);
            hi.y = (w[2] >> 16) | (w[3] & 0xffff0000u);
            *reinterpret_cast<uint2*>(dst + o) = lo;
            *reinterpret_cast<uint2*>(dst + o + half) = hi;
          }
        }
      }
    }
  } else if constexpr (EPI == EPI_QKV16) {
    const QkvEpilogue& e = a.qkv;
    const int half = e.Dh / 2, gpq = half / 16;
    const bool vec4 = (e.Tq % 4 == 0) && (e.pos0 % 4 == 0) && (e.Tpad % 4 == 0) && (!e.seq_gb || e.pos_per_gb % 4 == 0);
    const int up = (lj >> 4) & 1;   // 0: this lane's column is a first-half feature, 1: its rotation partner
    const int lr = lj & 3;
    // which matrix / head / 16-feature group each of the wavefront's column fragments belongs to (uniform)
    int f_mat[FN], f_head[FN], f_gi[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int Gq = tile_n * (BN / 32) + wn * FN + j;
      const int hg = Gq / gpq;
      f_gi[j] = Gq % gpq;
      f_mat[j] = hg / e.H;
      f_head[j] = hg % e.H;
    }
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      // Sequence and position of this lane's 16 rows (register r: row (r/4)*8 + hf*4 + r%4 of the fragment), worked
      // out once per row fragment and shared by all column fragments.
      int seq_r[16], pos_r[16];
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int row0 = row_base + i * 32 + rq * 8 + hf * 4;
        int t = row0 % e.Tq, bq = row0 / e.Tq;
        int off = (e.seq_gb && row0 < a.M) ? e.seq_gb[bq] * e.pos_per_gb : 0;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          seq_r[rq * 4 + rr] = bq;
          pos_r[rq * 4 + rr] = e.pos0 + off + t;
          if (++t == e.Tq) {   // next sequence of the batch
            t = 0;
            ++bq;
            off = (e.seq_gb && row0 + rr + 1 < a.M) ? e.seq_gb[bq] * e.pos_per_gb : 0;
          }
        }
      }
      // after the transposes a lane stores row `lr` of each group of four
      int seq_st[4], pos_st[4];
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        seq_st[rq] = lr == 0 ? seq_r[rq * 4] : (lr == 1 ? seq_r[rq * 4 + 1] : (lr == 2 ? seq_r[rq * 4 + 2] : seq_r[rq * 4 + 3]));
        pos_st[rq] = lr == 0 ? pos_r[rq * 4] : (lr == 1 ? pos_r[rq * 4 + 1] : (lr == 2 ? pos_r[rq * 4 + 2] : pos_r[rq * 4 + 3]));
      }
      // Rotation tables, one column fragment ahead: the reads for fragment j + 1 are issued before fragment j's
      // arithmetic and stores (the compiler cannot move a load above a store that might alias it, so read in
      // place every fragment would wait out a memory round trip of its own).
      float cst[2][16], snt[2][16];
      auto load_tab = [&](int j, int buf) {
        if (f_mat[j] >= 2) return;                           // V (or past the last column): no rotation
        const int dim1 = f_gi[j] * 16 + (lj & 15);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const bool live = row_base + i * 32 + (r >> 2) * 8 + hf * 4 + (r & 3) < a.M;
          const unsigned ti = (unsigned)pos_r[r] * (unsigned)half + (unsigned)dim1;   // < 2^31 by construction
          cst[buf][r] = live ? e.cos_t[ti] : 0.f;
          snt[buf][r] = live ? e.sin_t[ti] : 0.f;
        }
      };
      load_tab(0, 0);
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        if (j + 1 < FN) load_tab(j + 1, (j + 1) & 1);
        const float* cs = cst[j & 1];
        const float* sn = snt[j & 1];
        const int mat = f_mat[j], head = f_head[j];
        if (mat > 2) continue;                               // uniform over the wavefront
        const int dim1 = f_gi[j] * 16 + (lj & 15);
        const int dim = dim1 + up * half;                    // this lane's own feature
        if (mat == 2) {
          unsigned short* vt = reinterpret_cast<unsigned short*>(e.vtstore);
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const int row0 = row_base + i * 32 + rq * 8 + hf * 4;
            if (vec4 && row0 + 3 < a.M) {
              const size_t o = ((size_t)(seq_r[rq * 4] * e.H + head) * e.Dh + dim) * e.Tpad + pos_r[rq * 4];
              uint2 v4;
              v4.x = pack_bf16(acc[i][j][rq * 4 + 0], acc[i][j][rq * 4 + 1]);
              v4.y = pack_bf16(acc[i][j][rq * 4 + 2], acc[i][j][rq * 4 + 3]);
              *reinterpret_cast<uint2*>(vt + o) = v4;
            } else {
#pragma unroll
              for (int rr = 0; rr < 4; ++rr) {
                if (row0 + rr >= a.M) continue;
                vt[((size_t)(seq_r[rq * 4 + rr] * e.H + head) * e.Dh + dim) * e.Tpad + pos_r[rq * 4 + rr]] =
                    f2bf(acc[i][j][rq * 4 + rr]);
              }
            }
          }
        } else {
          unsigned short* dst = reinterpret_cast<unsigned short*>(mat == 0 ? e.q : e.kstore);
          float o[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float x = acc[i][j][r];
            const float xp = __shfl_xor(x, 16, 64);
            const float ps = __fmul_rn(xp, sn[r]);
            o[r] = __fmaf_rn(x, cs[r], up ? ps : -ps);
          }
          const int c4 = f_gi[j] * 16 + (lj & 12) + up * half;   // after the transpose: first of this lane's four features
#pragma unroll
          for (int rq = 0; rq < 4; rq += 2) {   // two row groups share one transpose: low / high half words
            unsigned w[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) w[rr] = pack_bf16(o[rq * 4 + rr], o[rq * 4 + 4 + rr]);
            quad_transpose(w, lane);
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
              const int row = row_base + i * 32 + (rq + h2) * 8 + hf * 4 + lr;
              if (row >= a.M) continue;
              const size_t oo = mat == 0 ? (size_t)row * e.d + head * e.Dh + c4
                                         : ((size_t)seq_st[rq + h2] * e.Tpad + pos_st[rq + h2]) * e.d + head * e.Dh + c4;
              uint2 st;
              st.x = h2 ? (w[0] >> 16) | (w[1] & 0xffff0000u) : (w[0] & 0xffffu) | (w[1] << 16);
              st.y = h2 ? (w[2] >> 16) | (w[3] & 0xffff0000u) : (w[2] & 0xffffu) | (w[3] << 16);
              *reinterpret_cast<uint2*>(dst + oo) = st;
            }
          }
        }
      }
    }
  } else {  // EPI_LMHEAD
    const LmHeadEpilogue& e = a.lm;
    float* s_m = reinterpret_cast<float*>(smem);            // [WN][BM]   (tile buffers are dead now)
    float* s_s = s_m + WN * BM;
    int* s_i = reinterpret_cast<int*>(s_s + WN * BM);
    __syncthreads();
    const bool biased = e.bias.value != 0.f && a.gate.ctl;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int lrow = wm * (BM / WM) + i * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
        int row = m0 + lrow;
        float vals[FN];
        float m = -INFINITY;
        int mi = 0x7fffffff;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          int col = n0 + wn * (BN / WN) + j * 32 + lj;
          float v = acc[i][j][r];
          if (biased && col == e.bias.token_id && row < a.M &&
              a.gate.ctl[CTL_SEQ_GB + row / e.bias.block_len] * e.bias.block_len + (row % e.bias.block_len) >=
                  e.bias.gen_pos_from)
            v += e.bias.value;
          if (e.logits && row < a.M && col < a.N) e.logits[(size_t)row * a.N + col] = v;
          if (col == e.mask_id || col >= a.N) v = -INFINITY;
          vals[j] = v;
          if (v > m) { m = v; mi = col; }   // columns ascend with j: first maximum wins
        }
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) {
          float m2 = __shfl_xor(m, o, 64);
          int i2 = __shfl_xor(mi, o, 64);
          if (m2 > m || (m2 == m && i2 < mi)) { m = m2; mi = i2; }
        }
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < FN; ++j) sum += (m == -INFINITY) ? 0.f : __expf(vals[j] - m);
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
        if (lj == 0) {
          s_m[wn * BM + lrow] = m;
          s_s[wn * BM + lrow] = sum;
          s_i[wn * BM + lrow] = mi;
        }
      }
    __syncthreads();
    if (e.part_max) {
      for (int lrow = tid; lrow < BM; lrow += NT) {
        int row = m0 + lrow;
        if (row >= a.M) continue;
        float m = s_m[lrow], sum = s_s[lrow];
        int mi = s_i[lrow];
#pragma unroll
        for (int w = 1; w < WN; ++w) {
          float m2 = s_m[w * BM + lrow], s2 = s_s[w * BM + lrow];
          int i2 = s_i[w * BM + lrow];
          float M = fmaxf(m, m2);
          float f1 = (m == -INFINITY) ? 0.f : __expf(m - M), f2 = (m2 == -INFINITY) ? 0.f : __expf(m2 - M);
          sum = sum * f1 + s2 * f2;
          if (m2 > m || (m2 == m && i2 < mi)) mi = i2;
          m = M;
        }
        size_t o = (size_t)row * e.n_part + tile_n;
        e.part_max[o] = m;
        e.part_sum[o] = sum;
        e.part_idx[o] = mi;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int BK, int WM, int WN, int NS, int EPI, bool AREG = false>
static void launch(GemmArgs& a, hipStream_t s) {
  auto kern = k_gemm_bf16<BM, BN, BK, WM, WN, NS, EPI, AREG>;
  constexpr int smem = NS * ((AREG ? 0 : BM) + BN) * BK * 2;
  static DynLdsAttr attr;
  attr.ensure(reinterpret_cast<const void*>(kern), smem);
  a.tiles_m = (a.M + BM - 1) / BM;
  a.tiles_n = (a.N + BN - 1) / BN;
  int total = a.tiles_m * a.tiles_n * a.splits;
  int grid = ((total + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), smem, s, a);
}

// Tile choice.  One CU moves about 64 B/clk from L2 into LDS, which a 128x128 tile needs in full to
// keep its MFMAs fed (64 flop per loaded byte); 256-wide tiles halve that traffic and win whenever
// there are enough of them to occupy the 256 CUs.  cost = rounds over the CUs x work per tile /
// measured relative per-CU rate of the configuration.  256x192 exists because 512 rows x 24576
// gate/up columns make exactly 256 such tiles, one round with every CU busy; for the 12288 Q/K/V
// columns 256x96 (pick_tile_qkv, A in registers) and, where that is not available, 128x192 do the same.
// (With random operands the chip is power limited: the shader clock sits well below its 2.4 GHz inside
// these kernels, and a register-resident MFMA stream alone tops out at 1.78 PFLOP/s.)
static double tile_cost(int M, int N, int bm, int bn, double rate) {
  const double tiles = (double)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
  const double rounds = (double)(((long long)tiles + 255) / 256);
  return rounds * bm * bn / rate;
}
constexpr double kRate256x96 = 1.20;   // 256 x 96, A in registers (Q/K/V only)
static int pick_tile(int M, int N) {   // 0: 128x128, 1: 256x128, 2: 256x256, 3: 256x192, 4: 128x192
  if (M <= 128) return 0;
  const double c[5] = {tile_cost(M, N, 128, 128, 0.80), tile_cost(M, N, 256, 128, 0.95),
                       tile_cost(M, N, 256, 256, 1.25), tile_cost(M, N, 256, 192, 1.30),
                       tile_cost(M, N, 128, 192, 0.90)};
  int best = 0;
  for (int i = 1; i < 5; ++i)
    if (c[i] < c[best]) best = i;
  return best;
}

// The A-in-registers loop is unrolled over its four register sets: K must be a whole number of four stages
// (32 wide in the 256 x 192 tile, 64 wide in the 256 x 96 one); the widths are those for which the RMSNorm has
// a kernel that writes the quad-tiled layout.  (The layout changes no arithmetic: a row's results are the same
// bits on either path.)  Only tiles whose wavefronts feed two A fragments to every K-step take it: gate/up at
// 512 rows 101 -> 90 us; with the single A fragment of the 128 x 192 tile, LDS traffic is nearly all B's and
// the register path gains nothing (Q/K/V at 512 rows: 77.3 -> 78.7 us).
static bool quad_tiled_widths(int K, int stage) { return K % (4 * stage) == 0 && K >= 2048 && K <= 8192; }
bool gemm_swiglu_a_quad_tiled(int M, int F, int K) { return pick_tile(M, 2 * F) == 3 && quad_tiled_widths(K, 64); }

// Q/K/V: besides the tiles of pick_tile, 256 x 96 with A in registers (EPI_QKV16): 512 rows x 12288 columns
// are 256 such tiles, one per CU, where 256 x 192 would occupy half the chip and 128 x 192 (one A fragment
// per wavefront) is bound by its LDS traffic.  Index 5.
static int pick_tile_qkv(int M, int N, int K, int Dh) {
  const int t = pick_tile(M, N);
  if (M <= 128 || !quad_tiled_widths(K, 64) || Dh % 32 != 0) return t;
  static const int bm[5] = {128, 256, 256, 256, 128}, bn[5] = {128, 128, 256, 192, 192};
  static const double rate[5] = {0.80, 0.95, 1.25, 1.30, 0.90};
  return tile_cost(M, N, 256, 96, kRate256x96) < tile_cost(M, N, bm[t], bn[t], rate[t]) ? 5 : t;
}
bool gemm_qkv_a_quad_tiled(int M, int d, int K, int Dh) {
  const int t = pick_tile_qkv(M, 3 * d, K, Dh);
  return t == 5 || (t == 3 && quad_tiled_widths(K, 64));
}

void launch_gemm_qkv_bf16(const bf16* A, const bf16* wq, const bf16* wk, const bf16* wv, int M, int K,
                          const QkvEpilogue& e, Gate g, hipStream_t s) {
  GemmArgs a = {};
  a.A = A; a.B0 = wq; a.B1 = wk; a.B2 = wv;
  a.M = M; a.N = 3 * e.d; a.K = K; a.splits = 1; a.gate = g; a.qkv = e;
  switch (pick_tile_qkv(M, a.N, K, e.Dh)) {
    case 5: launch<256, 96, 64, 4, 1, 4, EPI_QKV16, true>(a, s); break;
    case 4: launch<128, 192, 32, 4, 1, 4, EPI_QKV>(a, s); break;
    case 3:
      if (quad_tiled_widths(K, 64)) launch<256, 192, 64, 4, 1, 4, EPI_QKV, true>(a, s);
      else launch<256, 192, 32, 4, 1, 4, EPI_QKV>(a, s);
      break;
    case 2: launch<256, 256, 32, 4, 2, 4, EPI_QKV>(a, s); break;
    case 1: launch<256, 128, 32, 4, 2, 6, EPI_QKV>(a, s); break;
    default: launch<128, 128, 64, 2, 2, 4, EPI_QKV>(a, s);
  }
}

static bool partial_serial(int M, int N);
void launch_gemm_partial_bf16(const bf16* A, const bf16* W, float* parts, size_t part_stride, int M, int N, int K,
                              int splits, Gate g, hipStream_t s) {
  GemmArgs a = {};
  a.A = A; a.B0 = W; a.M = M; a.N = N; a.K = K; a.splits = splits; a.gate = g;
  a.parts = parts; a.part_stride = part_stride;
  if (gemm_partial_a_quad_tiled(M, N, K) && (splits == 4 || (splits == 1 && partial_serial(M, N)))) {
    if (splits == 1) {
      a.serial = 4;
      launch<256, 128, 64, 4, 1, 4, EPI_PARTIAL_SER, true>(a, s);
    } else {
      launch<256, 128, 64, 4, 1, 4, EPI_PARTIAL, true>(a, s);
    }
  } else if (splits == 1 && pick_tile(M, N) == 2) {
    launch<256, 256, 32, 4, 2, 4, EPI_PARTIAL>(a, s);
  } else {
    launch<128, 128, 64, 2, 2, 4, EPI_PARTIAL>(a, s);
  }
}

// Wide path, [d, d] and [d, F] projections: 128 x 128 tiles of these narrow outputs do not fill the
// chip at a few hundred rows, so K is split, each K range staying a multiple of the 64-wide stage and
// at least 512 long; the partials are folded by the next RMSNorm in order.  Above 256 rows the depth is
// a function of the widths alone (four ways with the A-in-registers tile below, else two ways whenever K
// allows it), never of the row count: a sequence must sum
// its projections in the same order whatever batch it is decoded in (full-recompute forwards of one
// sequence and of a batch then give the same bits row by row).  Up to 256 rows (batched block-only steps
// of the cached modes, bound by the weight stream) the split goes up to eight ways, until the launch
// has about 256 workgroups: 256 rows of the 8B shape split 4 ways, 128 rows 8 ways.
// Above 256 rows: 256 x 128 tiles with A in registers and K split four ways when the widths allow (512 rows of
// the 8B shape: 2 x 32 tiles x 4 = one workgroup per CU).  The tile has half the LDS traffic per MFMA of the
// 128 x 128 one (only B is staged, and a wavefront reuses each B fragment for two A fragments), which pays for
// the two extra partials: projection 45 -> 39 us, the RMSNorm that folds them 9.3 -> 11.8 us.
bool gemm_partial_a_quad_tiled(int M, int N, int K) {
  return M > 256 && N % 128 == 0 && K % 1024 == 0 && K / 4 >= 512 && N % 8 == 0;
}
// With about a tile per CU or more, four workgroups per tile buy no parallelism and cost three more partials
// to write and to fold (2048 rows of the 8B shape: projection 163 us and RMSNorm 43 us, against 157 and 28): one workgroup
// then walks the four K ranges itself and writes the one sum.  Same bits either way (GemmArgs::serial), so
// this may depend on the row count.
static bool partial_serial(int M, int N) { return ((M + 255) / 256) * ((N + 127) / 128) >= 224; }
int wide_splits(int M, int N, int K) {
  if (M > 256 && gemm_partial_a_quad_tiled(M, N, K)) return partial_serial(M, N) ? 1 : 4;
  if (M > 256) return (K % 128 == 0 && K / 2 >= 512) ? 2 : 1;
  const int tiles = ((M + 127) / 128) * ((N + 127) / 128);
  int S = 1;
  while (tiles * S < 256 && S < 8 && K % (S * 2 * 64) == 0 && K / (S * 2) >= 512) S *= 2;
  return S;
}

int skinny_splits(int N, int K) {
  const int tiles = (N + 127) / 128;
  int S = 1;
  while (tiles * S < 256 && S < 16 && K % (S * 2 * 64) == 0 && K / (S * 2) >= 256) S *= 2;
  return S;
}

// Few rows (a block-only step of the cached decode modes: 32 or 64 rows): every GEMM is bound by
// streaming its weights once, which needs several workgroups per CU with deep rings in flight.
// 32- or 64-row tiles, 128 columns, K split `splits` ways into fp32 partials; up to three weight
// matrices of n_sub rows each are stacked along N (Q/K/V, gate/up) so that one launch covers them.
// The nonlinear epilogues (RoPE, SwiGLU) run afterwards on the summed partials.
void launch_gemm_skinny_bf16(const bf16* A, const bf16* w0, const bf16* w1, const bf16* w2, int n_sub, float* parts,
                             size_t part_stride, int M, int N, int K, int splits, Gate g, hipStream_t s) {
  GemmArgs a = {};
  a.A = A; a.B0 = w0; a.B1 = w1; a.B2 = w2; a.n_sub = w1 ? n_sub : 0;
  a.M = M; a.N = N; a.K = K; a.splits = splits; a.gate = g;
  a.parts = parts; a.part_stride = part_stride;
  if (M <= 32) launch<32, 128, 64, 1, 4, 4, EPI_PARTIAL>(a, s);
  else launch<64, 128, 64, 2, 2, 4, EPI_PARTIAL>(a, s);
}

// Few rows and a wide FFN: 64 (32 gate + 32 up) columns per workgroup already make a few hundred
// workgroups, so the weights stream once without splitting K and SwiGLU stays in the epilogue
// (measured against split-K partials plus a finishing kernel, weights coming from HBM: 40.6 us
// against 44.1 + 4.6 us at 32 rows, 43.5 against 51.4 + 4.6 us at 64 rows, d_model 4096, d_ffn 12288).
bool swiglu_few_rows_fused(int M, int F) { return M <= kSkinnyRows && F % 64 == 0 && 2 * F / 64 >= 256; }

void launch_gemm_swiglu_bf16(const bf16* A, const bf16* wg, const bf16* wu, bf16* act, int M, int F, int K, Gate g,
                             hipStream_t s, bool act_quad_tiled) {
  GemmArgs a = {};
  a.A = A; a.B0 = wg; a.B1 = wu; a.M = M; a.N = 2 * F; a.K = K; a.splits = 1; a.gate = g;
  a.act = act; a.F = F; a.act_quad_tiled = (act_quad_tiled && F % 8 == 0) ? 1 : 0;
  if (swiglu_few_rows_fused(M, F)) {
    if (M <= 32) launch<32, 64, 64, 1, 1, 6, EPI_SWIGLU>(a, s);   // one wavefront per workgroup, 72 KB ring
    else launch<64, 128, 64, 2, 2, 4, EPI_SWIGLU>(a, s);
    return;
  }
  switch (pick_tile(M, a.N)) {
    case 4: launch<128, 192, 32, 4, 1, 4, EPI_SWIGLU>(a, s); break;
    case 3:
      if (quad_tiled_widths(K, 64)) launch<256, 192, 64, 4, 1, 4, EPI_SWIGLU, true>(a, s);
      else launch<256, 192, 32, 4, 1, 4, EPI_SWIGLU>(a, s);
      break;
    case 2: launch<256, 256, 32, 4, 2, 4, EPI_SWIGLU>(a, s); break;
    case 1: launch<256, 128, 32, 4, 2, 6, EPI_SWIGLU>(a, s); break;
    default: launch<128, 128, 64, 2, 2, 4, EPI_SWIGLU>(a, s);
  }
}

int lmhead_n_part(int V) { return (V + 127) / 128; }
bool gemm_lmhead_a_quad_tiled(int M, int V, int K) { (void)V; return M > 128 && quad_tiled_widths(K, 64); }

void launch_gemm_lmhead_bf16(const bf16* A, const bf16* W, int M, int V, int K, const LmHeadEpilogue& e, Gate g,
                             hipStream_t s) {
  GemmArgs a = {};
  a.A = A; a.B0 = W; a.M = M; a.N = V; a.K = K; a.splits = 1; a.gate = g; a.lm = e;
  // 128 columns per tile in every configuration: the partial (max, sum, argmax) triples are per 128 logits
  if (M <= 32)
    launch<32, 128, 64, 1, 4, 4, EPI_LMHEAD>(a, s);
  else if (M <= 128)
    launch<128, 128, 64, 2, 2, 4, EPI_LMHEAD>(a, s);
  else if (gemm_lmhead_a_quad_tiled(M, V, K))
    launch<256, 128, 64, 4, 1, 4, EPI_LMHEAD, true>(a, s);   // batched blocks: compute bound, A from registers
  else
    launch<256, 128, 32, 4, 2, 6, EPI_LMHEAD>(a, s);   // the 1 GB of weights is read once per 256 rows
}

}  // namespace l2pd
