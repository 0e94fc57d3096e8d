// Bidirectional (non-causal) flash-style attention on bf16 MFMA for gfx950.
//
// Inputs are what the QKV GEMM epilogue leaves: rotated queries q [B*Tq, d], rotated keys
// kstore [B, Tpad, d] and transposed values vtstore [B, H, Dh, Tpad].  A workgroup owns 32*NQ
// queries of one (sequence, head) and splits the keys into NSPL contiguous ranges; wavefront
// (query group, key range) runs the online softmax of its 32 queries over its range, and the
// ranges are merged at the end.  Key/value tiles of 64 keys are staged in LDS (XOR-swizzled rows,
// NST buffers per range; the next tile waits in registers meanwhile), one tile per range and
// iteration, shared by the query groups.
//
// The wave computes S^T = K Q^T (keys are MFMA rows, queries are columns), so that a lane holds
// scores of ONE query: the row maximum is 31 register maxima plus one cross-lane exchange, and the
// exponentiated scores are already laid out as the B operand of O^T = V^T P^T.  The key order
// inside each 16-key MFMA step is the accumulator's (keys {4h..4h+3, 8+4h..8+4h+3} for lane half h);
// V^T is read from LDS in that same order, which is legal because the contraction is a sum.
#include "common.h"

namespace l2pd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi) {   // v_cvt_pk_bf16_f32, round to nearest even
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2_t));
}

template <int DH, int NQ, int NSPL, int NST>
__global__ void __launch_bounds__(NQ * NSPL * 64) k_attn_bf16(const bf16* __restrict__ q, const bf16* __restrict__ kstore,
                                                              const bf16* __restrict__ vtstore, bf16* __restrict__ out,
                                                              int B, int Tq, int Tk_all, int Tpad, int H, int n_chunks,
                                                              float* __restrict__ chunk_out,
                                                              const int* __restrict__ tk_dev, int out_quad_tiled, Gate g) {
  if (gate_skip(g)) return;
  constexpr int NW = NQ * NSPL;
  constexpr int NT = NW * 64;
  constexpr int KT = 64;                       // keys per LDS tile
  constexpr int K_ROW = DH * 2;                // bytes per key row
  constexpr int K_BYTES = KT * K_ROW;
  constexpr int V_BYTES = DH * KT * 2;         // [DH rows][64 keys]
  constexpr int STAGE = K_BYTES + V_BYTES;
  constexpr int KCH = K_BYTES / 16 / NT, VCH = V_BYTES / 16 / NT;
  static_assert(KCH * NT * 16 == K_BYTES && VCH * NT * 16 == V_BYTES, "tile/threads mismatch");
  constexpr int KK = DH / 16;                  // MFMA steps over the feature dim
  constexpr int FO = DH / 32;                  // output row fragments
  constexpr int XW = FO * 16 + 2;              // floats a wave hands over per lane: O^T fragments, m, l
  static_assert(NST == 1 || NST == 2, "tile buffers are single or double");
  // the exchange area of the final merge reuses the tile buffers; the launch sizes LDS for the larger of the two
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [NST stages][NSPL key ranges][K tile | V^T tile]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, lj = lane & 31;
  const int qg = wave % NQ, sp = wave / NQ;    // query group and key range of this wavefront
  // Workgroups are dealt to the 8 XCDs round-robin by their linear id.  All query tiles of one
  // (sequence, head) read the same K / V^T, so they are given ids that land on one XCD and share
  // its L2 (T = 512: 1 MB of K/V per XCD instead of all 8 MB through every L2).
  const int per_head = gridDim.x / (H * B);     // query tiles x key chunks
  int hb, inner;
  if ((H * B) % 8 == 0) {
    const int slot = blockIdx.x >> 3;
    hb = (slot / per_head) * 8 + (blockIdx.x & 7);
    inner = slot % per_head;
  } else {
    hb = blockIdx.x / per_head;
    inner = blockIdx.x % per_head;
  }
  const int b = hb / H, h = hb % H;
  // per-sequence key count (sequences shortened by step-granular EoTP), else the launch's
  const int Tk = tk_dev ? min(Tk_all, tk_dev[b]) : Tk_all;
  const int d = H * DH;
  // With n_chunks > 1 the keys are also dealt to n_chunks workgroups per query tile (few queries,
  // many keys: one workgroup per head would leave most CUs idle); each writes its unnormalised
  // (O^T, m, l) to chunk_out and k_attn_merge combines them.
  const int qt = inner / n_chunks, ch = inner % n_chunks;
  const int q0 = qt * (32 * NQ) + qg * 32;
  const int qrow = min(q0 + lj, Tq - 1);

  // Q as the B operand: lane (query lj, half hf) holds features kk*16 + hf*8 .. +7
  bf16x8_t fq[KK];
  {
    const bf16* qp = q + ((size_t)b * Tq + qrow) * d + h * DH + hf * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) fq[kk] = *reinterpret_cast<const bf16x8_t*>(qp + kk * 16);
  }

  const bf16* kbase = kstore + (size_t)b * Tpad * d + h * DH;
  const bf16* vbase = vtstore + (size_t)(b * H + h) * DH * Tpad;
  // LDS swizzle: the 64 banks sweep 256 bytes.  A K row is 256 B (DH = 128: key = row & 15 over its
  // 16 chunks) or 128 B (DH = 64: two rows per sweep, key = (row >> 1) & 7); a V^T row is 128 B.
  auto kkey = [](int r) { return DH == 128 ? (r & 15) : ((r >> 1) & 7); };
  const bf16* srcK[KCH];
  int dstK[KCH];
#pragma unroll
  for (int i = 0; i < KCH; ++i) {
    int c = tid + i * NT;
    int r = c / (DH / 8), cc = c % (DH / 8);
    srcK[i] = kbase + (size_t)r * d + cc * 8;
    dstK[i] = r * K_ROW + ((cc ^ kkey(r)) << 4);
  }
  const bf16* srcV[VCH];
  int dstV[VCH];
#pragma unroll
  for (int i = 0; i < VCH; ++i) {
    int c = tid + i * NT;
    int r = c >> 3, cc = c & 7;
    srcV[i] = vbase + (size_t)r * Tpad + cc * 8;
    dstV[i] = K_BYTES + r * (KT * 2) + ((cc ^ ((r >> 1) & 7)) << 4);
  }
  // The key tiles are dealt to the NSPL key ranges in contiguous runs of `per` tiles; every range
  // is walked by NQ wavefronts (one per query group), and all ranges advance together, one tile
  // per iteration, so the dependent chain of a wavefront is `per` tiles long instead of n_tiles.
  const int n_tiles = (Tk + KT - 1) / KT;
  const int per_chunk = (n_tiles + n_chunks - 1) / n_chunks;    // the host picks n_chunks so that no chunk is empty
  const int wg_first = ch * per_chunk, wg_count = min(per_chunk, n_tiles - wg_first);
  const int per = (wg_count + NSPL - 1) / NSPL;
  u32x4 rk[NSPL][KCH], rv[NSPL][VCH];
  auto gload = [&](int it) {
#pragma unroll
    for (int x = 0; x < NSPL; ++x) {
      const int k0 = min(wg_first + x * per + it, n_tiles - 1) * KT;   // ranges that have run out re-read a valid tile
#pragma unroll
      for (int i = 0; i < KCH; ++i) rk[x][i] = *reinterpret_cast<const u32x4*>(srcK[i] + (size_t)k0 * d);
#pragma unroll
      for (int i = 0; i < VCH; ++i) rv[x][i] = *reinterpret_cast<const u32x4*>(srcV[i] + k0);
    }
  };
  auto sstore = [&](int stage) {
#pragma unroll
    for (int x = 0; x < NSPL; ++x) {
      unsigned char* base = smem + ((NST == 2 ? stage : 0) * NSPL + x) * STAGE;
#pragma unroll
      for (int i = 0; i < KCH; ++i) *reinterpret_cast<u32x4*>(base + dstK[i]) = rk[x][i];
#pragma unroll
      for (int i = 0; i < VCH; ++i) *reinterpret_cast<u32x4*>(base + dstV[i]) = rv[x][i];
    }
  };

  f32x16 o[FO];
#pragma unroll
  for (int f = 0; f < FO; ++f)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[f][r] = 0.f;
  float m = -INFINITY, lsum = 0.f;
  const float sc = rsqrtf((float)DH) * 1.4426950408889634f;   // softmax scale folded with log2(e)
  const int keyK = kkey(lj), keyV = (lj >> 1) & 7;   // fragment rows are lj modulo 32
  const int my_first = wg_first + sp * per, my_count = max(0, min(per, wg_first + wg_count - my_first));

  gload(0);
  sstore(0);
  __syncthreads();
  for (int t = 0; t < per; ++t) {
    const bool more = t + 1 < per;
    if (more) gload(t + 1);
    if (t < my_count) {
      const unsigned char* base = smem + ((NST == 2 ? (t & 1) : 0) * NSPL + sp) * STAGE;
      const int k0 = (my_first + t) * KT;

      // S^T for the two 32-key halves of the tile
      f32x16 s[2];
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
        const unsigned char* krow = base + (sub * 32 + lj) * K_ROW;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          bf16x8_t fk = *reinterpret_cast<const bf16x8_t*>(krow + (((kk * 2 + hf) ^ keyK) << 4));
          s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk, fq[kk], s[sub], 0, 0, 0);
        }
      }
      float tmax = -INFINITY;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int kidx = k0 + sub * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
          float v = kidx < Tk ? s[sub][r] * sc : -INFINITY;
          s[sub][r] = v;
          tmax = fmaxf(tmax, v);
        }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float mn = fmaxf(m, tmax);
      const float alpha = __builtin_amdgcn_exp2f(m - mn);       // m = -inf on the first tile gives 0
      m = mn;
      float ps = 0.f;
      unsigned int pk[2][8];                   // bf16 pairs: [sub][4 per 16-key step * 2 steps]
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          // v_exp_f32 directly: arguments are <= 0, and a result below the normal range may flush to zero
          float p0 = __builtin_amdgcn_exp2f(s[sub][r] - mn), p1 = __builtin_amdgcn_exp2f(s[sub][r + 1] - mn);
          ps += p0 + p1;
          pk[sub][r >> 1] = pack_bf16x2(p0, p1);
        }
      lsum = lsum * alpha + ps;
#pragma unroll
      for (int f = 0; f < FO; ++f)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[f][r] *= alpha;

      // O^T += V^T P^T, 16 keys per MFMA
#pragma unroll
      for (int m16 = 0; m16 < 4; ++m16) {
        const int sub = m16 >> 1, mm = m16 & 1;
        u32x4 pw = {pk[sub][mm * 4 + 0], pk[sub][mm * 4 + 1], pk[sub][mm * 4 + 2], pk[sub][mm * 4 + 3]};
        bf16x8_t fp = __builtin_bit_cast(bf16x8_t, pw);
#pragma unroll
        for (int f = 0; f < FO; ++f) {
          const unsigned char* vrow = base + K_BYTES + (f * 32 + lj) * (KT * 2) + hf * 8;
          u32x2 v0 = *reinterpret_cast<const u32x2*>(vrow + (((m16 * 2) ^ keyV) << 4));
          u32x2 v1 = *reinterpret_cast<const u32x2*>(vrow + (((m16 * 2 + 1) ^ keyV) << 4));
          u32x4 vw = {v0.x, v0.y, v1.x, v1.y};
          bf16x8_t fv = __builtin_bit_cast(bf16x8_t, vw);
          o[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv, fp, o[f], 0, 0, 0);
        }
      }
    }
    if constexpr (NST == 1) __syncthreads();   // single buffer: every wavefront is done with the tiles before the refill
    if (more) sstore((t + 1) & 1);
    __syncthreads();
  }

  // Merge the key ranges: range 0 of each query group folds in the others' (m, l, O^T), in range
  // order, through the tile buffers (dead now).  A range without keys hands over m = -inf, l = 0.
  if constexpr (NSPL > 1) {
    float* xch = reinterpret_cast<float*>(smem);
    if (sp > 0) {
      float* mine = xch + (size_t)((sp - 1) * NQ + qg) * XW * 64 + lane;
#pragma unroll
      for (int f = 0; f < FO; ++f)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[(f * 16 + r) * 64] = o[f][r];
      mine[(FO * 16) * 64] = m;
      mine[(FO * 16 + 1) * 64] = lsum;
    }
    __syncthreads();
    if (sp > 0) return;
#pragma unroll
    for (int x = 1; x < NSPL; ++x) {
      const float* oth = xch + (size_t)((x - 1) * NQ + qg) * XW * 64 + lane;
      const float m2 = oth[(FO * 16) * 64], l2 = oth[(FO * 16 + 1) * 64];
      const float M = fmaxf(m, m2);   // m is finite: range 0 always holds the first tile
      const float a1 = __builtin_amdgcn_exp2f(m - M), a2 = __builtin_amdgcn_exp2f(m2 - M);
#pragma unroll
      for (int f = 0; f < FO; ++f)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[f][r] = o[f][r] * a1 + oth[(f * 16 + r) * 64] * a2;
      lsum = lsum * a1 + l2 * a2;
      m = M;
    }
  }

  const float l = lsum + __shfl_xor(lsum, 32, 64);
  if (n_chunks > 1) {
    if (q0 + lj < Tq) {
      float* po = chunk_out + ((((size_t)b * H + h) * Tq + q0 + lj) * n_chunks + ch) * (DH + 2);
#pragma unroll
      for (int f = 0; f < FO; ++f)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq)
          *reinterpret_cast<float4*>(po + f * 32 + rq * 8 + hf * 4) =
              make_float4(o[f][rq * 4 + 0], o[f][rq * 4 + 1], o[f][rq * 4 + 2], o[f][rq * 4 + 3]);
      if (hf == 0) { po[DH] = m; po[DH + 1] = l; }
    }
    return;
  }
  const float inv = 1.f / l;
  if (q0 + lj < Tq) {
    // row-major [rows, d], or the quad-tiled layout the output projection reads into registers
    // (gemm_qkv_a_quad_tiled in common.h describes it): four features are half a 16-byte chunk either way
    const size_t row = (size_t)b * Tq + q0 + lj;
    unsigned short* op = reinterpret_cast<unsigned short*>(out) +
                         (out_quad_tiled ? ((row >> 2) * (d / 8) + h * (DH / 8)) * 32 + (row & 3) * 8 : row * d + h * DH);
#pragma unroll
    for (int f = 0; f < FO; ++f)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        u32x2 w;
        w.x = pack_bf16x2(o[f][rq * 4 + 0] * inv, o[f][rq * 4 + 1] * inv);
        w.y = pack_bf16x2(o[f][rq * 4 + 2] * inv, o[f][rq * 4 + 3] * inv);
        const int col = f * 32 + rq * 8 + hf * 4;   // feature within the head
        *reinterpret_cast<u32x2*>(op + (out_quad_tiled ? (col >> 3) * 32 + (col & 7) : col)) = w;
      }
  }
}

// One thread per (sequence, head, query, 4 features): combines the key chunks in ascending order.
template <int DH>
__global__ void __launch_bounds__(256) k_attn_merge(const float* __restrict__ chunk_out, bf16* __restrict__ out, int B,
                                                   int Tq, int H, int n_chunks, Gate g) {
  if (gate_skip(g)) return;
  const int t = blockIdx.x * 256 + threadIdx.x;
  const int per_q = DH / 4;
  if (t >= B * H * Tq * per_q) return;
  const int f4 = t % per_q, qi = (t / per_q) % Tq, h = (t / per_q / Tq) % H, b = t / per_q / Tq / H;
  const float* p = chunk_out + ((((size_t)b * H + h) * Tq + qi) * n_chunks) * (DH + 2);
  float M = -INFINITY;
  for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, p[c * (DH + 2) + DH]);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float L = 0.f;
  for (int c = 0; c < n_chunks; ++c) {
    const float w = __builtin_amdgcn_exp2f(p[c * (DH + 2) + DH] - M);
    const float4 v = *reinterpret_cast<const float4*>(p + c * (DH + 2) + f4 * 4);
    acc.x += v.x * w; acc.y += v.y * w; acc.z += v.z * w; acc.w += v.w * w;
    L += p[c * (DH + 2) + DH + 1] * w;
  }
  const float inv = 1.f / L;
  u32x2 w2;
  w2.x = pack_bf16x2(acc.x * inv, acc.y * inv);
  w2.y = pack_bf16x2(acc.z * inv, acc.w * inv);
  unsigned short* op = reinterpret_cast<unsigned short*>(out) + ((size_t)b * Tq + qi) * (H * DH) + h * DH + f4 * 4;
  *reinterpret_cast<u32x2*>(op) = w2;
}

template <int DH, int NQ, int NSPL, int NST>
static void launch(const bf16* q, const bf16* kstore, const bf16* vtstore, bf16* out, int B, int Tq, int Tk,
                   int Tpad, int H, float* chunk_ws, size_t chunk_ws_bytes, const int* tk_dev, Gate g, hipStream_t s,
                   bool out_quad_tiled) {
  auto kern = k_attn_bf16<DH, NQ, NSPL, NST>;
  constexpr int tiles = NST * NSPL * (64 * DH * 2 + DH * 64 * 2);
  constexpr int xchg = (NSPL - 1) * NQ * ((DH / 32) * 16 + 2) * 64 * 4;
  constexpr int smem = tiles > xchg ? tiles : xchg;
  static DynLdsAttr attr;
  attr.ensure(reinterpret_cast<const void*>(kern), smem);
  const int q_tiles = (Tq + 32 * NQ - 1) / (32 * NQ), n_tiles = (Tk + 63) / 64;
  // few queries against many keys: deal the key tiles to several workgroups per query tile
  int n_chunks = 1;
  if (chunk_ws && !tk_dev && !out_quad_tiled && q_tiles * H * B < 128 && n_tiles >= 2 * NSPL) {   // chunks must not be empty: launch-wide key count only; the merge writes row-major
    int want = (256 + q_tiles * H * B - 1) / (q_tiles * H * B);
    if (want > 16) want = 16;
    if (want > n_tiles / NSPL) want = n_tiles / NSPL;   // a tile for every key range of a chunk
    const int per_chunk = (n_tiles + want - 1) / want;
    n_chunks = (n_tiles + per_chunk - 1) / per_chunk;       // every chunk gets at least one tile
    if ((size_t)B * H * Tq * n_chunks * (DH + 2) * 4 > chunk_ws_bytes) n_chunks = 1;
  }
  dim3 grid(q_tiles * n_chunks * H * B);
  hipLaunchKernelGGL(kern, grid, dim3(NQ * NSPL * 64), smem, s, q, kstore, vtstore, out, B, Tq, Tk, Tpad, H, n_chunks,
                     chunk_ws, tk_dev, out_quad_tiled ? 1 : 0, g);
  if (n_chunks > 1) {
    const int n = B * H * Tq * (DH / 4);
    hipLaunchKernelGGL(k_attn_merge<DH>, dim3((n + 255) / 256), dim3(256), 0, s, chunk_ws, out, B, Tq, H, n_chunks, g);
  }
}

// 64 queries per workgroup, keys in four ranges, single-buffered tiles (128 KB of LDS at head size
// 128): with one sequence of a few hundred tokens this gives a workgroup to every CU, two wavefronts
// to every SIMD and a short chain of dependent key tiles per wavefront.  Measured at 32 heads of 128
// (us, 512 / 1280 / 4096 tokens): two ranges double-buffered 15.9 / 93.5 / 756, four ranges
// single-buffered 14.4 / 71.9 / 521; before the XCD-aware workgroup ids the first was 21.5.  The
// configuration depends on the head size, the head count and the query rows per sequence, and the
// chunking across workgroups on the shape of the launch, never on the data.
void launch_attn_bf16(const bf16* q, const bf16* kstore, const bf16* vtstore, bf16* out, int B, int Tq, int Tk,
                      int Tpad, int H, int Dh, float* chunk_ws, size_t chunk_ws_bytes, const int* tk_dev, Gate g,
                      hipStream_t s, bool out_quad_tiled) {
  // A sequence long enough to give every CU a workgroup of 128 queries by itself: the key tiles
  // then serve four query groups instead of two (half the L2 -> LDS traffic per flop) and two
  // workgroups of 64 KB fit a CU.  Measured at 32 heads of 128, one sequence (us): 1024 tokens
  // 40.5 -> 27.8, 2048 tokens 141 -> 99, 4096 tokens 520 -> 375.  The batch size is left out of the
  // criterion on purpose: the two configurations merge key ranges in different orders, and a row's
  // result must not depend on the batch it is part of.
  if ((long long)((Tq + 127) / 128) * H >= 256) {
    if (Dh == 128) launch<128, 4, 2, 1>(q, kstore, vtstore, out, B, Tq, Tk, Tpad, H, chunk_ws, chunk_ws_bytes, tk_dev, g, s, out_quad_tiled);
    else launch<64, 4, 2, 1>(q, kstore, vtstore, out, B, Tq, Tk, Tpad, H, chunk_ws, chunk_ws_bytes, tk_dev, g, s, out_quad_tiled);
    return;
  }
  if (Dh == 128) launch<128, 2, 4, 1>(q, kstore, vtstore, out, B, Tq, Tk, Tpad, H, chunk_ws, chunk_ws_bytes, tk_dev, g, s, out_quad_tiled);
  else launch<64, 2, 4, 1>(q, kstore, vtstore, out, B, Tq, Tk, Tpad, H, chunk_ws, chunk_ws_bytes, tk_dev, g, s, out_quad_tiled);
}

}  // namespace l2pd
