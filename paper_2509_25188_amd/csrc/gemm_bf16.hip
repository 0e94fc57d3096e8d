// bf16 MFMA GEMM for gfx950:  C[M, N] = A[M, K] * W[N, K]^T, fp32 accumulation.
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants: a lane feeds
// eight consecutive K elements of one row.  Tiles go global -> LDS with 16-byte accesses; the LDS
// rows (128 B = one bank sweep) are XOR-swizzled at 16-byte granularity so that the 32 rows a
// wavefront reads together spread over all banks.  The fused epilogues are the ones the decoding
// step needs: rotary embedding + K / V^T store (QKV), SiLU(gate) * up (FFN), fp32 split-K partials
// that the next RMSNorm folds into the residual stream (O and down projections), and the LM head's
// per-tile (max, sum exp, argmax) reduction so that logits are never written.
//
// "Pair" epilogues need two columns in one lane (feature i and i + Dh/2 for the rotation, gate and
// up column for SwiGLU).  That is arranged by the order in which weight rows are placed in the LDS
// tile: fragment 2p of a wave holds side 0 and fragment 2p+1 side 1 of the same 32 columns.
#include "common.h"

namespace l2pd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int BK = 64;  // K elements per LDS tile row: 128 bytes
enum { EPI_PARTIAL = 0, EPI_QKV = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3 };

struct GemmArgs {
  const bf16* A;
  const bf16* B0;
  const bf16* B1;
  const bf16* B2;
  int M, N, K;          // N counts tile-space columns (for pair epilogues: both sides)
  int tiles_m, tiles_n, splits;
  Gate gate;
  // EPI_PARTIAL
  float* part0;
  float* part1;
  // EPI_SWIGLU
  bf16* act;
  int F;
  // EPI_QKV
  QkvEpilogue qkv;
  // EPI_LMHEAD
  LmHeadEpilogue lm;
};

__device__ __forceinline__ unsigned short f2bf(float f) {   // round to nearest even
  unsigned int u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ void __launch_bounds__(WM* WN * 64) k_gemm_bf16(GemmArgs a) {
  constexpr int NT = WM * WN * 64;
  constexpr int FM = BM / WM / 32, FN = BN / WN / 32;
  constexpr bool PAIR = (EPI == EPI_QKV || EPI == EPI_SWIGLU);
  static_assert(!PAIR || (FN % 2 == 0), "pair epilogues need an even number of column fragments");
  constexpr int CH_A = BM * 8 / NT, CH_B = BN * 8 / NT;   // 16-byte chunks per thread per tile
  static_assert(CH_A * NT == BM * 8 && CH_B * NT == BN * 8, "tile/threads mismatch");

  if (gate_skip(a.gate)) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // [stage][A: BM rows | B: BN rows][64 bf16]
  constexpr int STAGE_BYTES = (BM + BN) * BK * 2;

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

  // ---- per-thread source pointers for the global -> LDS copies (fixed over the K loop) ----
  const bf16* srcA[CH_A];
  int dstA[CH_A];
#pragma unroll
  for (int i = 0; i < CH_A; ++i) {
    int q = tid + i * NT;
    int r = q >> 3, c = q & 7;
    int gr = min(m0 + r, a.M - 1);
    srcA[i] = a.A + (size_t)gr * a.K + k_begin + c * 8;
    dstA[i] = r * (BK * 2) + ((c ^ (r & 7)) << 4);
  }
  const bf16* srcB[CH_B];
  int dstB[CH_B];
#pragma unroll
  for (int i = 0; i < CH_B; ++i) {
    int q = tid + i * NT;
    int r = q >> 3, c = q & 7;
    const bf16* base;
    size_t grow;
    if constexpr (!PAIR) {
      base = a.B0;
      grow = (size_t)min(n0 + r, a.N - 1);
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
    srcB[i] = base + grow * a.K + k_begin + c * 8;
    dstB[i] = BM * (BK * 2) + r * (BK * 2) + ((c ^ (r & 7)) << 4);
  }

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 ra[CH_A], rb[CH_B];
  auto gload = [&](int kt) {
#pragma unroll
    for (int i = 0; i < CH_A; ++i) ra[i] = *reinterpret_cast<const u32x4*>(srcA[i] + kt * BK);
#pragma unroll
    for (int i = 0; i < CH_B; ++i) rb[i] = *reinterpret_cast<const u32x4*>(srcB[i] + kt * BK);
  };
  auto sstore = [&](int stage) {
    unsigned char* base = smem + stage * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < CH_A; ++i) *reinterpret_cast<u32x4*>(base + dstA[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < CH_B; ++i) *reinterpret_cast<u32x4*>(base + dstB[i]) = rb[i];
  };

  // fragment row byte offsets inside a stage (row * 128) and the row's swizzle key
  int offA[FM], offB[FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) offA[i] = (wm * (BM / WM) + i * 32 + lj) * (BK * 2);
#pragma unroll
  for (int j = 0; j < FN; ++j) offB[j] = BM * (BK * 2) + (wn * (BN / WN) + j * 32 + lj) * (BK * 2);
  const int key = lj & 7;   // all fragment rows are lj mod 8 (fragment bases are multiples of 32)

  gload(0);
  sstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const bool more = kt + 1 < nk;
    if (more) gload(kt + 1);
    const unsigned char* base = smem + (kt & 1) * STAGE_BYTES;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int sw = ((kk * 2 + hf) ^ key) << 4;
      bf16x8_t fa[FM], fb[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) fa[i] = *reinterpret_cast<const bf16x8_t*>(base + offA[i] + sw);
#pragma unroll
      for (int j = 0; j < FN; ++j) fb[j] = *reinterpret_cast<const bf16x8_t*>(base + offB[j] + sw);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (more) sstore((kt + 1) & 1);
    __syncthreads();
  }

  // ------------------------------------------------------------------------------------------
  // C layout of the 32x32 MFMA: register r of a lane is row (r/4)*8 + hf*4 + r%4, column lj.
  const int row_base = m0 + wm * (BM / WM);
  if constexpr (EPI == EPI_PARTIAL) {
    float* out = z == 0 ? a.part0 : a.part1;
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
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int p = 0; p < FN / 2; ++p) {
        int G = tile_n * (BN / 64) + wn * (FN / 2) + p;
        int col = G * 32 + lj;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int row = row_base + i * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
          float gt = acc[i][2 * p][r], up = acc[i][2 * p + 1][r];
          float v = gt / (1.f + __expf(-gt)) * up;
          if (row < a.M && col < a.F)
            reinterpret_cast<unsigned short*>(a.act)[(size_t)row * a.F + col] = f2bf(v);
        }
      }
  } else if constexpr (EPI == EPI_QKV) {
    const QkvEpilogue& e = a.qkv;
    const int half = e.Dh / 2, gph = half / 32;
    const bool vec4 = (e.Tq % 4 == 0) && (e.pos0 % 4 == 0) && (e.Tpad % 4 == 0);
#pragma unroll
    for (int p = 0; p < FN / 2; ++p) {
      int G = tile_n * (BN / 64) + wn * (FN / 2) + p;
      int hg = G / gph, gi = G % gph;
      int mat = hg / e.H, head = hg % e.H;
      if (mat > 2) continue;
      int dim = gi * 32 + lj;   // first-half feature index; partner is dim + half
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        if (mat == 2) {
          // V is stored transposed ([B, H, Dh, Tpad]) so that attention reads keys contiguously
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            int row0 = row_base + i * 32 + rq * 8 + hf * 4;
            if (vec4 && row0 + 3 < a.M) {
              int b = row0 / e.Tq, pos = e.pos0 + row0 % e.Tq;
              size_t o = ((size_t)(b * e.H + head) * e.Dh + dim) * e.Tpad + pos;
              unsigned short* vt = reinterpret_cast<unsigned short*>(e.vtstore);
              ushort4 lo4, hi4;
              lo4.x = f2bf(acc[i][2 * p][rq * 4 + 0]); lo4.y = f2bf(acc[i][2 * p][rq * 4 + 1]);
              lo4.z = f2bf(acc[i][2 * p][rq * 4 + 2]); lo4.w = f2bf(acc[i][2 * p][rq * 4 + 3]);
              hi4.x = f2bf(acc[i][2 * p + 1][rq * 4 + 0]); hi4.y = f2bf(acc[i][2 * p + 1][rq * 4 + 1]);
              hi4.z = f2bf(acc[i][2 * p + 1][rq * 4 + 2]); hi4.w = f2bf(acc[i][2 * p + 1][rq * 4 + 3]);
              *reinterpret_cast<ushort4*>(vt + o) = lo4;
              *reinterpret_cast<ushort4*>(vt + o + (size_t)half * e.Tpad) = hi4;
            } else {
#pragma unroll
              for (int rr = 0; rr < 4; ++rr) {
                int row = row0 + rr;
                if (row >= a.M) continue;
                int b = row / e.Tq, pos = e.pos0 + row % e.Tq;
                size_t o = ((size_t)(b * e.H + head) * e.Dh + dim) * e.Tpad + pos;
                unsigned short* vt = reinterpret_cast<unsigned short*>(e.vtstore);
                vt[o] = f2bf(acc[i][2 * p][rq * 4 + rr]);
                vt[o + (size_t)half * e.Tpad] = f2bf(acc[i][2 * p + 1][rq * 4 + rr]);
              }
            }
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            int row = row_base + i * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
            if (row >= a.M) continue;
            int b = row / e.Tq, pos = e.pos0 + row % e.Tq;
            float cs = e.cos_t[(size_t)pos * half + dim], sn = e.sin_t[(size_t)pos * half + dim];
            float x1 = acc[i][2 * p][r], x2 = acc[i][2 * p + 1][r];
            float o1 = x1 * cs - x2 * sn, o2 = x2 * cs + x1 * sn;
            unsigned short* dst;
            size_t o;
            if (mat == 0) {
              dst = reinterpret_cast<unsigned short*>(e.q);
              o = (size_t)row * e.d + head * e.Dh + dim;
            } else {
              dst = reinterpret_cast<unsigned short*>(e.kstore);
              o = ((size_t)b * e.Tpad + pos) * e.d + head * e.Dh + dim;
            }
            dst[o] = f2bf(o1);
            dst[o + half] = f2bf(o2);
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
    const int gb = (e.bias.value != 0.f && a.gate.ctl) ? a.gate.ctl[CTL_GB] : 0;
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
          if (e.bias.value != 0.f && col == e.bias.token_id &&
              gb * e.bias.block_len + (row % e.bias.block_len) >= e.bias.gen_pos_from)
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
template <int BM, int BN, int WM, int WN, int EPI>
static void launch(GemmArgs& a, hipStream_t s) {
  auto kern = k_gemm_bf16<BM, BN, WM, WN, EPI>;
  constexpr int smem = 2 * (BM + BN) * BK * 2;
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    attr_done = true;
  }
  a.tiles_m = (a.M + BM - 1) / BM;
  a.tiles_n = (a.N + BN - 1) / BN;
  int total = a.tiles_m * a.tiles_n * a.splits;
  int grid = ((total + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), smem, s, a);
}

void launch_gemm_qkv_bf16(const bf16* A, const bf16* wq, const bf16* wk, const bf16* wv, int M, int K,
                          const QkvEpilogue& e, Gate g, hipStream_t s) {
  GemmArgs a = {};
  a.A = A; a.B0 = wq; a.B1 = wk; a.B2 = wv;
  a.M = M; a.N = 3 * e.d; a.K = K; a.splits = 1; a.gate = g; a.qkv = e;
  launch<128, 128, 2, 2, EPI_QKV>(a, s);
}

void launch_gemm_partial_bf16(const bf16* A, const bf16* W, float* part0, float* part1, int M, int N, int K,
                              int splits, Gate g, hipStream_t s) {
  GemmArgs a = {};
  a.A = A; a.B0 = W; a.M = M; a.N = N; a.K = K; a.splits = splits; a.gate = g;
  a.part0 = part0; a.part1 = part1;
  launch<128, 128, 2, 2, EPI_PARTIAL>(a, s);
}

void launch_gemm_swiglu_bf16(const bf16* A, const bf16* wg, const bf16* wu, bf16* act, int M, int F, int K, Gate g,
                             hipStream_t s) {
  GemmArgs a = {};
  a.A = A; a.B0 = wg; a.B1 = wu; a.M = M; a.N = 2 * F; a.K = K; a.splits = 1; a.gate = g;
  a.act = act; a.F = F;
  launch<128, 128, 2, 2, EPI_SWIGLU>(a, s);
}

int lmhead_n_part(int V) { return (V + 127) / 128; }

void launch_gemm_lmhead_bf16(const bf16* A, const bf16* W, int M, int V, int K, const LmHeadEpilogue& e, Gate g,
                             hipStream_t s) {
  GemmArgs a = {};
  a.A = A; a.B0 = W; a.M = M; a.N = V; a.K = K; a.splits = 1; a.gate = g; a.lm = e;
  if (M <= 32)
    launch<32, 128, 1, 4, EPI_LMHEAD>(a, s);
  else
    launch<128, 128, 2, 2, EPI_LMHEAD>(a, s);
}

}  // namespace l2pd
