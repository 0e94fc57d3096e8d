// Stand-alone timing of the library's bf16 kernels at one layer's shapes, and a probe of the MFMA
// rate the chip sustains with different operand data.  Measurement tool; not part of libl2pd.so.
//
//   kernel_bench layer [rows] [d_model] [d_ffn] [heads] [keys]   per-kernel time of one transformer layer
//                                                               (keys > rows: a block-only step over a K/V store)
//   kernel_bench mfma                                     register-resident MFMA stream + shader clock
//
// "layer" calls the same launchers the library calls (same tile choice), in the order of a layer, on
// random weights and a random residual stream that stay resident in HBM (each kernel consumes what the
// one before it produced).  "mfma" shows what bounds them on a power-limited part: the same instruction
// stream runs at a lower shader clock when the operands are random instead of constant.
#include "common.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

using namespace l2pd;

#define CK(x)                                                                      \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      exit(1);                                                                     \
    }                                                                              \
  } while (0)

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) unsigned short u16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static bf16* random_bf16(size_t n, unsigned seed, float scale) {
  std::vector<unsigned short> h(n);
  unsigned s = seed;
  for (size_t i = 0; i < n; ++i) {
    s = s * 1664525u + 1013904223u;
    float f = ((int)(s >> 9) % 2001 - 1000) * 0.001f * scale;
    unsigned u;
    memcpy(&u, &f, 4);
    h[i] = (unsigned short)((u + 0x7fff + ((u >> 16) & 1)) >> 16);
  }
  bf16* d;
  CK(hipMalloc(&d, n * 2));
  CK(hipMemcpy(d, h.data(), n * 2, hipMemcpyHostToDevice));
  return d;
}

static int g_iters = 300;   // tens of milliseconds per kernel; KERNEL_BENCH_ITERS overrides (sustained-load checks)
template <typename F>
static float time_us(F f) {
  const int iters = g_iters;
  hipEvent_t a, b;
  CK(hipEventCreate(&a));
  CK(hipEventCreate(&b));
  for (int i = 0; i < 5; ++i) f();
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(a, 0));
  for (int i = 0; i < iters; ++i) f();
  CK(hipEventRecord(b, 0));
  CK(hipEventSynchronize(b));
  float ms;
  CK(hipEventElapsedTime(&ms, a, b));
  CK(hipGetLastError());
  CK(hipEventDestroy(a));
  CK(hipEventDestroy(b));
  return ms * 1e3f / iters;
}

static int bench_layer(int rows, int d, int F, int H, int keys) {
  if (keys < rows) keys = rows;
  const int Dh = d / H, Tpad = ((keys + 63) / 64) * 64;
  if (d % 64 || F % 64 || (Dh != 64 && Dh != 128)) {
    fprintf(stderr, "unsupported shape\n");
    return 2;
  }
  bf16* xn = random_bf16((size_t)rows * d, 1, 1.f);
  bf16* act_in = random_bf16((size_t)rows * F, 2, 1.f);
  bf16 *wq = random_bf16((size_t)d * d, 3, 0.02f), *wk = random_bf16((size_t)d * d, 4, 0.02f),
       *wv = random_bf16((size_t)d * d, 5, 0.02f), *wo = random_bf16((size_t)d * d, 6, 0.02f);
  bf16 *wg = random_bf16((size_t)F * d, 7, 0.02f), *wu = random_bf16((size_t)F * d, 8, 0.02f),
       *wd = random_bf16((size_t)d * F, 9, 0.02f), *gain = random_bf16(d, 10, 1.f);
  bf16 *q, *ks, *vts, *ao, *act;
  float *parts, *h, *cs, *sn;
  CK(hipMalloc(&q, (size_t)rows * d * 2));
  CK(hipMalloc(&ks, (size_t)Tpad * d * 2));
  CK(hipMalloc(&vts, (size_t)Tpad * d * 2));
  CK(hipMalloc(&ao, (size_t)rows * d * 2));
  CK(hipMalloc(&act, (size_t)rows * F * 2));
  CK(hipMalloc(&h, (size_t)rows * d * 4));
  CK(hipMalloc(&cs, (size_t)Tpad * (Dh / 2) * 4));
  CK(hipMalloc(&sn, (size_t)Tpad * (Dh / 2) * 4));
  {
    // a random residual stream: the RMSNorm timed first writes xn from it, and every later kernel works
    // on what its predecessor left, so no kernel here sees constant (cheap to switch) operands
    std::vector<float> hv((size_t)rows * d);
    unsigned sd = 11;
    for (auto& v : hv) {
      sd = sd * 1664525u + 1013904223u;
      v = ((int)(sd >> 9) % 2001 - 1000) * 0.001f;
    }
    CK(hipMemcpy(h, hv.data(), hv.size() * 4, hipMemcpyHostToDevice));
  }
  CK(hipMemset(ks, 0, (size_t)Tpad * d * 2));
  CK(hipMemset(vts, 0, (size_t)Tpad * d * 2));
  {
    std::vector<float> c((size_t)Tpad * (Dh / 2)), s(c.size());
    for (size_t i = 0; i < c.size(); ++i) { c[i] = cosf(0.001f * i); s[i] = sinf(0.001f * i); }
    CK(hipMemcpy(cs, c.data(), c.size() * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(sn, s.data(), s.size() * 4, hipMemcpyHostToDevice));
  }
  const Gate g = {nullptr, -1};
  const RowMap ident = {rows, 0, 0, 0};
  const QkvEpilogue qe = {q, ks, vts, cs, sn, rows, 0, Tpad, H, Dh, d};
  // routing and split counts as in the library: the few-row path up to kSkinnyRows rows, else the wide path,
  // which splits K in two on the [d, d] and [d, F] projections when there are few row tiles
  const bool skinny = rows <= kSkinnyRows;
  const int so = skinny ? skinny_splits(d, d) : wide_splits(rows, d, d);
  const int sd = skinny ? skinny_splits(d, F) : wide_splits(rows, d, F);
  const int sq = skinny ? skinny_splits(3 * d, d) : 1, sg = skinny ? skinny_splits(2 * F, d) : 1;
  size_t pbytes = (size_t)2 * rows * d * 4;
  for (size_t b : {(size_t)sq * rows * 3 * d * 4, (size_t)sg * rows * 2 * F * 4, (size_t)so * rows * d * 4,
                   (size_t)sd * rows * d * 4})
    if (b > pbytes) pbytes = b;
  CK(hipMalloc(&parts, pbytes));
  CK(hipMemset(parts, 0, pbytes));
  const size_t stride_d = (size_t)rows * d;
  printf("one layer, %d rows (one sequence), d_model %d, d_ffn %d, %d heads of %d; bf16, random operands; %s path\n", rows,
         d, F, H, Dh, skinny ? "few-row" : "wide");
  auto line = [](const char* name, float us, double flop, double bytes) {
    printf("  %-52s %8.1f us", name, us);
    if (flop > 0) printf("  %7.1f TFLOP/s", flop / us / 1e6);
    if (bytes > 0) printf("  %7.1f GB/s", bytes / us / 1e3);
    printf("\n");
    fflush(stdout);
  };
  const double wb = 2.0;   // bytes per weight
  float t;
  t = time_us([&] { launch_rmsnorm(h, parts, so, stride_d, ident, gain, L2PD_BF16, xn, rows, d, 1e-5f, g, 0); });
  line("RMSNorm (+ fold of split-K partials)", t, 0, (double)rows * d * (4.0 * (2 + so) + 2));
  if (skinny) {
    t = time_us([&] {
      launch_gemm_skinny_bf16(xn, wq, wk, wv, d, parts, (size_t)rows * 3 * d, rows, 3 * d, d, sq, g, 0);
      launch_skinny_qkv_finish(parts, sq, (size_t)rows * 3 * d, rows, qe, g, 0);
    });
    line("QKV projection (split-K) + RoPE / store kernel", t, 0, wb * 3 * d * d);
  } else {
    t = time_us([&] { launch_gemm_qkv_bf16(xn, wq, wk, wv, rows, d, qe, g, 0); });
    line("QKV projection + RoPE + K / V^T store", t, 2.0 * rows * d * 3 * d, 0);
  }
  float* aws;
  CK(hipMalloc(&aws, attn_chunk_ws_bytes(H, Dh)));
  t = time_us([&] { launch_attn_bf16(q, ks, vts, ao, 1, rows, keys, Tpad, H, Dh, aws, attn_chunk_ws_bytes(H, Dh), nullptr, g, 0); });
  char an[64];
  snprintf(an, sizeof an, "bidirectional attention, %d keys", keys);
  line(an, t, 4.0 * rows * keys * d, 0);
  if (skinny) {
    t = time_us([&] { launch_gemm_skinny_bf16(ao, wo, nullptr, nullptr, 0, parts, stride_d, rows, d, d, so, g, 0); });
    line("output projection (split-K partials)", t, 0, wb * d * d);
    if (swiglu_few_rows_fused(rows, F)) {
      t = time_us([&] { launch_gemm_swiglu_bf16(xn, wg, wu, act, rows, F, d, g, 0); });
      line("gate / up projection + SwiGLU (few-row tiles)", t, 0, wb * 2 * F * d);
    } else {
      t = time_us([&] {
        launch_gemm_skinny_bf16(xn, wg, wu, nullptr, F, parts, (size_t)rows * 2 * F, rows, 2 * F, d, sg, g, 0);
        launch_skinny_swiglu_finish(parts, sg, (size_t)rows * 2 * F, rows, F, act, g, 0);
      });
      line("gate / up projection (split-K) + SwiGLU kernel", t, 0, wb * 2 * F * d);
    }
    t = time_us([&] { launch_gemm_skinny_bf16(act_in, wd, nullptr, nullptr, 0, parts, stride_d, rows, d, F, sd, g, 0); });
    line("down projection (split-K partials)", t, 0, wb * d * F);
  } else {
    t = time_us([&] { launch_gemm_partial_bf16(ao, wo, parts, stride_d, rows, d, d, so, g, 0); });
    line("output projection (split-K partials)", t, 2.0 * rows * d * d, 0);
    t = time_us([&] { launch_gemm_swiglu_bf16(xn, wg, wu, act, rows, F, d, g, 0); });
    line("gate / up projection + SwiGLU", t, 2.0 * rows * d * 2 * F, 0);
    t = time_us([&] { launch_gemm_partial_bf16(act_in, wd, parts, stride_d, rows, d, F, sd, g, 0); });
    line("down projection (split-K partials)", t, 2.0 * rows * d * F, 0);
  }
  return 0;
}

// ------------------------------------------------------------------------------------------------
__device__ long long g_clk[2];
__device__ unsigned mix(unsigned x) {
  x ^= x >> 16; x *= 0x45d9f3bu; x ^= x >> 16; x *= 0x45d9f3bu; x ^= x >> 16;
  return x;
}
// MODE 0: zero operands, 1: all ones, 2: random sign / exponent / mantissa
template <int MODE>
__global__ void __launch_bounds__(256) k_mfma_stream(float* out, int iters) {
  const int tid = threadIdx.x;
  const long long c0 = clock64(), w0 = wall_clock64();
  bf16x8_t fa[8], fb[8];
  for (int s = 0; s < 8; ++s) {
    u16x8 ua, ub;
    for (int e = 0; e < 8; ++e) {
      const unsigned h1 = mix((blockIdx.x * 256 + tid) * 64 + s * 8 + e), h2 = mix(h1 + 12345);
      const unsigned short ra = (unsigned short)((h1 & 0x8000) | (0x3f00 - ((h1 >> 16) & 3) * 0x80) | (h1 & 0xff));
      const unsigned short rb = (unsigned short)((h2 & 0x8000) | (0x3c00 - ((h2 >> 16) & 3) * 0x80) | (h2 & 0xff));
      ua[e] = MODE == 0 ? 0 : (MODE == 1 ? 0x3f80 : ra);
      ub[e] = MODE == 0 ? 0 : (MODE == 1 ? 0x3f80 : rb);
    }
    fa[s] = __builtin_bit_cast(bf16x8_t, ua);
    fb[s] = __builtin_bit_cast(bf16x8_t, ub);
  }
  f32x16 acc[4];
  for (int n = 0; n < 4; ++n)
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int n = 0; n < 4; ++n)
        acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[(s + (n >> 1)) & 7], fb[(s + 3 + (n & 1)) & 7], acc[n], 0, 0, 0);
  }
  float s = 0;
  for (int n = 0; n < 4; ++n)
    for (int r = 0; r < 16; ++r) s += acc[n][r];
  out[blockIdx.x * 256 + tid] = s;
  if (blockIdx.x == 17 && tid == 0) {
    g_clk[0] = clock64() - c0;
    g_clk[1] = wall_clock64() - w0;   // 100 MHz
  }
}
template <int MODE>
static void run_stream(float* out, const char* name) {
  const int iters = 20000, wgs = 256;
  hipEvent_t a, b;
  CK(hipEventCreate(&a));
  CK(hipEventCreate(&b));
  hipLaunchKernelGGL(k_mfma_stream<MODE>, dim3(wgs), dim3(256), 0, 0, out, 100);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(a, 0));
  hipLaunchKernelGGL(k_mfma_stream<MODE>, dim3(wgs), dim3(256), 0, 0, out, iters);
  CK(hipEventRecord(b, 0));
  CK(hipEventSynchronize(b));
  float ms;
  CK(hipEventElapsedTime(&ms, a, b));
  CK(hipGetLastError());
  long long h[2];
  CK(hipMemcpyFromSymbol(h, HIP_SYMBOL(g_clk), sizeof(h)));
  const double flops = (double)wgs * 4 * iters * 32 * 2.0 * 32 * 32 * 16;
  printf("  %-18s %8.3f ms  %7.1f TFLOP/s  shader clock %4.0f MHz\n", name, ms, flops / ms / 1e9,
         h[0] * 100.0 / (double)h[1]);
  fflush(stdout);
}

int main(int argc, char** argv) {
  const char* mode = argc > 1 ? argv[1] : "layer";
  if (const char* it = getenv("KERNEL_BENCH_ITERS")) {
    const int v = atoi(it);
    if (v >= 1 && v <= 100000) g_iters = v;
  }
  if (!strcmp(mode, "mfma")) {
    float* out;
    CK(hipMalloc(&out, 256 * 256 * 4));
    printf("v_mfma_f32_32x32x16_bf16 from registers, one wavefront per SIMD on every CU, ~10 ms per run\n");
    for (int rep = 0; rep < 2; ++rep) {
      run_stream<0>(out, "zero operands");
      run_stream<1>(out, "all ones");
      run_stream<2>(out, "random operands");
    }
    return 0;
  }
  if (!strcmp(mode, "layer")) {
    const int rows = argc > 2 ? atoi(argv[2]) : 512, d = argc > 3 ? atoi(argv[3]) : 4096,
              F = argc > 4 ? atoi(argv[4]) : 12288, H = argc > 5 ? atoi(argv[5]) : 32,
              keys = argc > 6 ? atoi(argv[6]) : 0;
    if (rows < 1 || rows > 65536 || keys > 65536 || d < 128 || H < 1 || d % H) {
      fprintf(stderr, "bad shape\n");
      return 2;
    }
    return bench_layer(rows, d, F, H, keys);
  }
  fprintf(stderr, "usage: kernel_bench layer [rows d_model d_ffn heads keys] | kernel_bench mfma\n");
  return 2;
}
