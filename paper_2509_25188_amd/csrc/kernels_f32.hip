// fp32 path (small models, tight tolerance): plain tiled kernels, fp32 everywhere.
#include "common.h"

namespace l2pd {

// C[M,N] (+)= A[M,K] * W[N,K]^T.  64x64 tile, 16x16 threads, 4x4 outputs per thread, K tile 16.
__global__ void __launch_bounds__(256) k_gemm_f32(const float* __restrict__ A, const float* __restrict__ W,
                                                  float* __restrict__ C, int M, int N, int K, int accumulate,
                                                  Gate g) {
  if (gate_skip(g)) return;
  __shared__ float sA[16][64 + 1];
  __shared__ float sW[16][64 + 1];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = tid; i < 64 * 16; i += 256) {
      int r = i >> 4, k = i & 15;
      int gm = m0 + r, gn = n0 + r, gk = k0 + k;
      sA[k][r] = (gm < M && gk < K) ? A[(size_t)gm * K + gk] : 0.f;
      sW[k][r] = (gn < N && gk < K) ? W[(size_t)gn * K + gk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sA[k][ty * 4 + i]; w[i] = sW[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * w[j];
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i) {
    int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
    for (int j = 0; j < 4; ++j) {
      int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      size_t o = (size_t)gm * N + gn;
      C[o] = accumulate ? C[o] + acc[i][j] : acc[i][j];
    }
  }
}
void launch_gemm_f32(const float* A, const float* W, float* C, int M, int N, int K, int accumulate, Gate g,
                     hipStream_t s) {
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  hipLaunchKernelGGL(k_gemm_f32, grid, dim3(256), 0, s, A, W, C, M, N, K, accumulate, g);
}

// Rotary embedding (pairs (i, i + Dh/2)) on q in place; k rotated and v copied into the key/value
// stores at absolute position pos0 + t.
__global__ void k_rope_store_f32(float* q, const float* k, const float* v, float* kstore, float* vstore, int B,
                                 int Tq, int pos0, int Tmax, int H, int Dh, const float* cos_t, const float* sin_t,
                                 const int* seq_gb, int pos_per_gb, Gate g) {
  if (gate_skip(g)) return;
  const int half = Dh / 2, d = H * Dh;
  size_t n = (size_t)B * Tq * H * half;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int e = i % half;
  int hh = (i / half) % H;
  int r = i / ((size_t)half * H);
  int b = r / Tq, t = r % Tq, pos = pos0 + seq_pos_offset(seq_gb, pos_per_gb, b) + t;
  float c = cos_t[pos * half + e], sn = sin_t[pos * half + e];
  size_t src = (size_t)r * d + hh * Dh + e;
  size_t dst = ((size_t)b * Tmax + pos) * d + hh * Dh + e;
  float q1 = q[src], q2 = q[src + half];
  q[src] = q1 * c - q2 * sn;
  q[src + half] = q2 * c + q1 * sn;
  float k1 = k[src], k2 = k[src + half];
  kstore[dst] = k1 * c - k2 * sn;
  kstore[dst + half] = k2 * c + k1 * sn;
  vstore[dst] = v[src];
  vstore[dst + half] = v[src + half];
}
void launch_rope_store_f32(float* q, const float* k, const float* v, float* kstore, float* vstore, int B, int Tq,
                           int pos0, int Tmax, int H, int Dh, const float* cos_t, const float* sin_t,
                           const int* seq_gb, int pos_per_gb, Gate g, hipStream_t s) {
  size_t n = (size_t)B * Tq * H * (Dh / 2);
  hipLaunchKernelGGL(k_rope_store_f32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, q, k, v, kstore, vstore,
                     B, Tq, pos0, Tmax, H, Dh, cos_t, sin_t, seq_gb, pos_per_gb, g);
}

// Bidirectional softmax attention, one wavefront per (sequence, head, query): lanes own keys for the
// scores and feature dims for the output.  Scores are staged in LDS in chunks of 1024 keys with an
// online rescale between chunks.
__global__ void __launch_bounds__(64) k_attn_f32(const float* q, const float* kstore, const float* vstore,
                                                 float* out, int B, int Tq, int Tk_all, int Tmax, int H, int Dh,
                                                 const int* tk_dev, Gate g) {
  if (gate_skip(g)) return;
  const int Tk = tk_dev ? min(Tk_all, tk_dev[blockIdx.z]) : Tk_all;   // per-sequence key count when given
  __shared__ float s_q[256];
  __shared__ float s_p[1024];
  const int lane = threadIdx.x;
  const int t = blockIdx.x, hh = blockIdx.y, b = blockIdx.z;
  const int d = H * Dh;
  const float scale = rsqrtf((float)Dh);
  const float* qv = q + ((size_t)b * Tq + t) * d + hh * Dh;
  for (int e = lane; e < Dh; e += 64) s_q[e] = qv[e];
  __syncthreads();
  float m = -INFINITY, l = 0.f;
  float o[4] = {0.f, 0.f, 0.f, 0.f};   // Dh <= 256
  for (int k0 = 0; k0 < Tk; k0 += 1024) {
    int kn = min(1024, Tk - k0);
    float cm = -INFINITY;
    for (int j = lane; j < kn; j += 64) {
      const float* kv = kstore + ((size_t)b * Tmax + k0 + j) * d + hh * Dh;
      float sc = 0.f;
      for (int e = 0; e < Dh; ++e) sc += s_q[e] * kv[e];
      sc *= scale;
      s_p[j] = sc;
      cm = fmaxf(cm, sc);
    }
#pragma unroll
    for (int of = 32; of > 0; of >>= 1) cm = fmaxf(cm, __shfl_xor(cm, of, 64));
    float mn = fmaxf(m, cm);
    float alpha = (m == -INFINITY) ? 0.f : expf(m - mn);
    float ls = 0.f;
    __syncthreads();
    for (int j = lane; j < kn; j += 64) {
      float p = expf(s_p[j] - mn);
      s_p[j] = p;
      ls += p;
    }
#pragma unroll
    for (int of = 32; of > 0; of >>= 1) ls += __shfl_xor(ls, of, 64);
    l = l * alpha + ls;
    m = mn;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      int e = lane + c * 64;
      if (e < Dh) {
        float acc = o[c] * alpha;
        for (int j = 0; j < kn; ++j) acc += s_p[j] * vstore[((size_t)b * Tmax + k0 + j) * d + hh * Dh + e];
        o[c] = acc;
      }
    }
    __syncthreads();
  }
  float* ov = out + ((size_t)b * Tq + t) * d + hh * Dh;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    int e = lane + c * 64;
    if (e < Dh) ov[e] = o[c] / l;
  }
}
void launch_attn_f32(const float* q, const float* kstore, const float* vstore, float* out, int B, int Tq, int Tk,
                     int Tmax, int H, int Dh, const int* tk_dev, Gate g, hipStream_t s) {
  hipLaunchKernelGGL(k_attn_f32, dim3(Tq, H, B), dim3(64), 0, s, q, kstore, vstore, out, B, Tq, Tk, Tmax, H, Dh, tk_dev,
                     g);
}

__global__ void k_swiglu_f32(const float* gate, const float* up, float* act, size_t n, Gate g) {
  if (gate_skip(g)) return;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float x = gate[i];
  act[i] = x / (1.f + expf(-x)) * up[i];
}
void launch_swiglu_f32(const float* gate, const float* up, float* act, size_t n, Gate g, hipStream_t s) {
  hipLaunchKernelGGL(k_swiglu_f32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, gate, up, act, n, g);
}

}  // namespace l2pd
