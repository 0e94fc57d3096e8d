// Small kernels of the decoding loop: embedding gather, RMSNorm (wavefront reduction), the
// vocabulary reduction over materialised logits, the filter + unmask + EoTP update, loop control.
#include "common.h"

namespace l2pd {

// ------------------------------------------------------------------------------------------------
__global__ void k_fill_u32(uint32_t* p, size_t n, uint32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}
void launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s) {
  if (!n) return;
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, s, p, n, v);
}

// cos/sin of pos * base^(-2i/Dh), evaluated in double and stored as float.
__global__ void k_rope_table(float* cos_t, float* sin_t, int max_pos, int half, int head_dim, float base) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= max_pos * half) return;
  int pos = idx / half, i = idx % half;
  double inv = pow((double)base, -2.0 * (double)i / (double)head_dim);
  double a = (double)pos * inv;
  cos_t[idx] = (float)cos(a);
  sin_t[idx] = (float)sin(a);
}
void launch_rope_table(float* cos_t, float* sin_t, int max_pos, int head_dim, float base, hipStream_t s) {
  int half = head_dim / 2, n = max_pos * half;
  hipLaunchKernelGGL(k_rope_table, dim3((n + 255) / 256), dim3(256), 0, s, cos_t, sin_t, max_pos, half, head_dim,
                     base);
}

// X <- prompt || [MASK]^G ; state <- 0   (Alg. 2, initialisation of X)
__global__ void k_init_decode(int32_t* X, const int32_t* prompt, int B, int P, int G, int mask_id, int32_t* state,
                              int* ctl) {
  int T = P + G;
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B * T) {
    int b = i / T, t = i % T;
    X[i] = t < P ? prompt[b * P + t] : mask_id;
  }
  if (i < B * 3) state[i] = 0;
  if (i < CTL_WORDS) ctl[i] = 0;
}
void launch_init_decode(int32_t* X, const int32_t* prompt, int B, int P, int G, int mask_id, int32_t* state,
                        int* ctl, hipStream_t s) {
  int n = B * (P + G);
  if (n < 64) n = 64;
  hipLaunchKernelGGL(k_init_decode, dim3((n + 255) / 256), dim3(256), 0, s, X, prompt, B, P, G, mask_id, state,
                     ctl);
}

// Active block of the lock-step batch = smallest block index among sequences that are not done.
// With `ragged` every sequence works on its own block (per-sequence block pointers): nobody idles
// while another sequence finishes the common block.
__global__ void k_prepare(const int32_t* state, int B, int n_blocks, int ragged, int* ctl, int done_at) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    int gb = n_blocks, all_done = 1, n_active = 0;
    for (int b = 0; b < B; ++b) {
      if (!state[b * 3 + 2]) {
        all_done = 0;
        ++n_active;
        int bi = state[b * 3 + 0];
        gb = bi < gb ? bi : gb;
      }
    }
    if (gb >= n_blocks) all_done = 1;
    const int last = n_blocks > 0 ? n_blocks - 1 : 0;
    ctl[CTL_GB] = all_done ? last : gb;
    ctl[CTL_ALL_DONE] = all_done;
    ctl[CTL_ACTIVE] = all_done ? 0 : n_active;
    for (int b = 0; b < B; ++b) {
      const int own = state[b * 3 + 0] < last ? state[b * 3 + 0] : last;
      ctl[CTL_SEQ_GB + b] = ragged ? own : ctl[CTL_GB];
      if (done_at > 0) ctl[done_at + b] = state[b * 3 + 2] ? 1 : 0;
    }
  }
}
void launch_prepare(const int32_t* state, int B, int n_blocks, int ragged, int* ctl, hipStream_t s, int done_at) {
  hipLaunchKernelGGL(k_prepare, dim3(1), dim3(64), 0, s, state, B, n_blocks, ragged, ctl, done_at);
}

__global__ void k_block_keys(const int* ctl, int B, int base, int per_gb, int* keys) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) keys[b] = base + ctl[CTL_SEQ_GB + b] * per_gb;
}
void launch_block_keys(const int* ctl, int B, int base, int per_gb, int* keys, hipStream_t s) {
  hipLaunchKernelGGL(k_block_keys, dim3((B + 63) / 64), dim3(64), 0, s, ctl, B, base, per_gb, keys);
}

// Batch compaction: rows of sequences that are not done move to the front (order kept), finished
// ones behind them (order kept), so that later steps run over the leading rows only.  Reads the
// `src` copies of tokens / state / row->sequence map and writes the `dst` copies; perm_src == nullptr
// stands for the identity map.  Every workgroup works out the source row of its own destination row.
__global__ void __launch_bounds__(256) k_compact(const int32_t* X_src, int32_t* X_dst, const int32_t* state_src,
                                                 int32_t* state_dst, const int32_t* perm_src, int32_t* perm_dst,
                                                 int B, int T) {
  __shared__ int s_from;
  const int r = blockIdx.y;
  if (threadIdx.x == 0) {
    int n_live = 0;
    for (int b = 0; b < B; ++b) n_live += state_src[b * 3 + 2] ? 0 : 1;
    // destination rows [0, n_live) take the live rows in order, the rest the finished rows in order
    const bool want_done = r >= n_live;
    int k = want_done ? r - n_live : r, from = 0;
    for (int b = 0; b < B; ++b) {
      if ((state_src[b * 3 + 2] != 0) == want_done) {
        if (k == 0) { from = b; break; }
        --k;
      }
    }
    s_from = from;
  }
  __syncthreads();
  const int from = s_from;
  for (int t = blockIdx.x * 256 + threadIdx.x; t < T; t += gridDim.x * 256)
    X_dst[(size_t)r * T + t] = X_src[(size_t)from * T + t];
  if (blockIdx.x == 0 && threadIdx.x < 3) state_dst[r * 3 + threadIdx.x] = state_src[from * 3 + threadIdx.x];
  if (blockIdx.x == 0 && threadIdx.x == 3) perm_dst[r] = perm_src ? perm_src[from] : from;
}
void launch_compact(const int32_t* X_src, int32_t* X_dst, const int32_t* state_src, int32_t* state_dst,
                    const int32_t* perm_src, int32_t* perm_dst, int B, int T, hipStream_t s) {
  int gx = (T + 255) / 256;
  if (gx > 8) gx = 8;
  hipLaunchKernelGGL(k_compact, dim3(gx, B), dim3(256), 0, s, X_src, X_dst, state_src, state_dst, perm_src, perm_dst,
                     B, T);
}

// ------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ float to_f(T v);
template <>
__device__ __forceinline__ float to_f<float>(float v) { return v; }
template <>
__device__ __forceinline__ float to_f<bf16>(bf16 v) { return __bfloat162float(v); }
template <typename T>
__device__ __forceinline__ T from_f(float v);
template <>
__device__ __forceinline__ float from_f<float>(float v) { return v; }
template <>
__device__ __forceinline__ bf16 from_f<bf16>(float v) { return __float2bfloat16(v); }

template <typename T>
__global__ void k_embed(float* h, const T* emb, const int32_t* tokens, RowMap tokmap, int rows, int d, Gate g) {
  if (gate_skip(g)) return;
  int r = blockIdx.x;
  int tok = tokens[map_row(tokmap, r, g.ctl)];
  const T* e = emb + (size_t)tok * d;
  float* o = h + (size_t)r * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) o[i] = to_f<T>(e[i]);
}
void launch_embed(float* h, const void* emb, int dtype, const int32_t* tokens, RowMap tokmap, int rows, int d,
                  Gate g, hipStream_t s) {
  if (dtype == L2PD_FP32)
    hipLaunchKernelGGL(k_embed<float>, dim3(rows), dim3(256), 0, s, h, (const float*)emb, tokens, tokmap, rows, d, g);
  else
    hipLaunchKernelGGL(k_embed<bf16>, dim3(rows), dim3(256), 0, s, h, (const bf16*)emb, tokens, tokmap, rows, d, g);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One wavefront per row: the row's sum of squares is a 64-lane butterfly, no LDS.
// When partial buffers are given the residual update h += (((part[0] + part[1]) + part[2]) + ...) is folded
// in: the partials are summed first, in ascending order, and their sum is added to h.  (A projection whose
// workgroups walk the K ranges one after the other forms the same sum in registers and writes it as its only
// partial: summing the partials before h is what makes the two bit-identical.)  Part z is at
// parts + z * part_stride, laid out like h.
template <typename T>
__global__ void k_rmsnorm(float* h, const float* parts, int n_parts, size_t part_stride, RowMap src, const T* gain,
                          T* y, int rows, int d, float eps, int wb, Gate g) {
  if (gate_skip(g)) return;
  int lane = threadIdx.x & 63;
  int r = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (r >= rows) return;
  size_t srow = (size_t)map_row(src, r, g.ctl);
  float* x = h + srow * d;
  const float* a0 = parts + srow * d;
  float ss = 0.f;
  for (int i = lane; i < d; i += 64) {
    float v = x[i];
    if (n_parts > 0) {
      float ps = a0[i];
      for (int z = 1; z < n_parts; ++z) ps += a0[z * part_stride + i];
      v += ps;
      if (wb) x[i] = v;
    }
    ss += v * v;
  }
  ss = wave_sum(ss);
  float inv = rsqrtf(ss / (float)d + eps);
  T* o = y + (size_t)r * d;
  for (int i = lane; i < d; i += 64) {
    float v = x[i];
    if (n_parts > 0 && !wb) {
      float ps = a0[i];
      for (int z = 1; z < n_parts; ++z) ps += a0[z * part_stride + i];
      v += ps;
    }
    o[i] = from_f<T>(v * inv * to_f<T>(gain[i]));
  }
}
// Same, with the row held in registers: VPL float4 per lane, all loads of a row in flight at once,
// one pass over memory.  Used when d is a multiple of 4 and d <= 1024 * VPL.
template <typename T, int VPL>
__global__ void __launch_bounds__(256) k_rmsnorm_vec(float* h, const float* parts, int n_parts, size_t part_stride,
                                                    RowMap src, const T* gain, T* y, int rows, int d, float eps,
                                                    int wb, Gate g) {
  if (gate_skip(g)) return;
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (r >= rows) return;
  const size_t srow = (size_t)map_row(src, r, g.ctl);
  const int d4 = d >> 2;
  float4* x = reinterpret_cast<float4*>(h + srow * d);
  float4 v[VPL];
#pragma unroll
  for (int k = 0; k < VPL; ++k) {
    const int i = lane + 64 * k;
    v[k] = i < d4 ? x[i] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  if (n_parts > 0) {
    float4 ps[VPL];
    for (int z = 0; z < n_parts; ++z) {
      const float4* az = reinterpret_cast<const float4*>(parts + z * part_stride + srow * d);
#pragma unroll
      for (int k = 0; k < VPL; ++k) {
        const int i = lane + 64 * k;
        float4 t = i < d4 ? az[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        if (z == 0) ps[k] = t;
        else { ps[k].x += t.x; ps[k].y += t.y; ps[k].z += t.z; ps[k].w += t.w; }
      }
    }
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
      const int i = lane + 64 * k;
      v[k].x += ps[k].x; v[k].y += ps[k].y; v[k].z += ps[k].z; v[k].w += ps[k].w;
      if (wb && i < d4) x[i] = v[k];
    }
  }
  float ss = 0.f;
#pragma unroll
  for (int k = 0; k < VPL; ++k) ss += v[k].x * v[k].x + v[k].y * v[k].y + v[k].z * v[k].z + v[k].w * v[k].w;
  ss = wave_sum(ss);
  const float inv = rsqrtf(ss / (float)d + eps);
  T* o = y + (size_t)r * d;
#pragma unroll
  for (int k = 0; k < VPL; ++k) {
    const int i = lane + 64 * k;
    if (i < d4) {
      const T* gp = gain + 4 * i;
      if constexpr (sizeof(T) == 4) {
        float4 gg = *reinterpret_cast<const float4*>(gp);
        *reinterpret_cast<float4*>(o + 4 * i) =
            make_float4(v[k].x * inv * gg.x, v[k].y * inv * gg.y, v[k].z * inv * gg.z, v[k].w * inv * gg.w);
      } else {
        T o4[4] = {from_f<T>(v[k].x * inv * to_f<T>(gp[0])), from_f<T>(v[k].y * inv * to_f<T>(gp[1])),
                   from_f<T>(v[k].z * inv * to_f<T>(gp[2])), from_f<T>(v[k].w * inv * to_f<T>(gp[3]))};
        *reinterpret_cast<uint2*>(o + 4 * i) = *reinterpret_cast<const uint2*>(o4);
      }
    }
  }
}

// Wide rows (d >= 2048): one row per workgroup of NTH threads (1024: a float4 per thread and stream at the 8B
// width), the row's sum of squares combined across the wavefronts through LDS in a fixed pairwise tree.
// Many wavefronts with few loads each hide the latency of the partials, which the preceding projection has
// just written: 7.2 -> 5.6 us at 32 rows folding eight partials, 11.7 -> 11.2 us at 512 rows folding four
// (256 threads per row before).  The choice between this kernel and the one-wavefront-per-row kernels
// depends on d only, never on the number of rows, so that a row's result does not depend on the batch it
// is part of.
template <typename T, int VPL, int NTH>
__global__ void __launch_bounds__(NTH) k_rmsnorm_row(float* h, const float* parts, int n_parts, size_t part_stride,
                                                    RowMap src, const T* gain, T* y, int rows, int d, float eps,
                                                    int wb, int quad_tiled, Gate g) {
  if (gate_skip(g)) return;
  __shared__ float s_part[NTH / 64];
  const int tid = threadIdx.x;
  int r = blockIdx.x;
  if (quad_tiled) {
    // Quad-tiled output interleaves four rows inside every 128-byte line.  Workgroups are dealt to the 8
    // XCDs round-robin by their id; give the four rows of a group to workgroups of one XCD, so that the
    // line is completed in that XCD's L2 before it is written back.  (A permutation of [0, gridDim.x), the
    // grid being the row count rounded up to 32.)
    const int xcd = r & 7, slot = r >> 3;
    r = ((slot >> 2) * 8 + xcd) * 4 + (slot & 3);
    if (r >= rows) return;
  }
  const size_t srow = (size_t)map_row(src, r, g.ctl);
  const int d4 = d >> 2;
  float4* x = reinterpret_cast<float4*>(h + srow * d);
  float4 v[VPL];
#pragma unroll
  for (int k = 0; k < VPL; ++k) {
    const int i = tid + NTH * k;
    v[k] = i < d4 ? x[i] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  // partials four at a time (the few-row path folds eight or more): the loads of a group are in
  // flight together, the adds stay in ascending order
  constexpr int GRP = 4;
  float4 ps[VPL];
#pragma unroll
  for (int k = 0; k < VPL; ++k) ps[k] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int z0 = 0; z0 < n_parts; z0 += GRP) {
    float4 t[GRP][VPL];
#pragma unroll
    for (int z = 0; z < GRP; ++z) {
      const bool have = z0 + z < n_parts;
      const float4* a = reinterpret_cast<const float4*>(parts + (have ? z0 + z : z0) * part_stride + srow * d);
#pragma unroll
      for (int k = 0; k < VPL; ++k) {
        const int i = tid + NTH * k;
        t[z][k] = (have && i < d4) ? a[i] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int z = 0; z < GRP; ++z)
      if (z0 + z < n_parts) {
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
          if (z0 + z == 0) ps[k] = t[z][k];
          else { ps[k].x += t[z][k].x; ps[k].y += t[z][k].y; ps[k].z += t[z][k].z; ps[k].w += t[z][k].w; }
        }
      }
  }
  if (n_parts > 0) {   // the partials' sum, then the residual: h + (p0 + p1 + ...)
#pragma unroll
    for (int k = 0; k < VPL; ++k) { v[k].x += ps[k].x; v[k].y += ps[k].y; v[k].z += ps[k].z; v[k].w += ps[k].w; }
  }
  float ss = 0.f;
#pragma unroll
  for (int k = 0; k < VPL; ++k) {
    const int i = tid + NTH * k;
    if (wb && n_parts > 0 && i < d4) x[i] = v[k];
    ss += v[k].x * v[k].x + v[k].y * v[k].y + v[k].z * v[k].z + v[k].w * v[k].w;
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) s_part[tid >> 6] = ss;
  __syncthreads();
  // the wavefronts' sums in a fixed pairwise tree
  float tree[NTH / 64];
#pragma unroll
  for (int w = 0; w < NTH / 64; ++w) tree[w] = s_part[w];
#pragma unroll
  for (int n = NTH / 64; n > 1; n >>= 1)
#pragma unroll
    for (int w = 0; w < n / 2; ++w) tree[w] = tree[2 * w] + tree[2 * w + 1];
  ss = tree[0];
  const float inv = rsqrtf(ss / (float)d + eps);
  T* o = y + (size_t)r * d;
  // quad-tiled: the row's 16-byte chunk c sits at ((r / 4) * (d / 8) + c) * 32 + (r % 4) * 8 elements
  T* oq = y + (size_t)(r >> 2) * 4 * d + (r & 3) * 8;
#pragma unroll
  for (int k = 0; k < VPL; ++k) {
    const int i = tid + NTH * k;
    if (i < d4) {
      const T* gp = gain + 4 * i;
      if constexpr (sizeof(T) == 4) {
        float4 gg = *reinterpret_cast<const float4*>(gp);
        *reinterpret_cast<float4*>(o + 4 * i) =
            make_float4(v[k].x * inv * gg.x, v[k].y * inv * gg.y, v[k].z * inv * gg.z, v[k].w * inv * gg.w);
      } else {
        T o4[4] = {from_f<T>(v[k].x * inv * to_f<T>(gp[0])), from_f<T>(v[k].y * inv * to_f<T>(gp[1])),
                   from_f<T>(v[k].z * inv * to_f<T>(gp[2])), from_f<T>(v[k].w * inv * to_f<T>(gp[3]))};
        T* dst = quad_tiled ? oq + (i >> 1) * 32 + (i & 1) * 4 : o + 4 * i;
        *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(o4);
      }
    }
  }
}

constexpr int NORM_TX = 4;   // threads per row = 256 * NORM_TX
template <typename T>
static void launch_rmsnorm_t(float* h, const float* parts, int n_parts, size_t part_stride, RowMap src, const T* gain,
                             T* y, int rows, int d, float eps, bool write_back, Gate g, hipStream_t s, bool quad_tiled) {
  const int wb = write_back ? 1 : 0;
  if (quad_tiled) {
    // only the one-row-per-workgroup kernels write it (gemm_qkv_a_quad_tiled() asks for it within their range only)
    if (sizeof(T) != 2 || d % 8 != 0 || d < 2048 || d > 8192) {
      // a caller's mistake, not an input's: the consumer would read another layout than the one written
      fprintf(stderr, "l2pd: quad-tiled RMSNorm output asked for outside its range (d = %d)\n", d);
      abort();
    }
    const int grid_q = (rows + 31) / 32 * 32;
    if (d <= 4096)
      hipLaunchKernelGGL((k_rmsnorm_row<T, 4 / NORM_TX, 256 * NORM_TX>), dim3(grid_q), dim3(256 * NORM_TX), 0, s, h, parts, n_parts, part_stride, src, gain, y, rows, d, eps, wb, 1, g);
    else
      hipLaunchKernelGGL((k_rmsnorm_row<T, 8 / NORM_TX, 256 * NORM_TX>), dim3(grid_q), dim3(256 * NORM_TX), 0, s, h, parts, n_parts, part_stride, src, gain, y, rows, d, eps, wb, 1, g);
    return;
  }
  dim3 grid((rows + 3) / 4), block(256);
  if (rows <= 4096) { grid = dim3(rows); block = dim3(64); }   // few rows: one wavefront per workgroup fills more CUs
  if (d % 4 == 0 && d >= 2048 && d <= 4096)
    hipLaunchKernelGGL((k_rmsnorm_row<T, 4 / NORM_TX, 256 * NORM_TX>), dim3(rows), dim3(256 * NORM_TX), 0, s, h, parts, n_parts, part_stride, src, gain, y, rows, d, eps, wb, 0, g);
  else if (d % 4 == 0 && d > 4096 && d <= 8192)
    hipLaunchKernelGGL((k_rmsnorm_row<T, 8 / NORM_TX, 256 * NORM_TX>), dim3(rows), dim3(256 * NORM_TX), 0, s, h, parts, n_parts, part_stride, src, gain, y, rows, d, eps, wb, 0, g);
  else if (d % 4 == 0 && d <= 1024)
    hipLaunchKernelGGL((k_rmsnorm_vec<T, 4>), grid, block, 0, s, h, parts, n_parts, part_stride, src, gain, y, rows, d, eps, wb, g);
  else if (d % 4 == 0 && d <= 4096)
    hipLaunchKernelGGL((k_rmsnorm_vec<T, 16>), grid, block, 0, s, h, parts, n_parts, part_stride, src, gain, y, rows, d, eps, wb, g);
  else if (d % 4 == 0 && d <= 8192)
    hipLaunchKernelGGL((k_rmsnorm_vec<T, 32>), grid, block, 0, s, h, parts, n_parts, part_stride, src, gain, y, rows, d, eps, wb, g);
  else
    hipLaunchKernelGGL(k_rmsnorm<T>, grid, block, 0, s, h, parts, n_parts, part_stride, src, gain, y, rows, d, eps, wb, g);
}
void launch_rmsnorm(float* h, const float* parts, int n_parts, size_t part_stride, RowMap src, const void* gain,
                    int dtype, void* y, int rows, int d, float eps, bool write_back, Gate g, hipStream_t s,
                    bool quad_tiled) {
  if (!parts) n_parts = 0;
  if (dtype == L2PD_FP32)
    launch_rmsnorm_t<float>(h, parts, n_parts, part_stride, src, (const float*)gain, (float*)y, rows, d, eps, write_back, g, s, quad_tiled);
  else
    launch_rmsnorm_t<bf16>(h, parts, n_parts, part_stride, src, (const bf16*)gain, (bf16*)y, rows, d, eps, write_back, g, s, quad_tiled);
}

// ------------------------------------------------------------------------------------------------
// Finishing kernels of the few-row ("skinny") GEMM path: the GEMM leaves fp32 partial products per
// K range; these sum them in ascending range order and apply what the wide path fuses into its
// GEMM epilogues.  Rows are few (<= 64 per launch), so this is a few hundred KB of traffic.
__device__ __forceinline__ unsigned short bf16_bits(float f) { return __builtin_bit_cast(unsigned short, (__bf16)f); }

// parts [n_parts][rows, 3d] (Q | K | V columns) -> rotated q [rows, d], K store, V^T store
__global__ void __launch_bounds__(256) k_skinny_qkv_finish(const float* parts, int n_parts, size_t part_stride,
                                                          int rows, QkvEpilogue e, Gate g) {
  if (gate_skip(g)) return;
  const int half = e.Dh / 2, per_row = 3 * e.H * half;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= rows * per_row) return;
  const int row = t / per_row, rem = t % per_row;
  const int hg = rem / half, i = rem % half;
  const int mat = hg / e.H, head = hg % e.H;
  const size_t col = (size_t)mat * e.d + head * e.Dh + i;
  const float* p = parts + (size_t)row * 3 * e.d + col;
  float x1 = 0.f, x2 = 0.f;
  for (int z = 0; z < n_parts; ++z) {
    x1 += p[z * part_stride];
    x2 += p[z * part_stride + half];
  }
  const int b = row / e.Tq, pos = e.pos0 + seq_pos_offset(e.seq_gb, e.pos_per_gb, b) + row % e.Tq;
  if (mat == 2) {
    unsigned short* vt = reinterpret_cast<unsigned short*>(e.vtstore);
    const size_t o = ((size_t)(b * e.H + head) * e.Dh + i) * e.Tpad + pos;
    vt[o] = bf16_bits(x1);
    vt[o + (size_t)half * e.Tpad] = bf16_bits(x2);
    return;
  }
  const float cs = e.cos_t[(size_t)pos * half + i], sn = e.sin_t[(size_t)pos * half + i];
  const float o1 = __fmaf_rn(x1, cs, -__fmul_rn(x2, sn)), o2 = __fmaf_rn(x2, cs, __fmul_rn(x1, sn));
  unsigned short* dst = reinterpret_cast<unsigned short*>(mat == 0 ? e.q : e.kstore);
  const size_t o = (mat == 0 ? (size_t)row * e.d : ((size_t)b * e.Tpad + pos) * e.d) + head * e.Dh + i;
  dst[o] = bf16_bits(o1);
  dst[o + half] = bf16_bits(o2);
}
void launch_skinny_qkv_finish(const float* parts, int n_parts, size_t part_stride, int rows, const QkvEpilogue& e,
                              Gate g, hipStream_t s) {
  const int n = rows * 3 * e.H * (e.Dh / 2);
  hipLaunchKernelGGL(k_skinny_qkv_finish, dim3((n + 255) / 256), dim3(256), 0, s, parts, n_parts, part_stride, rows, e,
                     g);
}

// parts [n_parts][rows, 2F] (gate | up columns) -> act [rows, F] = SiLU(gate) * up
__global__ void __launch_bounds__(256) k_skinny_swiglu_finish(const float* parts, int n_parts, size_t part_stride,
                                                             int rows, int F, bf16* act, Gate g) {
  if (gate_skip(g)) return;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= rows * F) return;
  const int row = t / F, col = t % F;
  const float* p = parts + (size_t)row * 2 * F + col;
  float gt = 0.f, up = 0.f;
  for (int z = 0; z < n_parts; ++z) {
    gt += p[z * part_stride];
    up += p[z * part_stride + F];
  }
  const float v = __fmul_rn(__fmul_rn(gt, __builtin_amdgcn_rcpf(__fadd_rn(1.f, __expf(-gt)))), up);
  reinterpret_cast<unsigned short*>(act)[t] = bf16_bits(v);
}
void launch_skinny_swiglu_finish(const float* parts, int n_parts, size_t part_stride, int rows, int F, bf16* act,
                                 Gate g, hipStream_t s) {
  const int n = rows * F;
  hipLaunchKernelGGL(k_skinny_swiglu_finish, dim3((n + 255) / 256), dim3(256), 0, s, parts, n_parts, part_stride, rows,
                     F, act, g);
}

// ------------------------------------------------------------------------------------------------
// Vocabulary reduction over materialised fp32 logits: per (row, column chunk) the running
// (max, sum exp(x - max), argmax) triple of Eq. 3 / Eq. 4; the mask id is not a data token.
__global__ void k_vocab_partials(float* logits, int rows, int V, int chunk, int mask_id, BiasArgs bias,
                                 float* part_max, float* part_sum, int32_t* part_idx, int n_part, Gate g) {
  if (gate_skip(g)) return;
  __shared__ float s_m[256];
  __shared__ int s_i[256];
  __shared__ float s_s[256];
  int p = blockIdx.x, r = blockIdx.y, tid = threadIdx.x;
  float* row = logits + (size_t)r * V;
  int c0 = p * chunk, c1 = min(V, c0 + chunk);
  if (bias.value != 0.f && bias.token_id >= c0 && bias.token_id < c1 && tid == 0) {
    int gb = g.ctl ? g.ctl[CTL_SEQ_GB + r / bias.block_len] : 0;
    int genpos = gb * bias.block_len + (r % bias.block_len);
    if (genpos >= bias.gen_pos_from) row[bias.token_id] += bias.value;
  }
  __syncthreads();
  float m = -INFINITY;
  int mi = 0x7fffffff;
  for (int c = c0 + tid; c < c1; c += 256) {
    float v = c == mask_id ? -INFINITY : row[c];
    if (v > m || (v == m && c < mi)) { m = v; mi = c; }
  }
  s_m[tid] = m; s_i[tid] = mi;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) {
      float m2 = s_m[tid + o]; int i2 = s_i[tid + o];
      if (m2 > s_m[tid] || (m2 == s_m[tid] && i2 < s_i[tid])) { s_m[tid] = m2; s_i[tid] = i2; }
    }
    __syncthreads();
  }
  float M = s_m[0];
  float sum = 0.f;
  for (int c = c0 + tid; c < c1; c += 256) {
    float v = c == mask_id ? -INFINITY : row[c];
    sum += (M == -INFINITY) ? 0.f : expf(v - M);
  }
  s_s[tid] = sum;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) s_s[tid] += s_s[tid + o];
    __syncthreads();
  }
  if (tid == 0) {
    size_t o = (size_t)r * n_part + p;
    part_max[o] = M; part_sum[o] = s_s[0]; part_idx[o] = s_i[0];
  }
}
void launch_vocab_partials(float* logits, int rows, int V, int chunk, int mask_id, BiasArgs bias, float* part_max,
                           float* part_sum, int32_t* part_idx, int n_part, Gate g, hipStream_t s) {
  hipLaunchKernelGGL(k_vocab_partials, dim3(n_part, rows), dim3(256), 0, s, logits, rows, V, chunk, mask_id, bias,
                     part_max, part_sum, part_idx, n_part, g);
}

// ------------------------------------------------------------------------------------------------
// Per sequence: combine the vocabulary partials into conf / pre (Eq. 3, Eq. 4), evaluate the filter
// p = sigmoid(W2 relu(W1 c + b1) + b2) on the block's confidences (committed positions enter as 1.0),
// unmask where p > tau plus the most confident masked position, advance the block, apply EoTP.
__global__ void __launch_bounds__(1024) k_update(UpdateArgs a, Gate g) {
  if (gate_skip(g)) return;
  __shared__ float s_conf[256];
  __shared__ int s_pred[256];
  __shared__ float s_cin[256];
  __shared__ float s_hid[2][1024];
  __shared__ unsigned char s_masked[256];
  __shared__ unsigned char s_sel[256];
  __shared__ int s_flag[6];   // masked, committed, end-of-text seen, still masked afterwards, first end-of-text, EGP hits
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s = a.s;
  const int gb = a.ctl[CTL_SEQ_GB + b];   // the batch's common block, or this sequence's own
  const int lo = a.P + gb * s;
  int32_t* X = a.X + (size_t)b * a.T;
  int32_t* st = a.state + b * 3;

  const int n_waves = blockDim.x >> 6;
  for (int j = wave; j < s; j += n_waves) {
    size_t base = (size_t)(b * s + j) * a.n_part;
    float m = -INFINITY, sum = 0.f;
    int idx = 0x7fffffff;
    // partials are fetched eight per lane at a time, all loads in flight together, and folded in
    // ascending order of p
    for (int p0 = lane; p0 < a.n_part; p0 += 64 * 8) {
      float pm8[8], ps8[8];
      int pi8[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int p = p0 + 64 * u;
        const bool in = p < a.n_part;
        pm8[u] = in ? a.part_max[base + p] : -INFINITY;
        ps8[u] = in ? a.part_sum[base + p] : 0.f;
        pi8[u] = in ? a.part_idx[base + p] : 0x7fffffff;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float pm = pm8[u], ps = ps8[u];
        const int pi = pi8[u];
        if (pm > m) {
          sum = sum * (m == -INFINITY ? 0.f : expf(m - pm)) + ps;
          m = pm; idx = pi;
        } else if (pm > -INFINITY) {
          sum += ps * expf(pm - m);
          if (pm == m && pi < idx) idx = pi;
        }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      float m2 = __shfl_xor(m, o, 64), s2 = __shfl_xor(sum, o, 64);
      int i2 = __shfl_xor(idx, o, 64);
      float M = fmaxf(m, m2);
      float f1 = (m == -INFINITY) ? 0.f : expf(m - M), f2 = (m2 == -INFINITY) ? 0.f : expf(m2 - M);
      sum = sum * f1 + s2 * f2;
      if (m2 > m || (m2 == m && i2 < idx)) idx = i2;
      m = M;
    }
    if (lane == 0) { s_conf[j] = 1.f / sum; s_pred[j] = idx; }
  }
  if (tid < 4 || tid == 5) s_flag[tid] = 0;
  if (tid == 4) s_flag[4] = 0x7fffffff;
  // step-granular EoTP (Sec. 3.3): the sequence is teff tokens long; block positions at or after
  // teff are discarded: never decoded, and they enter the filter as 1.0 like committed ones
  const int teff = a.teff ? a.teff[b] : a.T;
  __syncthreads();
  if (tid < s) {
    bool mk = X[lo + tid] == a.mask_id && lo + tid < teff;
    s_masked[tid] = mk;
    s_cin[tid] = mk ? s_conf[tid] : 1.0f;
    if (a.conf_out) a.conf_out[b * s + tid] = s_conf[tid];
    if (a.pred_out) a.pred_out[b * s + tid] = s_pred[tid];
    if (mk) atomicAdd(&s_flag[0], 1);   // integer count of masked positions
  }
  __syncthreads();
  const int32_t* ref = a.reference ? a.reference + (size_t)b * a.gen_len + gb * s : nullptr;
  // hidden layers of the filter (none for the single-layer variant), activations alternating
  // between two LDS vectors
  const float* act = s_cin;
  int width = s;
  for (int k = 0; !ref && k + 1 < a.n_layers; ++k) {
    float* nxt = s_hid[k & 1];
    for (int t = tid; t < a.hidden; t += blockDim.x) {
      float acc = a.fb[k][t];
      const float* w = a.fw[k] + (size_t)t * width;
      for (int j = 0; j < width; ++j) acc += w[j] * act[j];
      nxt[t] = fmaxf(acc, 0.f);
    }
    __syncthreads();
    act = nxt;
    width = a.hidden;
  }
  if (tid < s) {
    if (ref) {
      // EGP (Alg. 1): a masked position is unmasked exactly when its prediction is the reference token
      const bool hit = s_masked[tid] && s_pred[tid] == ref[tid];
      s_sel[tid] = hit;
      if (hit) atomicAdd(&s_flag[5], 1);
    } else {
      float z = a.fb[a.n_layers - 1][tid];
      const float* w = a.fw[a.n_layers - 1] + (size_t)tid * width;
      for (int t = 0; t < width; ++t) z += w[t] * act[t];
      float p = 1.f / (1.f + expf(-z));
      if (a.filt_out) a.filt_out[b * s + tid] = p;
      s_sel[tid] = s_masked[tid] && (p > a.tau);
    }
  }
  __syncthreads();
  const int n_masked = s_flag[0];
  const bool mine = !st[2] && st[0] == gb;
  if (ref && mine && n_masked > 0 && tid < s) {
    // the step's training row: confidences as the filter would see them, labels 1 = may be unmasked
    const size_t row = ((size_t)b * a.gen_len + st[1]) * s + tid;
    a.egp_conf[row] = s_cin[tid];
    a.egp_label[row] = (!s_masked[tid] || s_sel[tid]) ? 1.f : 0.f;
  }
  __syncthreads();   // labels are read before the forced position is added to the selection
  // the most confident masked position always goes (in an EGP rollout only when nothing agreed,
  // and then with the reference token)
  if (tid == 0 && n_masked > 0 && !(ref && s_flag[5] > 0)) {
    float best = -INFINITY;
    int bj = -1;
    for (int j = 0; j < s; ++j)
      if (s_masked[j] && (bj < 0 || s_conf[j] > best)) { best = s_conf[j]; bj = j; }
    s_sel[bj] = 1;
  }
  __syncthreads();
  if (tid < s) {
    bool sel = mine && s_sel[tid];
    if (a.unmask_out) a.unmask_out[b * s + tid] = sel ? 1 : 0;
    if (sel) {
      X[lo + tid] = ref ? ref[tid] : s_pred[tid];
      atomicAdd(&s_flag[1], 1);
    }
  }
  __syncthreads();
  if (!mine) return;
  bool complete = s_flag[1] == n_masked;   // also true when nothing was masked
  if (a.eotp == 2) {
    // after this step's commits: the first end-of-text of the response shortens the sequence, and
    // the block is complete when nothing is masked before that point
    const int end = min(lo + s, teff);
    for (int t = a.P + tid; t < end; t += blockDim.x)
      if (X[t] == a.eos_id) atomicMin(&s_flag[4], t);
    __syncthreads();
    const int new_teff = s_flag[4] == 0x7fffffff ? teff : s_flag[4] + 1;
    if (tid < s && lo + tid < new_teff && X[lo + tid] == a.mask_id) atomicAdd(&s_flag[3], 1);
    if (tid == 0 && s_flag[4] != 0x7fffffff) s_flag[2] = 1;
    __syncthreads();
    complete = s_flag[3] == 0;
  } else if (complete && a.eotp) {
    for (int t = a.P + tid; t < lo + s; t += blockDim.x)
      if (X[t] == a.eos_id) s_flag[2] = 1;
  }
  __syncthreads();
  if (tid == 0) {
    if (n_masked > 0) st[1] += 1;
    if (complete) {
      st[0] = gb + 1;
      if (s_flag[2] || gb + 1 >= a.n_blocks) st[2] = 1;
    }
  }
}
void launch_update(const UpdateArgs& a, Gate g, hipStream_t s) {
  hipLaunchKernelGGL(k_update, dim3(a.B), dim3(1024), 0, s, a, g);   // 16 wavefronts share the block's rows
}

// response_i = X[P : P+G], steps, decoded length
// With `teff` (step-granular EoTP) the decoded length is the shortened sequence's response part and
// discarded positions come back as mask_id.  `perm` (after batch compaction; nullptr = identity) maps
// a row of X / state to the sequence it holds: outputs go to that sequence's slot.
__global__ void k_finalize(const int32_t* X, const int32_t* state, const int* teff, const int32_t* perm, int B, int P,
                           int G, int s_len, int mask_id, int32_t* tokens_out, int32_t* steps_out,
                           int32_t* dlen_out) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (tokens_out && i < B * G) {
    int b = i / G, t = i % G;
    int v = X[(size_t)b * (P + G) + P + t];
    if (teff && P + t >= teff[b]) v = mask_id;
    tokens_out[(size_t)(perm ? perm[b] : b) * G + t] = v;
  }
  if (i < B) {
    const int o = perm ? perm[i] : i;
    if (steps_out) steps_out[o] = state[i * 3 + 1];
    if (dlen_out) dlen_out[o] = teff ? teff[i] - P : state[i * 3 + 0] * s_len;
  }
}
void launch_finalize(const int32_t* X, const int32_t* state, const int* teff, const int32_t* perm, int B, int P,
                     int G, int s_len, int mask_id, int32_t* tokens_out, int32_t* steps_out, int32_t* dlen_out,
                     hipStream_t s) {
  int n = B * G;
  hipLaunchKernelGGL(k_finalize, dim3((n + 255) / 256), dim3(256), 0, s, X, state, teff, perm, B, P, G, s_len,
                     mask_id, tokens_out, steps_out, dlen_out);
}

// Step-granular EoTP (Sec. 3.3): teff[b] = index after the first end-of-text token of sequence b's
// response region, or the full length; ctl[CTL_TMAX] = the largest of them.  One workgroup.
__global__ void __launch_bounds__(256) k_seq_len(const int32_t* X, int B, int P, int G, int eos_id, int* teff,
                                                int* ctl) {
  __shared__ int s_first;
  __shared__ int s_max;
  const int tid = threadIdx.x, T = P + G;
  if (tid == 0) s_max = 0;
  for (int b = 0; b < B; ++b) {
    if (tid == 0) s_first = T - 1;   // "none": the sequence keeps its full length
    __syncthreads();
    const int32_t* x = X + (size_t)b * T;
    for (int t = P + tid; t < T; t += 256)
      if (x[t] == eos_id) atomicMin(&s_first, t);
    __syncthreads();
    if (tid == 0) {
      teff[b] = s_first + 1;
      s_max = max(s_max, s_first + 1);
    }
    __syncthreads();
  }
  if (tid == 0) ctl[CTL_TMAX] = s_max;
}
void launch_seq_len(const int32_t* X, int B, int P, int G, int eos_id, int* teff, int* ctl, hipStream_t s) {
  hipLaunchKernelGGL(k_seq_len, dim3(1), dim3(256), 0, s, X, B, P, G, eos_id, teff, ctl);
}

// ------------------------------------------------------------------------------------------------
// Filter training (Sec. 3.2, Eq. 6; Sec. 4.1: AdamW): full-batch epochs on the mean binary
// cross-entropy of sigmoid(W2 relu(W1 c + b1) + b2) against the EGP labels.  One workgroup: the
// model has a few thousand parameters and a data set of a few thousand rows, so the whole of it is
// a latency-bound loop that wants no grid synchronisation.  Parameters and the chunk's
// intermediates live in LDS; every thread owns a few parameters, accumulates their gradient over
// the rows in ascending order (deterministic) and applies the AdamW update.
constexpr int kTrainThreads = 1024;
constexpr int kTrainMaxOwn = 20;                 // parameters per thread
constexpr int kTrainLdsFloats = 36 * 1024;       // 144 KB
int filter_param_count(int s, int hidden, int n_layers) {
  int n = 0;
  for (int k = 0; k < n_layers; ++k) {
    const int in = k == 0 ? s : hidden, out = k == n_layers - 1 ? s : hidden;
    n += out * in + out;
  }
  return n;
}
static int train_chunk_rows(int s, int hidden, int n_layers) {
  const int left = kTrainLdsFloats - filter_param_count(s, hidden, n_layers) - 64;
  int ch = left / (2 * (s + (n_layers - 1) * hidden));
  return ch > 64 ? 64 : ch;
}
int filter_train_supported(int s, int hidden, int n_layers) {
  return n_layers >= 1 && n_layers <= kFilterMaxLayers && s >= 1 && (n_layers == 1 || hidden >= 1) &&
         filter_param_count(s, hidden, n_layers) <= kTrainThreads * kTrainMaxOwn &&
         train_chunk_rows(s, hidden, n_layers) >= 8;
}
__global__ void __launch_bounds__(kTrainThreads) k_filter_train(TrainArgs a, int chunk) {
  extern __shared__ float lds[];
  const int s = a.s, h = a.hidden, L = a.n_layers, tid = threadIdx.x;
  // layer k maps width in(k) to width out(k); its parameters sit at off(k) (weights, then biases).
  // Closed forms rather than tables, so nothing here is indexed dynamically out of registers.
  auto in = [&](int k) { return k == 0 ? s : h; };
  auto out = [&](int k) { return k == L - 1 ? s : h; };
  const int first = h * s + h, mid = h * h + h;            // parameters of layer 0 / of a hidden->hidden layer
  auto off = [&](int k) { return k == 0 ? 0 : first + (k - 1) * mid; };
  const int n_params = off(L - 1) + s * in(L - 1) + s;
  auto layer_of = [&](int p) {
    if (L == 1 || p < first) return 0;
    const int k = 1 + (p - first) / mid;
    return k < L - 1 ? k : L - 1;
  };
  // LDS: parameters, then per chunk the input of every layer (A(0) = the confidence rows) and the
  // loss gradient at every layer's pre-activation (D), then reduction scratch
  float* th = lds;
  float* const baseA = th + n_params;
  float* const baseD = baseA + chunk * (s + (L - 1) * h);
  auto A = [&](int k) { return baseA + (k == 0 ? 0 : chunk * s + (k - 1) * chunk * h); };
  auto D = [&](int k) { return baseD + k * chunk * h; };
  float* red = baseD + chunk * ((L - 1) * h + s);          // 64 floats
  for (int p = tid; p < n_params; p += kTrainThreads) {
    const int k = layer_of(p), q = p - off(k), nw = out(k) * in(k);
    th[p] = q < nw ? a.w[k][q] : a.b[k][q - nw];
    a.opt_state[p] = 0.f;
    a.opt_state[n_params + p] = 0.f;
  }
  __syncthreads();
  const float inv_m = 1.f / ((float)a.n * (float)s);
  float b1t = 1.f, b2t = 1.f;     // beta^t
  for (int ep = 0; ep < a.epochs; ++ep) {
    float g[kTrainMaxOwn];
#pragma unroll
    for (int o = 0; o < kTrainMaxOwn; ++o) g[o] = 0.f;
    float loss = 0.f;
    for (long long c0 = 0; c0 < a.n; c0 += chunk) {
      const int rows = (int)min((long long)chunk, a.n - c0);
      for (int i = tid; i < rows * s; i += kTrainThreads) A(0)[i] = a.conf[c0 * s + i];
      __syncthreads();
      for (int k = 0; k + 1 < L; ++k) {                            // hidden activations
        const float* W = th + off(k);
        const float* Bv = W + out(k) * in(k);
        for (int i = tid; i < rows * out(k); i += kTrainThreads) {
          const int r = i / out(k), t = i % out(k);
          float acc = Bv[t];
          for (int j = 0; j < in(k); ++j) acc += W[t * in(k) + j] * A(k)[r * in(k) + j];
          A(k + 1)[i] = fmaxf(acc, 0.f);
        }
        __syncthreads();
      }
      {                                                            // logits, loss, dL/dz
        const int k = L - 1;
        const float* W = th + off(k);
        const float* Bv = W + s * in(k);
        for (int i = tid; i < rows * s; i += kTrainThreads) {
          const int r = i / s, j = i % s;
          float z = Bv[j];
          for (int t = 0; t < in(k); ++t) z += W[j * in(k) + t] * A(k)[r * in(k) + t];
          const float y = a.label[c0 * s + i];
          loss += fmaxf(z, 0.f) + log1pf(expf(-fabsf(z))) - y * z;   // softplus(z) - y z
          D(k)[i] = (1.f / (1.f + expf(-z)) - y) * inv_m;
        }
        __syncthreads();
      }
      for (int k = L - 1; k > 0; --k) {                            // back through layer k and the ReLU before it
        const float* W = th + off(k);
        for (int i = tid; i < rows * in(k); i += kTrainThreads) {
          const int r = i / in(k), t = i % in(k);
          float acc = 0.f;
          for (int j = 0; j < out(k); ++j) acc += D(k)[r * out(k) + j] * W[j * in(k) + t];
          D(k - 1)[i] = A(k)[i] > 0.f ? acc : 0.f;
        }
        __syncthreads();
      }
#pragma unroll
      for (int o = 0; o < kTrainMaxOwn; ++o) {                     // gradient of the owned parameters
        const int p = tid + o * kTrainThreads;
        if (p >= n_params) break;
        const int k = layer_of(p), q = p - off(k), nw = out(k) * in(k);
        float acc = 0.f;
        if (q < nw) {
          const int t = q / in(k), j = q % in(k);
          for (int r = 0; r < rows; ++r) acc += D(k)[r * out(k) + t] * A(k)[r * in(k) + j];
        } else {
          const int t = q - nw;
          for (int r = 0; r < rows; ++r) acc += D(k)[r * out(k) + t];
        }
        g[o] += acc;
      }
      __syncthreads();
    }
    // loss of the epoch (before its update)
    if (a.loss_out) {
#pragma unroll
      for (int of = 32; of > 0; of >>= 1) loss += __shfl_xor(loss, of, 64);
      if ((tid & 63) == 0) red[tid >> 6] = loss;
      __syncthreads();
      if (tid == 0) {
        float tot = 0.f;
        for (int w = 0; w < kTrainThreads / 64; ++w) tot += red[w];
        a.loss_out[ep] = tot * inv_m;
      }
    }
    // AdamW, decoupled weight decay
    b1t *= a.beta1;
    b2t *= a.beta2;
#pragma unroll
    for (int o = 0; o < kTrainMaxOwn; ++o) {
      const int p = tid + o * kTrainThreads;
      if (p >= n_params) break;
      const float m = a.beta1 * a.opt_state[p] + (1.f - a.beta1) * g[o];
      const float v = a.beta2 * a.opt_state[n_params + p] + (1.f - a.beta2) * g[o] * g[o];
      a.opt_state[p] = m;
      a.opt_state[n_params + p] = v;
      const float mh = m / (1.f - b1t), vh = v / (1.f - b2t);
      th[p] = th[p] - a.lr * (mh / (sqrtf(vh) + a.eps) + a.weight_decay * th[p]);
    }
    __syncthreads();
  }
  for (int p = tid; p < n_params; p += kTrainThreads) {
    const int k = layer_of(p), q = p - off(k), nw = out(k) * in(k);
    if (q < nw) a.w[k][q] = th[p];
    else a.b[k][q - nw] = th[p];
  }
}
void launch_filter_train(const TrainArgs& a, hipStream_t s) {
  const int chunk = train_chunk_rows(a.s, a.hidden, a.n_layers);
  const int n_params = filter_param_count(a.s, a.hidden, a.n_layers);
  const size_t smem =
      (size_t)(n_params + chunk * 2 * (a.s + (a.n_layers - 1) * a.hidden) + 64) * sizeof(float);
  static DynLdsAttr attr;
  attr.ensure(reinterpret_cast<const void*>(k_filter_train), kTrainLdsFloats * (int)sizeof(float));
  hipLaunchKernelGGL(k_filter_train, dim3(1), dim3(kTrainThreads), smem, s, a, chunk);
}

}  // namespace l2pd
