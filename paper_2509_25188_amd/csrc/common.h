// Internal declarations shared by the HIP translation units of libl2pd.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>

#include <atomic>

#include "../../include/l2pd.h"

namespace l2pd {

typedef __hip_bfloat16 bf16;

// Device control block (int32 words).  Written by k_prepare at the start of every step.  The words
// from CTL_SEQ_GB on hold the active block of every sequence: the batch's common one in lock step,
// the sequence's own with per-sequence block pointers.
// After them (from CTL_SEQ_GB + max_batch on; k_prepare is told where) one word per sequence: 1 once it is done.
enum { CTL_GB = 0, CTL_ALL_DONE = 1, CTL_ACTIVE = 2, CTL_TMAX = 3, CTL_WORDS = 8, CTL_SEQ_GB = 8 };

// Every kernel of a step is gated: once decoding has stopped (or, with the prefix cache, once the
// block the host enqueued it for is finished) it returns at once, so steps that the host enqueued
// ahead of the device's progress cost a launch and nothing else.
struct Gate {
  const int* ctl;   // nullptr: never skip
  int expect_gb;    // >= 0: skip unless ctl[CTL_GB] == expect_gb
};
__device__ __forceinline__ bool gate_skip(const Gate& g) {
  if (!g.ctl) return false;
  if (g.ctl[CTL_ALL_DONE]) return true;
  return g.expect_gb >= 0 && g.ctl[CTL_GB] != g.expect_gb;
}

// Maps a compact row index r (b * rows_per_seq + j) to a row of a [B, seq_stride] array:
//   b * seq_stride + off_base + gb_b * off_per_gb + j,  gb_b = sequence b's active block from the control block.
struct RowMap {
  int rows_per_seq, seq_stride, off_base, off_per_gb;
};
__device__ __forceinline__ int map_row(const RowMap& m, int r, const int* ctl) {
  int gb = (m.off_per_gb && ctl) ? ctl[CTL_SEQ_GB + r / m.rows_per_seq] : 0;
  return (r / m.rows_per_seq) * m.seq_stride + m.off_base + gb * m.off_per_gb + (r % m.rows_per_seq);
}

// Raises a kernel's dynamic-LDS limit once per device: the attribute belongs to the device's copy of
// the kernel, and launchers may be called from several host threads (setting it twice is harmless).
struct DynLdsAttr {
  std::atomic<unsigned long long> done{0};
  void ensure(const void* kernel, int bytes) {
    int dev = 0;
    (void)hipGetDevice(&dev);
    const unsigned long long bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return;
    (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    done.fetch_or(bit, std::memory_order_release);
  }
};

// ---- small kernels (kernels_misc.hip) ----
void launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s);
void launch_rope_table(float* cos_t, float* sin_t, int max_pos, int head_dim, float base, hipStream_t s);
void launch_init_decode(int32_t* X, const int32_t* prompt, int B, int P, int G, int mask_id, int32_t* state,
                        int* ctl, hipStream_t s);
void launch_prepare(const int32_t* state, int B, int n_blocks, int ragged, int* ctl, hipStream_t s,
                    int done_at = 0);   // done_at > 0: also ctl[done_at + b] = sequence b's done flag
void launch_embed(float* h, const void* emb, int dtype, const int32_t* tokens, RowMap tokmap, int rows, int d,
                  Gate g, hipStream_t s);
// h (+= the sum part[0] + ... + part[n_parts-1], formed first, in that order, when given) -> y = rmsnorm(h) * gain, rows taken
// through `src`.  part z is at parts + z * part_stride, laid out like h.  The sum is written back to h
// when `write_back` is set; the final norm before the LM head leaves h alone (h is dead after it, and
// two head rows may map to one row of h, so a write-back would race).
// quad_tiled (bf16, d within the one-row-per-workgroup kernels' range): y is written in the
// layout gemm_qkv_a_quad_tiled() describes instead of row-major; the arithmetic is the same.
void launch_rmsnorm(float* h, const float* parts, int n_parts, size_t part_stride, RowMap src, const void* gain,
                    int dtype, void* y, int rows, int d, float eps, bool write_back, Gate g, hipStream_t s,
                    bool quad_tiled = false);
constexpr int kFilterMaxLayers = 4;
struct UpdateArgs {
  int32_t* X;            // [B, T]
  int32_t* state;        // [B, 3]
  int B, P, T, s, n_blocks, mask_id, eos_id, eotp;
  const float* part_max; // [B*s, n_part]
  const float* part_sum;
  const int32_t* part_idx;
  int n_part;
  // filter: n_layers layers of widths s -> hidden -> ... -> hidden -> s (layer k: fw[k] [out, in], fb[k] [out])
  const float* fw[kFilterMaxLayers];
  const float* fb[kFilterMaxLayers];
  int n_layers, hidden;
  float tau;
  float* conf_out;       // optional taps [B, s]
  int32_t* pred_out;
  float* filt_out;
  uint8_t* unmask_out;
  int* ctl;
  const int* teff;       // step-granular EoTP: per-sequence length in force (else null)
  // EGP rollout (Alg. 1): unmask where the prediction equals the reference answer; one training row per step
  const int32_t* reference;   // [B, gen_len] or null
  float* egp_conf;            // [B, gen_len, s]: row = step index of the sequence
  float* egp_label;
  int gen_len;
};
void launch_update(const UpdateArgs& a, Gate g, hipStream_t s);
void launch_finalize(const int32_t* X, const int32_t* state, const int* teff, const int32_t* perm, int B, int P,
                     int G, int s_len, int mask_id, int32_t* tokens_out, int32_t* steps_out, int32_t* dlen_out,
                     hipStream_t s);
// live sequences to the leading rows (stable), src copies -> dst copies; perm_src nullptr = identity
void launch_compact(const int32_t* X_src, int32_t* X_dst, const int32_t* state_src, int32_t* state_dst,
                    const int32_t* perm_src, int32_t* perm_dst, int B, int T, hipStream_t s);
// `epochs` full-batch AdamW steps on the binary cross-entropy of Eq. 6 for a filter of n_layers layers
// (widths s -> hidden -> ... -> hidden -> s), in place.
struct TrainArgs {
  float* w[kFilterMaxLayers];   // device, updated in place; layer k: [out, in]
  float* b[kFilterMaxLayers];
  int n_layers, s, hidden;
  const float* conf;          // [n, s]
  const float* label;         // [n, s]
  long long n;
  int epochs;
  float lr, beta1, beta2, eps, weight_decay;
  float* opt_state;           // [2 * n_params], zeroed by the kernel
  float* loss_out;            // [epochs] or null
};
int filter_param_count(int s, int hidden, int n_layers);
int filter_train_supported(int s, int hidden, int n_layers);
void launch_filter_train(const TrainArgs& a, hipStream_t s);
void launch_seq_len(const int32_t* X, int B, int P, int G, int eos_id, int* teff, int* ctl, hipStream_t s);
// keys[b] = base + ctl[CTL_SEQ_GB + b] * per_gb: keys a sequence's block rows may see under the prefix cache
void launch_block_keys(const int* ctl, int B, int base, int per_gb, int* keys, hipStream_t s);

// ---- vocabulary reduction over materialised logits (fp32 path and the logits tap) ----
struct BiasArgs {
  int token_id, gen_pos_from, block_len;
  float value;           // 0: off
};
// partials over column chunks of `chunk` logits: max, sum exp(x - max), argmax (lowest id on ties),
// mask_id excluded.  logits [rows, V] are modified in place by the bias first.
void launch_vocab_partials(float* logits, int rows, int V, int chunk, int mask_id, BiasArgs bias, float* part_max,
                           float* part_sum, int32_t* part_idx, int n_part, Gate g, hipStream_t s);

// ---- fp32 path (kernels_f32.hip) ----
// C[M,N] (+)= A[M,K] * W[N,K]^T
void launch_gemm_f32(const float* A, const float* W, float* C, int M, int N, int K, int accumulate, Gate g,
                     hipStream_t s);
// rotate q [rows, d] in place and copy/rotate k, v rows into the [B, Tmax, d] key/value stores at pos0 + t
// (seq_gb / pos_per_gb: per-sequence position offsets as in QkvEpilogue)
void launch_rope_store_f32(float* q, const float* k, const float* v, float* kstore, float* vstore, int B, int Tq,
                           int pos0, int Tmax, int H, int Dh, const float* cos_t, const float* sin_t,
                           const int* seq_gb, int pos_per_gb, Gate g, hipStream_t s);
void launch_attn_f32(const float* q, const float* kstore, const float* vstore, float* out, int B, int Tq, int Tk,
                     int Tmax, int H, int Dh, const int* tk_dev, Gate g, hipStream_t s);
void launch_swiglu_f32(const float* gate, const float* up, float* act, size_t n, Gate g, hipStream_t s);

// ---- bf16 path ----
struct QkvEpilogue {
  bf16* q;               // [rows, d]
  bf16* kstore;          // [B, Tpad, d]
  bf16* vtstore;         // [B, H, Dh, Tpad]
  const float *cos_t, *sin_t;  // [max_pos, Dh/2]
  int Tq, pos0, Tpad, H, Dh, d;
  // per-sequence block pointers with a K/V cache: row t of sequence b sits at position
  // pos0 + seq_gb[b] * pos_per_gb + t (seq_gb = the control block's per-sequence active blocks); null: pos0 + t
  const int* seq_gb;
  int pos_per_gb;
};
__device__ __forceinline__ int seq_pos_offset(const int* seq_gb, int per_gb, int b) {
  return seq_gb ? seq_gb[b] * per_gb : 0;
}
// Whether the fused Q/K/V (M rows, model width d, head size Dh) / gate/up (M rows, FFN width F) GEMM of
// depth K reads its A operand straight into registers; it then expects it "quad-tiled": groups of four rows, and inside a group the
// 16-byte chunks (8 bf16) of the four rows interleaved, element (r, k) at
//   ((r / 4) * (K / 8) + k / 8) * 32 + (r % 4) * 8 + k % 8,
// so that the 32 rows x 2 chunks a wavefront feeds to one MFMA K-step are eight whole 128-byte lines.
// The buffer needs its row count rounded up to four.  A function of the launch shape only; the producer of
// A (the RMSNorm before the GEMM) asks the same question.
bool gemm_qkv_a_quad_tiled(int M, int d, int K, int Dh);
bool gemm_swiglu_a_quad_tiled(int M, int F, int K);
// the same question for the [N, K] projections that write split-K partials (output and down projection), whose
// A operands are written by the attention kernel and by the gate/up GEMM's epilogue
bool gemm_partial_a_quad_tiled(int M, int N, int K);
// and for the LM head, whose A operand the final RMSNorm writes
bool gemm_lmhead_a_quad_tiled(int M, int V, int K);
void launch_gemm_qkv_bf16(const bf16* A, const bf16* wq, const bf16* wk, const bf16* wv, int M, int K,
                          const QkvEpilogue& e, Gate g, hipStream_t s);
// partial[z][M,N] = A[:, z-th K slice] * W[:, slice]^T, z < splits (1 or 2)
void launch_gemm_partial_bf16(const bf16* A, const bf16* W, float* parts, size_t part_stride, int M, int N, int K,
                              int splits, Gate g, hipStream_t s);
// Few-row GEMMs (block-only steps of the cached decode modes, at most kSkinnyRows rows) stream their
// weights once; K is split until a launch has a few hundred workgroups, each K range staying a
// multiple of the 64-wide stage.
constexpr int kSkinnyRows = 64;
constexpr int kSkinnyRowsAttn = 64;   // B * Tq up to which attention may chunk the keys across workgroups
int skinny_splits(int N, int K);
int wide_splits(int M, int N, int K);   // partial buffers the wide path's [d, d] / [d, F] projections write, at most 8
void launch_gemm_skinny_bf16(const bf16* A, const bf16* w0, const bf16* w1, const bf16* w2, int n_sub, float* parts,
                             size_t part_stride, int M, int N, int K, int splits, Gate g, hipStream_t s);
// sums of the skinny GEMM's partials -> rotated q, K store, V^T store / SiLU(gate) * up
void launch_skinny_qkv_finish(const float* parts, int n_parts, size_t part_stride, int rows, const QkvEpilogue& e,
                              Gate g, hipStream_t s);
void launch_skinny_swiglu_finish(const float* parts, int n_parts, size_t part_stride, int rows, int F, bf16* act,
                                 Gate g, hipStream_t s);
// act[M, F] = silu(A Wg^T) * (A Wu^T); few rows take the fused few-row tiles when swiglu_few_rows_fused says so
bool swiglu_few_rows_fused(int M, int F);
void launch_gemm_swiglu_bf16(const bf16* A, const bf16* wg, const bf16* wu, bf16* act, int M, int F, int K, Gate g,
                             hipStream_t s, bool act_quad_tiled = false);
struct LmHeadEpilogue {
  float* logits;         // optional [M, V]
  float* part_max;       // optional [M, n_part]
  float* part_sum;
  int32_t* part_idx;
  int n_part;            // = V / 128 rounded up
  int mask_id;
  BiasArgs bias;         // applied when value != 0 (needs ctl for the active block)
};
int lmhead_n_part(int V);
void launch_gemm_lmhead_bf16(const bf16* A, const bf16* W, int M, int V, int K, const LmHeadEpilogue& e, Gate g,
                             hipStream_t s);
// out_quad_tiled: write `out` in the layout gemm_partial_a_quad_tiled() asks for instead of row-major
void launch_attn_bf16(const bf16* q, const bf16* kstore, const bf16* vtstore, bf16* out, int B, int Tq, int Tk,
                      int Tpad, int H, int Dh, float* chunk_ws, size_t chunk_ws_bytes, const int* tk_dev, Gate g,
                      hipStream_t s, bool out_quad_tiled = false);
// bytes of chunk workspace that lets launch_attn_bf16 spread few queries' keys over workgroups
inline size_t attn_chunk_ws_bytes(int H, int Dh) { return (size_t)kSkinnyRowsAttn * H * 16 * (Dh + 2) * 4; }

}  // namespace l2pd
