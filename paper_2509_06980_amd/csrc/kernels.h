// Host-side launchers of the rollout kernels.  All pointers are device pointers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rl_common.h"

// One attention work item: up to 16 / (n_q / n_kv) batch rows and a range of pages.  Decode: one
// row; long contexts are cut into several items ("parts") so that workgroups carry similar amounts
// of keys / values whatever the mix of context lengths.  Chunked prefill: several consecutive rows
// of one trajectory, always one part.  Shared-prefix decode (gather = 1): the rows are members of a
// group of trajectories whose first pages are the same physical pages (a forked prompt); the item
// reads those pages once for all of them, every key visible to every row, and always leaves a
// partial result that the merge step combines with each member's own remainder.
struct AttnItem {
  int32_t row0;    // first batch row; gather: index of the first entry in the row list
  int32_t nrows;   // rows in this item
  int32_t slot;    // trajectory slot (row of the page table)
  int32_t pos0;    // position of row0; row r sits at pos0 + r and sees positions <= pos0 + r
  int32_t pg_lo;   // pages [pg_lo, pg_hi) of the trajectory are this item's share
  int32_t pg_hi;
  int32_t part;    // >= 0: partial result goes to scratch slot `part`; -1: the item is complete
  int32_t gather;  // bit 0: batch rows are rowlist[row0 + r] (shared-prefix item); bits 8..: number
                   // of leading pages of the trajectory that other trajectories share (decode: read
                   // with plain, cached loads; the rest is streamed)
};
// Rows whose attention was cut into parts: merge, in this order, the shared-prefix parts (scratch
// slots [sfirst, sfirst + snparts), where the row is row `sr` of the item) and the row's own parts
// (slots [first, first + nparts), row 0 of the item).
struct AttnMerge {
  int32_t row, first, nparts, sfirst, snparts, sr, pad0, pad1;
};

struct KvPool {      // one layer
  void* k;           // [pages][n_kv][16 * d] elements (bf16 / fp32, or one byte each: 8-bit cache)
  void* v;
};

struct ModelDims {
  int L, H, nq, nkv, d, I, V;
  float eps;
  int qk_norm;
  int max_pages_per_traj;  // row stride of the page table
  int kv_fp8;              // keys / values cached as E4M3 codes (MFMA path, head_dim 128 only)
};

// ---- generic kernels (TA: activation type, TW: weight type; float or bf16_t) -------------
template <typename TW>
void launch_embed(hipStream_t s, const TW* E, const int32_t* tok, float* h, int M, int H);

// out = rmsnorm(h) * g.  ATILE: write `out` in A-tile layout (bf16 MFMA path).
template <typename TW, typename TA>
void launch_rmsnorm(hipStream_t s, const float* h, const TW* g, TA* out, int M, int H, float eps,
                    bool atile);

// C[M,N] (+)= A[M,K] * W[N,K]^T, fp32 accumulate, C row-major fp32.
template <typename TA, typename TW>
void launch_gemm_generic(hipStream_t s, const TA* A, const TW* W, float* C, int M, int N, int K,
                         bool accumulate);

// q/k per-head RMSNorm (optional), rotate-half RoPE, q -> qout [M, nq*d] row-major, k and v into
// the paged cache at (page_table[slot][pos/16], pos%16).  The projection arrives as n_part
// split-K partial sums (qkv + p * part_stride), added here in ascending order.
template <typename TW, typename TA, typename TKV, bool SWZ>
void launch_qkrope(hipStream_t s, const float* qkv, int n_part, size_t part_stride, const TW* gq,
                   const TW* gk, const float* rope_cs, const int32_t* row_pos,
                   const int32_t* row_slot, const int32_t* page_table, TA* qout, KvPool pool,
                   const ModelDims& md, int M);

// h += sum of n_part split-K partial sums (ascending order), then out = rmsnorm(h) * g in A-tile
// layout (bf16 MFMA path).  rows != null: gather: output row i is made from row rows[i] of h /
// parts (M = number of gathered rows).
void launch_add_rmsnorm(hipStream_t s, float* h, const float* parts, int n_part, size_t part_stride,
                        const bf16_t* g, bf16_t* out, int M, int H, float eps,
                        const int32_t* rows = nullptr);

template <typename TA, typename TKV, bool SWZ>
void launch_attention_generic(hipStream_t s, const TA* q, KvPool pool, const int32_t* row_pos,
                              const int32_t* row_slot, const int32_t* page_table, TA* o,
                              const ModelDims& md, int M, bool o_atile);

// m = silu(gu[:, :I]) * gu[:, I:]
template <typename TA>
void launch_swiglu(hipStream_t s, const float* gu, TA* m, int M, int I, bool atile);

// ---- MFMA kernels (bf16, head_dim 128) -------------------------------------------------------
enum GemmEpilogue { EPI_STORE = 0, EPI_SWIGLU = 2, EPI_LSE = 3, EPI_STORE_MAX = 4 };
// A: bf16 A-tile layout [ceil(M/128)*128, K]; Wp: repacked weights (see repack kernel).
// EPI_STORE: split-K slice z writes its fp32 partial sum to C + z * M * N (row-major [M, N]); the
// consumer adds the `splits` partials.  EPI_SWIGLU (splits = 1): C is bf16 A-tile [.., N/2], gate
// and up interleaved in 16-column groups.  nw = waves per workgroup (2 or 4): tile 128 x 32*nw.
// K % 64 == 0, N % 32 == 0.  Returns the number of splits actually used.
int launch_gemm_mfma(hipStream_t s, const bf16_t* A, const bf16_t* Wp, void* C, int M, int N,
                     int K, int epilogue, int splits, int nw);
// lm-head fused with the log-softmax of the masked log-prob pass: for each of the M rows of A
// (bf16 A-tile layout) lp[row] = log softmax(z / T)[tgt[row]] with z = A[row] . Wp^T (V logits, never
// stored) and scale_c = log2(e) / T.  part: scratch of M * (V / 32) float pairs; zt: M floats.
void launch_lm_head_logprob(hipStream_t s, const bf16_t* A, const bf16_t* Wp, int M, int V, int K,
                            const int32_t* tgt, float scale_c, float* part, float* zt, float* lp);
// lm-head of a decode step (final norm -> lm-head -> sampler): logits[M, V] fp32 row-major and, from
// the same epilogue, stripmax[M, V / 32]: the maximum of every 32 consecutive logits of a row, from
// which the sampler takes the row maximum without a pass over the logits.  V % 32 == 0.
void launch_lm_head_logits(hipStream_t s, const bf16_t* A, const bf16_t* Wp, float* logits, int M,
                           int V, int K, float* stripmax);
// W[N,K] row-major -> operand strips.  interleave16: rows come from two matrices Wg, Wu
// ([N/2,K] each) interleaved in groups of 16 (gate, up, gate, up, ...).
void launch_repack_weight(hipStream_t s, const bf16_t* W, const bf16_t* Wu, bf16_t* Wp, int N,
                          int K, bool interleave16);

// paged GQA attention over work items; q bf16 row-major [M, nq*128]; o bf16 A-tile [.., nq*128].
// Decode (prefill = false): single-row items, possibly cut into parts; scratch: fp32
// [part slots][nkv][16 * 130] for items with part >= 0, merged by `merges`.
// Prefill: items of up to 4 * RL_PREFILL_CB * 16/G consecutive rows of one trajectory (G = n_q /
// n_kv), one part each.
#ifndef RL_PREFILL_CB
#define RL_PREFILL_CB 2   // 16-column blocks per wave of the prefill kernel (2: still two waves per SIMD)
#endif
void launch_attention_mfma(hipStream_t s, const bf16_t* q, KvPool pool, const AttnItem* items,
                           int n_items, const AttnMerge* merges, int n_merges,
                           const int32_t* rowlist, const int32_t* page_table, bf16_t* o,
                           float* scratch, const ModelDims& md, bool prefill);

// ---- sampler ---------------------------------------------------------------------------------
struct SamplerScratch {
  float* segmax;     // [rows * nseg]
  int32_t* segarg;   // [rows * nseg]
  uint64_t* segw;    // [rows * nseg]
  float* sege;       // [rows * nseg]
};
#define RL_SAMPLER_SEG 4096
static inline int sampler_nseg(int V) { return (V + RL_SAMPLER_SEG - 1) / RL_SAMPLER_SEG; }

// For each row of fp32 logits [rows, V] (row stride ldz): id and log-prob.
//  scale_c = fl32(log2(e)/T) (T > 0) or fl32(log2(e)) with greedy = 1.
//  u32 != null: use these draws; else draw from (seed, row_traj[r], row_newpos[r]).
//  forced != null: id = forced[r] (no draw).  out_mask != null: logprob forced to 0 where
//  out_mask[r] != 0.
//  stripmax != null (not with greedy): [rows, nstrips] maxima that together cover each row (from
//  the lm-head epilogue); the pass over the logits that finds the row maximum is then left out.
void launch_sampler(hipStream_t s, const float* logits, size_t ldz, int rows, int V, float scale_c,
                    int greedy, const uint32_t* u32, uint64_t seed, const int32_t* row_traj,
                    const int32_t* row_newpos, const int32_t* forced, const uint8_t* out_mask,
                    SamplerScratch sc, int32_t* ids_out, float* logp_out,
                    const float* stripmax = nullptr, int nstrips = 0);

// Sets the thread's rl_last_error() message and returns `code` (defined beside the C boundary).
int rl_fail(int code, const char* msg);
// Looks up the current device's copy of the sampler's fixed scratch array (used by the entry point
// that allocates nothing); 0 or a hipError_t.  Model load calls it so that the lookup has happened
// before a caller's first sampling call.
int sampler_noalloc_prepare();

// Masked GRPO objective (forward value).  advantages: adv[i] of trajectory i within its group of G
// consecutive rewards, (r - mean) / (std + eps_std), std with divisor G - ddof; also clears the 3 n
// accumulators acc.  terms: for every row k of segment (traj, k0, k1) with use[k] != 0 adds
// min(rho A, clip(rho, 1 -+ clip_eps) A) - beta k3 (rho = exp(lp - old_lp), k3 from ref_lp - lp;
// ref_lp null: no KL term) to the trajectory's accumulators.  finish: out[0] = mean over
// trajectories of their mean term, out[1] = likewise for k3, out[2] = number of tokens.
void launch_grpo_advantages(hipStream_t s, const float* rewards, int n, int G, double eps_std, int ddof,
                            double* adv, double* acc);
void launch_grpo_terms(hipStream_t s, const float* lp, const float* old_lp, const float* ref_lp,
                       const int32_t* use, const int32_t* segs, int nseg, const double* adv,
                       double clip_eps, double beta, double* acc);
void launch_grpo_finish(hipStream_t s, const double* acc, int n, double* out);

// copy one page (all kv heads) within a layer pool: dst page <- src page; n pairs
void launch_copy_pages(hipStream_t s, KvPool pool, const int32_t* src_dst_pairs, int n_pairs,
                       size_t page_bytes);
// page_table[upd[3i] * stride + upd[3i+1]] = upd[3i+2]
void launch_page_table_update(hipStream_t s, int32_t* page_table, const int32_t* upd, int n,
                              int stride);
