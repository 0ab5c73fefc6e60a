// Sampling a_t ~ pi_theta(a | s_t) (paper Section 2.2) from a row of fp32 logits, bit-reproducibly.
//
// The softmax is turned into integer weights so that the cumulative sums are associative and any
// parallel reduction order gives the same token:
//   m = max z;  t_i = fl(fl(z_i - m) * c),  c = fl(log2(e) / T);
//   e_i = 2^floor(t_i) * P(t_i - floor(t_i)), P a fixed degree-6 polynomial evaluated by Horner
//   with separately rounded multiply and add; e_i = 0 below 2^-40;
//   w_i = floor(e_i * 2^32);  W = sum w_i;  r = (u32 * W) >> 32;  id = min{k : w_0+..+w_k > r}.
// The log-prob is t_id * ln 2 - ln(sum e_i).  This file must be compiled with
// -ffp-contract=off: a fused multiply-add would change the weights' bits.
//
// Three launches over segments of RL_SAMPLER_SEG logits: per-segment max, per-segment weight sums,
// then one workgroup per row locates the segment and the token inside it.
#include "../../include/rl_rollout.h"
#include "kernels.h"

#pragma clang fp contract(off)

__device__ __forceinline__ void exp2_weight(float z, float m, float c, float& e, uint64_t& w) {
  const float C1 = 0x1.62e430p-1f, C2 = 0x1.ebfc40p-3f, C3 = 0x1.c69f6ap-5f, C4 = 0x1.3c4a8ap-7f,
              C5 = 0x1.4ca4ccp-10f, C6 = 0x1.b4d1e4p-13f;
  float t = __fmul_rn(__fsub_rn(z, m), c);
  float n = floorf(t);
  float r = __fsub_rn(t, n);
  float p = C6;
  p = __fadd_rn(__fmul_rn(p, r), C5);
  p = __fadd_rn(__fmul_rn(p, r), C4);
  p = __fadd_rn(__fmul_rn(p, r), C3);
  p = __fadd_rn(__fmul_rn(p, r), C2);
  p = __fadd_rn(__fmul_rn(p, r), C1);
  p = __fadd_rn(__fmul_rn(p, r), 1.0f);
  if (n < -40.0f) {
    e = 0.f;
    w = 0;
  } else {
    e = ldexpf(p, (int)n);
    w = (uint64_t)__fmul_rn(e, 4294967296.0f);
  }
}

__host__ __device__ __forceinline__ uint32_t splitmix_u32(uint64_t seed, int32_t traj, int32_t pos) {
  uint64_t ctr = (((uint64_t)(uint32_t)traj << 32) | (uint64_t)(uint32_t)pos) + 1ull;
  uint64_t z = seed + ctr * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return (uint32_t)(z >> 32);
}

extern "C" uint32_t rl_uniform_u32(uint64_t seed, int32_t traj_id, int32_t position) {
  return splitmix_u32(seed, traj_id, position);
}

// grid (nseg, rows), block 256
__global__ void seg_max_kernel(const float* __restrict__ z, size_t ldz, int V,
                               float* __restrict__ segmax, int32_t* __restrict__ segarg) {
  __shared__ float sv[4];
  __shared__ int si[4];
  int seg = blockIdx.x, row = blockIdx.y, nseg = gridDim.x;
  const float* zr = z + (size_t)row * ldz;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = 0; i < RL_SAMPLER_SEG / 256; i++) {
    int idx = seg * RL_SAMPLER_SEG + i * 256 + threadIdx.x;
    if (idx < V) {
      float v = zr[idx];
      if (v > best || (v == best && idx < bi)) { best = v; bi = idx; }
    }
  }
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(best, o, 64);
    int oi = __shfl_xor(bi, o, 64);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
  }
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < 4; k++)
      if (sv[k] > best || (sv[k] == best && si[k] < bi)) { best = sv[k]; bi = si[k]; }
    segmax[(size_t)row * nseg + seg] = best;
    segarg[(size_t)row * nseg + seg] = bi;
  }
}

// grid rows, block 256: the row maximum from the per-strip maxima that the lm-head epilogue left,
// written into every per-segment slot of the row, so that the two kernels below find it where
// seg_max_kernel would have put the segment maxima (the maximum does not depend on the order of
// the reduction: same bits either way).  The arg-max is not formed (sampling does not need it).
__global__ void row_max_kernel(const float* __restrict__ stripmax, int nstrips, int nseg,
                               float* __restrict__ segmax, int32_t* __restrict__ segarg) {
  __shared__ float red[4];
  const int row = blockIdx.x;
  const float* p = stripmax + (size_t)row * nstrips;
  float m = -INFINITY;
  for (int j = threadIdx.x; j < nstrips; j += 256) m = fmaxf(m, p[j]);
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  for (int k = threadIdx.x; k < nseg; k += 256) {
    segmax[(size_t)row * nseg + k] = m;
    segarg[(size_t)row * nseg + k] = 0;
  }
}

// grid (nseg, rows), block 256
__global__ void seg_weight_kernel(const float* __restrict__ z, size_t ldz, int V, float c,
                                  const float* __restrict__ segmax, uint64_t* __restrict__ segw,
                                  float* __restrict__ sege) {
  __shared__ uint64_t sw[4];
  __shared__ float se[4];
  int seg = blockIdx.x, row = blockIdx.y, nseg = gridDim.x;
  const float* zr = z + (size_t)row * ldz;
  float m = -INFINITY;
  for (int k = 0; k < nseg; k++) m = fmaxf(m, segmax[(size_t)row * nseg + k]);
  uint64_t ws = 0;
  float es = 0.f;
  for (int i = 0; i < RL_SAMPLER_SEG / 256; i++) {
    int idx = seg * RL_SAMPLER_SEG + i * 256 + threadIdx.x;
    if (idx < V) {
      float e;
      uint64_t w;
      exp2_weight(zr[idx], m, c, e, w);
      ws += w;
      es = __fadd_rn(es, e);
    }
  }
  for (int o = 32; o > 0; o >>= 1) {
    ws += __shfl_xor(ws, o, 64);
    es = __fadd_rn(es, __shfl_xor(es, o, 64));
  }
  if ((threadIdx.x & 63) == 0) { sw[threadIdx.x >> 6] = ws; se[threadIdx.x >> 6] = es; }
  __syncthreads();
  if (threadIdx.x == 0) {
    segw[(size_t)row * nseg + seg] = sw[0] + sw[1] + sw[2] + sw[3];
    sege[(size_t)row * nseg + seg] = __fadd_rn(__fadd_rn(se[0], se[1]), __fadd_rn(se[2], se[3]));
  }
}

// grid rows, block 256
__global__ void sample_final_kernel(const float* __restrict__ z, size_t ldz, int V, float c,
                                    int greedy, int nseg, const float* __restrict__ segmax,
                                    const int32_t* __restrict__ segarg,
                                    const uint64_t* __restrict__ segw,
                                    const float* __restrict__ sege, const uint32_t* __restrict__ u32,
                                    uint64_t seed, const int32_t* __restrict__ row_traj,
                                    const int32_t* __restrict__ row_newpos,
                                    const int32_t* __restrict__ forced,
                                    const uint8_t* __restrict__ out_mask,
                                    int32_t* __restrict__ ids_out, float* __restrict__ logp_out) {
  __shared__ uint64_t tsum[256];
  __shared__ int chosen;
  int row = blockIdx.x, tid = threadIdx.x;
  const float* zr = z + (size_t)row * ldz;
  float m = -INFINITY;
  int arg = 0;
  uint64_t W = 0;
  float E = 0.f;
  for (int k = 0; k < nseg; k++) {
    float v = segmax[(size_t)row * nseg + k];
    if (v > m) { m = v; arg = segarg[(size_t)row * nseg + k]; }   // first segment wins ties
    W += segw[(size_t)row * nseg + k];
    E = __fadd_rn(E, sege[(size_t)row * nseg + k]);
  }
  int id;
  if (forced) {
    id = forced[row];
  } else if (greedy) {
    id = arg;
  } else {
    uint32_t u = u32 ? u32[row] : splitmix_u32(seed, row_traj[row], row_newpos[row]);
    uint64_t hi = __umul64hi(W, (uint64_t)u), lo = W * (uint64_t)u;
    uint64_t r = (hi << 32) | (lo >> 32);          // floor(u * W / 2^32) < W
    int s = 0;
    uint64_t pre = 0;
    for (; s < nseg - 1; s++) {
      uint64_t w = segw[(size_t)row * nseg + s];
      if (pre + w > r) break;
      pre += w;
    }
    uint64_t rl = r - pre;                         // target inside segment s
    const int PER = RL_SAMPLER_SEG / 256;          // 16 consecutive logits per thread
    int base = s * RL_SAMPLER_SEG + tid * PER;
    uint64_t wloc[PER];
    uint64_t mine = 0;
    for (int j = 0; j < PER; j++) {
      float e;
      uint64_t w = 0;
      if (base + j < V) exp2_weight(zr[base + j], m, c, e, w);
      wloc[j] = w;
      mine += w;
    }
    tsum[tid] = mine;
    if (tid == 0) chosen = -1;
    __syncthreads();
    uint64_t before = 0;
    for (int k = 0; k < tid; k++) before += tsum[k];
    if (before <= rl && rl < before + mine) {
      uint64_t acc = before;
      for (int j = 0; j < PER; j++) {
        acc += wloc[j];
        if (acc > rl) { chosen = base + j; break; }
      }
    }
    __syncthreads();
    id = chosen;
  }
  if (tid == 0) {
    float lp = 0.f;
    if (!(out_mask && out_mask[row])) {
      float t = __fmul_rn(__fsub_rn(zr[id], m), c);
      lp = t * 0.6931471805599453f - logf(E);
    }
    if (ids_out) ids_out[row] = id;
    logp_out[row] = lp;
  }
}

void launch_sampler(hipStream_t s, const float* logits, size_t ldz, int rows, int V, float scale_c,
                    int greedy, const uint32_t* u32, uint64_t seed, const int32_t* row_traj,
                    const int32_t* row_newpos, const int32_t* forced, const uint8_t* out_mask,
                    SamplerScratch sc, int32_t* ids_out, float* logp_out, const float* stripmax,
                    int nstrips) {
  if (rows <= 0) return;
  int nseg = sampler_nseg(V);
  dim3 grid(nseg, rows);
  if (greedy || nstrips <= 0) stripmax = nullptr;   // the arg-max needs the pass over the logits
  if (stripmax) row_max_kernel<<<rows, 256, 0, s>>>(stripmax, nstrips, nseg, sc.segmax, sc.segarg);
  else seg_max_kernel<<<grid, 256, 0, s>>>(logits, ldz, V, sc.segmax, sc.segarg);
  seg_weight_kernel<<<grid, 256, 0, s>>>(logits, ldz, V, scale_c, sc.segmax, sc.segw, sc.sege);
  sample_final_kernel<<<rows, 256, 0, s>>>(logits, ldz, V, scale_c, greedy, nseg, sc.segmax,
                                           sc.segarg, sc.segw, sc.sege, u32, seed, row_traj,
                                           row_newpos, forced, out_mask, ids_out, logp_out);
}

// ---------------------------------------------------------------------------------------------
// The sampler for callers that must not allocate device memory.  Its per-segment scratch lives in
// a fixed array in the library's device image; every GPU holds its own copy at its own address,
// looked up once per device.  Host code uses that address only, never the array's name.
// ---------------------------------------------------------------------------------------------
#define RL_NOALLOC_MAX_SEGMENTS 16384   // rows x ceil(vocab / RL_SAMPLER_SEG) of one call
#define RL_NOALLOC_SEG_BYTES 24         // max 4 + arg 4 + weight 8 + sum 4, padded to keep 8-byte alignment
static __device__ __align__(256) unsigned char scratch[(size_t)RL_NOALLOC_MAX_SEGMENTS * RL_NOALLOC_SEG_BYTES];

#define RL_MAX_DEVICES 64
static unsigned char* g_scratch_ptr[RL_MAX_DEVICES];   // per device: address of its copy of `scratch`

// Address of the current device's scratch array (looked up on first use), or null with *err set.
static unsigned char* noalloc_scratch(hipError_t* err) {
  int dev = 0;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= RL_MAX_DEVICES) { *err = hipErrorInvalidDevice; return nullptr; }
  if (!g_scratch_ptr[dev]) {
    unsigned char* p = nullptr;
    *err = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

int sampler_noalloc_prepare() {
  hipError_t e;
  return noalloc_scratch(&e) ? 0 : (int)e;
}

extern "C" int rl_sample_device_logits(const float* d_logits, int32_t rows, int32_t vocab,
                                       float temperature, const uint32_t* d_u32, int32_t* d_ids_out,
                                       float* d_logprobs_out, void* stream) {
  if (!d_logits || !d_u32 || !d_ids_out || !d_logprobs_out || rows <= 0 || vocab <= 0 ||
      !(temperature >= 0.0f))
    return rl_fail(RL_E_ARG, "bad argument");
  const int nseg = sampler_nseg(vocab);
  const size_t seg_n = (size_t)rows * nseg;
  if (seg_n > RL_NOALLOC_MAX_SEGMENTS)
    return rl_fail(RL_E_ARG, "rows x ceil(vocab / 4096) exceeds the 16384 segments of the fixed scratch");
  hipError_t e;
  unsigned char* base = noalloc_scratch(&e);
  if (!base) return rl_fail(RL_E_HIP, hipGetErrorString(e));
  // every entry the final kernel reads is written by the two segment kernels of this call first:
  // nothing has to start at zero
  SamplerScratch sc;
  sc.segw = (uint64_t*)base;
  sc.segmax = (float*)(sc.segw + seg_n);
  sc.segarg = (int32_t*)(sc.segmax + seg_n);
  sc.sege = (float*)(sc.segarg + seg_n);
  const bool greedy = temperature == 0.0f;
  const float c = (float)(1.4426950408889634 / (greedy ? 1.0 : (double)temperature));
  launch_sampler((hipStream_t)stream, d_logits, (size_t)vocab, rows, vocab, c, greedy ? 1 : 0, d_u32, 0,
                 nullptr, nullptr, nullptr, nullptr, sc, d_ids_out, d_logprobs_out);
  e = hipGetLastError();
  if (e != hipSuccess) return rl_fail(RL_E_HIP, hipGetErrorString(e));
  return RL_OK;
}
