// Shape-generic kernels: fp32 mode, and bf16 models whose shape the MFMA kernels do not cover.
// One decoder block of the policy pi_theta(a | s_t) (paper Section 2.2) is
//   h += W_o attn(rope(norm(W_q a)), rope(norm(W_k a)), W_v a),  a = rmsnorm(h)
//   h += W_down (silu(W_gate b) * W_up b),                       b = rmsnorm(h)
// Each kernel below is one of those pieces; accumulation is always fp32.
#include "kernels.h"

template <typename TW>
__global__ void embed_kernel(const TW* __restrict__ E, const int32_t* __restrict__ tok,
                             float* __restrict__ h, int H) {
  int row = blockIdx.x;
  const TW* e = E + (size_t)tok[row] * H;
  for (int j = threadIdx.x; j < H; j += blockDim.x) h[(size_t)row * H + j] = ldf(e + j);
}

template <typename TW, typename TA, bool ATILE>
__global__ void rmsnorm_kernel(const float* __restrict__ h, const TW* __restrict__ g,
                               TA* __restrict__ out, int H, float eps) {
  __shared__ float red[4];
  int row = blockIdx.x;
  const float* x = h + (size_t)row * H;
  float ss = 0.f;
  for (int j = threadIdx.x; j < H; j += 256) ss += x[j] * x[j];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = red[0] + red[1] + red[2] + red[3];
  float inv = 1.0f / sqrtf(tot / (float)H + eps);
  if (ATILE) {
    // 8 consecutive k share one 16-byte lane slot of the A-tile layout (H % 16 == 0)
    for (int j = threadIdx.x * 8; j < H; j += 256 * 8) {
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 4; e++) {
        float y0 = x[j + 2 * e] * inv * ldf(g + j + 2 * e);
        float y1 = x[j + 2 * e + 1] * inv * ldf(g + j + 2 * e + 1);
        w[e] = (uint32_t)f2bf(y0) | ((uint32_t)f2bf(y1) << 16);
      }
      *(uint4*)((bf16_t*)out + atile_off(row, j, H)) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  } else {
    for (int j = threadIdx.x; j < H; j += 256) stf(out + (size_t)row * H + j, x[j] * inv * ldf(g + j));
  }
}

// grid M, block 256: h[row] += sum_p parts[p][row]; out = rmsnorm(h[row]) * g, A-tile layout
__global__ void add_rmsnorm_kernel(float* __restrict__ h, const float* __restrict__ parts, int n_part,
                                   size_t part_stride, const bf16_t* __restrict__ g,
                                   bf16_t* __restrict__ out, int H, float eps,
                                   const int32_t* __restrict__ rows) {
  __shared__ float red[4];
  const int orow = blockIdx.x;
  const int row = rows ? rows[orow] : orow;
  float* x = h + (size_t)row * H;
  const float* pr = parts + (size_t)row * H;
  float ss = 0.f;
  for (int j = threadIdx.x * 4; j < H; j += 1024) {
    float4 v = *(const float4*)(x + j);
    int p = 0;
    for (; p + 4 <= n_part; p += 4) {     // four independent loads in flight, added in order
      float4 u0 = *(const float4*)(pr + (size_t)p * part_stride + j);
      float4 u1 = *(const float4*)(pr + (size_t)(p + 1) * part_stride + j);
      float4 u2 = *(const float4*)(pr + (size_t)(p + 2) * part_stride + j);
      float4 u3 = *(const float4*)(pr + (size_t)(p + 3) * part_stride + j);
      v.x = (((v.x + u0.x) + u1.x) + u2.x) + u3.x;
      v.y = (((v.y + u0.y) + u1.y) + u2.y) + u3.y;
      v.z = (((v.z + u0.z) + u1.z) + u2.z) + u3.z;
      v.w = (((v.w + u0.w) + u1.w) + u2.w) + u3.w;
    }
    for (; p < n_part; p++) {
      float4 u = *(const float4*)(pr + (size_t)p * part_stride + j);
      v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
    }
    if (n_part > 0) *(float4*)(x + j) = v;
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();   // also makes every thread's updated h visible to the block
  float inv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)H + eps);
  for (int j = threadIdx.x * 8; j < H; j += 2048) {
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; e++) {
      float y0 = x[j + 2 * e] * inv * bf2f(g[j + 2 * e]);
      float y1 = x[j + 2 * e + 1] * inv * bf2f(g[j + 2 * e + 1]);
      w[e] = (uint32_t)f2bf(y0) | ((uint32_t)f2bf(y1) << 16);
    }
    *(uint4*)(out + atile_off(orow, j, H)) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// Same operation with the whole row in registers: every load of the row and of its (up to 8)
// partial sums is issued before the first use, so a row costs about one memory round trip instead
// of one per group of partials; the normalised row is written from registers.  H <= ITER * 1024.
template <int ITER>
__global__ __launch_bounds__(256) void add_rmsnorm_reg_kernel(
    float* __restrict__ h, const float* __restrict__ parts, int n_part, size_t part_stride,
    const bf16_t* __restrict__ g, bf16_t* __restrict__ out, int H, float eps,
    const int32_t* __restrict__ rows) {
  __shared__ float red[4];
  const int orow = blockIdx.x;
  const int row = rows ? rows[orow] : orow;
  float* x = h + (size_t)row * H;
  const float* pr = parts + (size_t)row * H;
  float4 v[ITER], u[ITER][8];
  uint2 gw[ITER];
#pragma unroll
  for (int it = 0; it < ITER; it++) {
    const int j = threadIdx.x * 4 + it * 1024;
    const bool ok = j < H;
    v[it] = ok ? *(const float4*)(x + j) : make_float4(0.f, 0.f, 0.f, 0.f);
    gw[it] = ok ? *(const uint2*)(g + j) : make_uint2(0u, 0u);
#pragma unroll
    for (int p = 0; p < 8; p++)
      u[it][p] = (ok && p < n_part) ? *(const float4*)(pr + (size_t)p * part_stride + j)
                                    : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < ITER; it++) {
#pragma unroll
    for (int p = 0; p < 8; p++)
      if (p < n_part) {   // ascending order, as the looping kernel adds them
        v[it].x += u[it][p].x; v[it].y += u[it][p].y; v[it].z += u[it][p].z; v[it].w += u[it][p].w;
      }
    const int j = threadIdx.x * 4 + it * 1024;
    if (n_part > 0 && j < H) *(float4*)(x + j) = v[it];
    ss += v[it].x * v[it].x + v[it].y * v[it].y + v[it].z * v[it].z + v[it].w * v[it].w;
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float inv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)H + eps);
#pragma unroll
  for (int it = 0; it < ITER; it++) {
    const int j = threadIdx.x * 4 + it * 1024;
    if (j < H) {
      float y0 = v[it].x * inv * bf2f((bf16_t)(gw[it].x & 0xffff));
      float y1 = v[it].y * inv * bf2f((bf16_t)(gw[it].x >> 16));
      float y2 = v[it].z * inv * bf2f((bf16_t)(gw[it].y & 0xffff));
      float y3 = v[it].w * inv * bf2f((bf16_t)(gw[it].y >> 16));
      uint2 w;
      w.x = (uint32_t)f2bf(y0) | ((uint32_t)f2bf(y1) << 16);
      w.y = (uint32_t)f2bf(y2) | ((uint32_t)f2bf(y3) << 16);
      *(uint2*)(out + atile_off(orow, j, H)) = w;   // 4 consecutive k share one 16-byte lane slot
    }
  }
}

void launch_add_rmsnorm(hipStream_t s, float* h, const float* parts, int n_part, size_t part_stride,
                        const bf16_t* g, bf16_t* out, int M, int H, float eps, const int32_t* rows) {
  if (M <= 0) return;
  if (n_part <= 8 && H % 4 == 0 && H <= 4096) {
    if (H <= 1024) add_rmsnorm_reg_kernel<1><<<M, 256, 0, s>>>(h, parts, n_part, part_stride, g, out, H, eps, rows);
    else if (H <= 2048) add_rmsnorm_reg_kernel<2><<<M, 256, 0, s>>>(h, parts, n_part, part_stride, g, out, H, eps, rows);
    else if (H <= 3072) add_rmsnorm_reg_kernel<3><<<M, 256, 0, s>>>(h, parts, n_part, part_stride, g, out, H, eps, rows);
    else add_rmsnorm_reg_kernel<4><<<M, 256, 0, s>>>(h, parts, n_part, part_stride, g, out, H, eps, rows);
    return;
  }
  add_rmsnorm_kernel<<<M, 256, 0, s>>>(h, parts, n_part, part_stride, g, out, H, eps, rows);
}

template <typename TA, typename TW>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const TA* __restrict__ A,
                                                           const TW* __restrict__ W,
                                                           float* __restrict__ C, int M, int N,
                                                           int K, int accumulate) {
  __shared__ float As[16][65];
  __shared__ float Ws[16][65];
  int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      int e = tid + i * 256, r = e >> 4, kk = e & 15;
      int gm = m0 + r, gn = n0 + r, gk = k0 + kk;
      As[kk][r] = (gm < M && gk < K) ? ldf(A + (size_t)gm * K + gk) : 0.f;
      Ws[kk][r] = (gn < N && gk < K) ? ldf(W + (size_t)gn * K + gk) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; kk++) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; i++) { a[i] = As[kk][ty * 4 + i]; b[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) {
      int gm = m0 + ty * 4 + i, gn = n0 + tx * 4 + j;
      if (gm < M && gn < N) {
        float* c = C + (size_t)gm * N + gn;
        *c = accumulate ? *c + acc[i][j] : acc[i][j];
      }
    }
}

// grid (M, nq + 2 nkv), block 64
template <typename TW, typename TA, typename TKV, bool SWZ>
__global__ void qkrope_kernel(const float* __restrict__ qkv, int n_part, size_t part_stride,
                              const TW* __restrict__ gq,
                              const TW* __restrict__ gk, const float* __restrict__ rope_cs,
                              const int32_t* __restrict__ row_pos,
                              const int32_t* __restrict__ row_slot,
                              const int32_t* __restrict__ page_table, TA* __restrict__ qout,
                              TKV* __restrict__ kpool, TKV* __restrict__ vpool, int nq, int nkv,
                              int d, float eps, int qk_norm, int pt_stride) {
  int row = blockIdx.x, hd = blockIdx.y, half = d >> 1;
  int pos = row_pos[row];
  const float* x = qkv + (size_t)row * (nq + 2 * nkv) * d + (size_t)hd * d;
  bool is_q = hd < nq, is_v = hd >= nq + nkv;
  float x1[2], x2[2];
  float ss = 0.f;
  int cnt = 0;
  for (int i = threadIdx.x; i < half; i += 64, cnt++) {
    float u = x[i], w = x[i + half];
    for (int p = 1; p < n_part; p++) { u += x[p * part_stride + i]; w += x[p * part_stride + i + half]; }
    x1[cnt] = u;
    x2[cnt] = w;
    ss += u * u + w * w;
  }
  ss = wave_sum(ss);
  float inv = (qk_norm && !is_v) ? 1.0f / sqrtf(ss / (float)d + eps) : 1.0f;
  TKV* blk = nullptr;
  int tok = pos & (RL_PAGE - 1);
  if (!is_q) {
    int page = page_table[(size_t)row_slot[row] * pt_stride + (pos >> 4)];
    int kvh = is_v ? hd - nq - nkv : hd - nq;
    blk = (is_v ? vpool : kpool) + ((size_t)page * nkv + kvh) * (RL_PAGE * d);
  }
  const TW* g = is_q ? gq : gk;
  cnt = 0;
  for (int i = threadIdx.x; i < half; i += 64, cnt++) {
    float a = x1[cnt], b = x2[cnt];
    if (is_v) {
      stf(blk + vblk_off<SWZ>(tok, i, d), a);
      stf(blk + vblk_off<SWZ>(tok, i + half, d), b);
      continue;
    }
    if (qk_norm) { a = a * inv * ldf(g + i); b = b * inv * ldf(g + i + half); }
    float c = rope_cs[((size_t)pos * half + i) * 2], s = rope_cs[((size_t)pos * half + i) * 2 + 1];
    float y1 = a * c - b * s, y2 = b * c + a * s;
    if (is_q) {
      stf(qout + (size_t)row * nq * d + (size_t)hd * d + i, y1);
      stf(qout + (size_t)row * nq * d + (size_t)hd * d + i + half, y2);
    } else {
      stf(blk + kblk_off<SWZ>(tok, i, d), y1);
      stf(blk + kblk_off<SWZ>(tok, i + half, d), y2);
    }
  }
}

// grid (M, nq), block 64: one wave per (row, q head); tokens in blocks of 64, online softmax
template <typename TA, typename TKV, bool SWZ, bool OATILE>
__global__ void attention_generic_kernel(const TA* __restrict__ q, const TKV* __restrict__ kpool,
                                         const TKV* __restrict__ vpool,
                                         const int32_t* __restrict__ row_pos,
                                         const int32_t* __restrict__ row_slot,
                                         const int32_t* __restrict__ page_table,
                                         TA* __restrict__ o, int nq, int nkv, int d,
                                         int pt_stride) {
  __shared__ float qs[128];
  __shared__ float ps[64];
  int row = blockIdx.x, qh = blockIdx.y, kvh = qh / (nq / nkv);
  int pos = row_pos[row];
  const int32_t* pt = page_table + (size_t)row_slot[row] * pt_stride;
  for (int e = threadIdx.x; e < d; e += 64) qs[e] = ldf(q + (size_t)row * nq * d + (size_t)qh * d + e);
  __syncthreads();
  float scale = 1.0f / sqrtf((float)d);
  float m = -INFINITY, l = 0.f, acc[2] = {0.f, 0.f};
  for (int t0 = 0; t0 <= pos; t0 += 64) {
    int t = t0 + threadIdx.x;
    float sc = -INFINITY;
    if (t <= pos) {
      const TKV* kb = kpool + ((size_t)pt[t >> 4] * nkv + kvh) * (RL_PAGE * d);
      float dot = 0.f;
      for (int e = 0; e < d; e++) dot += qs[e] * ldf(kb + kblk_off<SWZ>(t & 15, e, d));
      sc = dot * scale;
    }
    float mn = fmaxf(m, wave_max(sc));
    float p = (t <= pos) ? expf(sc - mn) : 0.f;
    float alpha = expf(m - mn);       // m = -inf on the first block: exp(-inf) = 0
    l = l * alpha + wave_sum(p);
    m = mn;
    __syncthreads();
    ps[threadIdx.x] = p;
    __syncthreads();
    int nt = min(64, pos + 1 - t0);
    int c = 0;
    for (int e = threadIdx.x; e < d; e += 64, c++) {
      float a = acc[c] * alpha;
      for (int j = 0; j < nt; j++) {
        int tt = t0 + j;
        const TKV* vb = vpool + ((size_t)pt[tt >> 4] * nkv + kvh) * (RL_PAGE * d);
        a += ps[j] * ldf(vb + vblk_off<SWZ>(tt & 15, e, d));
      }
      acc[c] = a;
    }
  }
  int c = 0;
  for (int e = threadIdx.x; e < d; e += 64, c++) {
    float y = acc[c] / l;
    if (OATILE) stf(o + atile_off(row, qh * d + e, nq * d), y);
    else stf(o + (size_t)row * nq * d + (size_t)qh * d + e, y);
  }
}

template <typename TA, bool ATILE>
__global__ void swiglu_kernel(const float* __restrict__ gu, TA* __restrict__ m, int I) {
  int row = blockIdx.y;
  int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= I) return;
  float g = gu[(size_t)row * 2 * I + j], u = gu[(size_t)row * 2 * I + I + j];
  float y = g / (1.0f + expf(-g)) * u;
  if (ATILE) stf(m + atile_off(row, j, I), y);
  else stf(m + (size_t)row * I + j, y);
}

__global__ void copy_pages_kernel(char* __restrict__ k, char* __restrict__ v,
                                  const int32_t* __restrict__ pairs, size_t page_bytes) {
  int p = blockIdx.x;
  size_t src = (size_t)pairs[2 * p] * page_bytes, dst = (size_t)pairs[2 * p + 1] * page_bytes;
  char* base = blockIdx.y ? v : k;
  const uint4* s4 = (const uint4*)(base + src);
  uint4* d4 = (uint4*)(base + dst);
  for (size_t i = threadIdx.x; i < page_bytes / 16; i += blockDim.x) d4[i] = s4[i];
}

__global__ void page_table_update_kernel(int32_t* __restrict__ pt, const int32_t* __restrict__ upd,
                                         int n, int stride) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) pt[(size_t)upd[3 * i] * stride + upd[3 * i + 1]] = upd[3 * i + 2];
}

// ---- launchers ---------------------------------------------------------------------------
template <typename TW>
void launch_embed(hipStream_t s, const TW* E, const int32_t* tok, float* h, int M, int H) {
  if (M > 0) embed_kernel<TW><<<M, 256, 0, s>>>(E, tok, h, H);
}
template void launch_embed<float>(hipStream_t, const float*, const int32_t*, float*, int, int);
template void launch_embed<bf16_t>(hipStream_t, const bf16_t*, const int32_t*, float*, int, int);

template <typename TW, typename TA>
void launch_rmsnorm(hipStream_t s, const float* h, const TW* g, TA* out, int M, int H, float eps,
                    bool atile) {
  if (M <= 0) return;
  if (atile) rmsnorm_kernel<TW, TA, true><<<M, 256, 0, s>>>(h, g, out, H, eps);
  else rmsnorm_kernel<TW, TA, false><<<M, 256, 0, s>>>(h, g, out, H, eps);
}
template void launch_rmsnorm<float, float>(hipStream_t, const float*, const float*, float*, int, int, float, bool);
template void launch_rmsnorm<bf16_t, bf16_t>(hipStream_t, const float*, const bf16_t*, bf16_t*, int, int, float, bool);

template <typename TA, typename TW>
void launch_gemm_generic(hipStream_t s, const TA* A, const TW* W, float* C, int M, int N, int K,
                         bool accumulate) {
  if (M <= 0) return;
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  gemm_generic_kernel<TA, TW><<<grid, 256, 0, s>>>(A, W, C, M, N, K, accumulate ? 1 : 0);
}
template void launch_gemm_generic<float, float>(hipStream_t, const float*, const float*, float*, int, int, int, bool);
template void launch_gemm_generic<bf16_t, bf16_t>(hipStream_t, const bf16_t*, const bf16_t*, float*, int, int, int, bool);

// head_dim 128, bf16, MFMA cache layout: grid (M, ceil(heads / 16)), block 256.  Sixteen lanes
// own one head: lane `sub` holds dims 4 sub .. 4 sub + 3 and their rotate-half partners 64 + ...,
// so partial sums arrive as 16-byte loads (all issued before the first add) and q, k leave as
// 8-byte stores.  FP8: keys and values go from fp32 straight to E4M3 codes (8-bit cache layout).
template <bool FP8>
__global__ __launch_bounds__(256) void qkrope128_kernel(
    const float* __restrict__ qkv, int n_part, size_t part_stride, const bf16_t* __restrict__ gq,
    const bf16_t* __restrict__ gk, const float* __restrict__ rope_cs,
    const int32_t* __restrict__ row_pos, const int32_t* __restrict__ row_slot,
    const int32_t* __restrict__ page_table, bf16_t* __restrict__ qout, bf16_t* __restrict__ kpool,
    bf16_t* __restrict__ vpool, int nq, int nkv, float eps, int qk_norm, int pt_stride) {
  const int row = blockIdx.x, sub = threadIdx.x & 15;
  const int hd = blockIdx.y * 16 + (threadIdx.x >> 4), NH = nq + 2 * nkv;
  if (hd >= NH) return;          // whole 16-lane groups leave together; no barrier below
  const int pos = row_pos[row];
  const float* x = qkv + ((size_t)row * NH + hd) * 128 + sub * 4;
  float4 lo[8], hi[8];
#pragma unroll
  for (int p = 0; p < 8; p++) {
    lo[p] = p < n_part ? *(const float4*)(x + (size_t)p * part_stride) : make_float4(0.f, 0.f, 0.f, 0.f);
    hi[p] = p < n_part ? *(const float4*)(x + (size_t)p * part_stride + 64) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  const bool is_q = hd < nq, is_v = hd >= nq + nkv;
  const bf16_t* g = is_q ? gq : gk;
  const uint2 glo = *(const uint2*)(g + sub * 4), ghi = *(const uint2*)(g + 64 + sub * 4);
  const float* cs = rope_cs + ((size_t)pos * 64 + sub * 4) * 2;     // (cos, sin) pairs of 4 dims
  const float4 cs0 = *(const float4*)cs, cs1 = *(const float4*)(cs + 4);
  float a[4] = {lo[0].x, lo[0].y, lo[0].z, lo[0].w}, b[4] = {hi[0].x, hi[0].y, hi[0].z, hi[0].w};
#pragma unroll
  for (int p = 1; p < 8; p++)
    if (p < n_part) {
      a[0] += lo[p].x; a[1] += lo[p].y; a[2] += lo[p].z; a[3] += lo[p].w;
      b[0] += hi[p].x; b[1] += hi[p].y; b[2] += hi[p].z; b[3] += hi[p].w;
    }
  float ss = 0.f;
#pragma unroll
  for (int e = 0; e < 4; e++) ss += a[e] * a[e] + b[e] * b[e];
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 16);
  bf16_t* blk = nullptr;
  const int tok = pos & (RL_PAGE - 1);
  int page_id = 0, kvh_id = 0;
  if (!is_q) {
    page_id = page_table[(size_t)row_slot[row] * pt_stride + (pos >> 4)];
    kvh_id = is_v ? hd - nq - nkv : hd - nq;
    blk = (is_v ? vpool : kpool) + ((size_t)page_id * nkv + kvh_id) * (RL_PAGE * 128);
  }
  if (is_v) {
    if constexpr (FP8) {
      uint8_t* blk8 = (uint8_t*)(is_v ? vpool : kpool) + ((size_t)page_id * nkv + kvh_id) * (RL_PAGE * 128);
#pragma unroll
      for (int e = 0; e < 4; e++) {
        blk8[vswz8_off(tok, sub * 4 + e)] = f2e4m3(a[e]);
        blk8[vswz8_off(tok, 64 + sub * 4 + e)] = f2e4m3(b[e]);
      }
      return;
    }
#pragma unroll
    for (int e = 0; e < 4; e++) {
      blk[vswz_off(tok, sub * 4 + e)] = f2bf(a[e]);
      blk[vswz_off(tok, 64 + sub * 4 + e)] = f2bf(b[e]);
    }
    return;
  }
  if (qk_norm) {
    const float inv = 1.0f / sqrtf(ss / 128.0f + eps);
    const float gl[4] = {bf2f((bf16_t)(glo.x & 0xffff)), bf2f((bf16_t)(glo.x >> 16)),
                         bf2f((bf16_t)(glo.y & 0xffff)), bf2f((bf16_t)(glo.y >> 16))};
    const float gh[4] = {bf2f((bf16_t)(ghi.x & 0xffff)), bf2f((bf16_t)(ghi.x >> 16)),
                         bf2f((bf16_t)(ghi.y & 0xffff)), bf2f((bf16_t)(ghi.y >> 16))};
#pragma unroll
    for (int e = 0; e < 4; e++) { a[e] = a[e] * inv * gl[e]; b[e] = b[e] * inv * gh[e]; }
  }
  const float c[4] = {cs0.x, cs0.z, cs1.x, cs1.z}, sn[4] = {cs0.y, cs0.w, cs1.y, cs1.w};
  if constexpr (FP8) {
    if (!is_q) {   // 4 consecutive dims = 4 consecutive bytes of one lane slot
      uint8_t* blk8 = (uint8_t*)kpool + ((size_t)page_id * nkv + kvh_id) * (RL_PAGE * 128);
      float r1[4], r2[4];
#pragma unroll
      for (int e = 0; e < 4; e++) {
        r1[e] = a[e] * c[e] - b[e] * sn[e];
        r2[e] = b[e] * c[e] + a[e] * sn[e];
      }
      *(uint32_t*)(blk8 + kswz8_off(tok, sub * 4)) = f2e4m3x4(r1[0], r1[1], r1[2], r1[3]);
      *(uint32_t*)(blk8 + kswz8_off(tok, 64 + sub * 4)) = f2e4m3x4(r2[0], r2[1], r2[2], r2[3]);
      return;
    }
  }
  uint32_t y1[4], y2[4];
#pragma unroll
  for (int e = 0; e < 4; e++) {
    y1[e] = f2bf(a[e] * c[e] - b[e] * sn[e]);
    y2[e] = f2bf(b[e] * c[e] + a[e] * sn[e]);
  }
  const uint2 w1 = make_uint2(y1[0] | (y1[1] << 16), y1[2] | (y1[3] << 16));
  const uint2 w2 = make_uint2(y2[0] | (y2[1] << 16), y2[2] | (y2[3] << 16));
  if (is_q) {
    bf16_t* dst = qout + ((size_t)row * nq + hd) * 128 + sub * 4;
    *(uint2*)dst = w1;
    *(uint2*)(dst + 64) = w2;
  } else {   // 4 consecutive dims lie in one 8-element lane slot of the swizzled key block
    *(uint2*)(blk + kswz_off(tok, sub * 4)) = w1;
    *(uint2*)(blk + kswz_off(tok, 64 + sub * 4)) = w2;
  }
}

template <typename TW, typename TA, typename TKV, bool SWZ>
void launch_qkrope(hipStream_t s, const float* qkv, int n_part, size_t part_stride, const TW* gq,
                   const TW* gk, const float* rope_cs, const int32_t* row_pos,
                   const int32_t* row_slot, const int32_t* page_table, TA* qout, KvPool pool,
                   const ModelDims& md, int M) {
  if (M <= 0) return;
  if constexpr (SWZ) {
    if (md.d == 128 && n_part <= 8) {
      dim3 grid128(M, (md.nq + 2 * md.nkv + 15) / 16);
      if (md.kv_fp8)
        qkrope128_kernel<true><<<grid128, 256, 0, s>>>(qkv, n_part, part_stride, gq, gk, rope_cs, row_pos,
                                                       row_slot, page_table, qout, (bf16_t*)pool.k,
                                                       (bf16_t*)pool.v, md.nq, md.nkv, md.eps, md.qk_norm,
                                                       md.max_pages_per_traj);
      else
        qkrope128_kernel<false><<<grid128, 256, 0, s>>>(qkv, n_part, part_stride, gq, gk, rope_cs, row_pos,
                                                        row_slot, page_table, qout, (bf16_t*)pool.k,
                                                        (bf16_t*)pool.v, md.nq, md.nkv, md.eps, md.qk_norm,
                                                        md.max_pages_per_traj);
      return;
    }
  }
  dim3 grid(M, md.nq + 2 * md.nkv);
  qkrope_kernel<TW, TA, TKV, SWZ><<<grid, 64, 0, s>>>(
      qkv, n_part, part_stride, gq, gk, rope_cs, row_pos, row_slot, page_table, qout, (TKV*)pool.k,
      (TKV*)pool.v, md.nq, md.nkv, md.d, md.eps, md.qk_norm, md.max_pages_per_traj);
}
template void launch_qkrope<float, float, float, false>(hipStream_t, const float*, int, size_t, const float*, const float*, const float*, const int32_t*, const int32_t*, const int32_t*, float*, KvPool, const ModelDims&, int);
template void launch_qkrope<bf16_t, bf16_t, bf16_t, false>(hipStream_t, const float*, int, size_t, const bf16_t*, const bf16_t*, const float*, const int32_t*, const int32_t*, const int32_t*, bf16_t*, KvPool, const ModelDims&, int);
template void launch_qkrope<bf16_t, bf16_t, bf16_t, true>(hipStream_t, const float*, int, size_t, const bf16_t*, const bf16_t*, const float*, const int32_t*, const int32_t*, const int32_t*, bf16_t*, KvPool, const ModelDims&, int);

template <typename TA, typename TKV, bool SWZ>
void launch_attention_generic(hipStream_t s, const TA* q, KvPool pool, const int32_t* row_pos,
                              const int32_t* row_slot, const int32_t* page_table, TA* o,
                              const ModelDims& md, int M, bool o_atile) {
  if (M <= 0) return;
  dim3 grid(M, md.nq);
  if (o_atile)
    attention_generic_kernel<TA, TKV, SWZ, true><<<grid, 64, 0, s>>>(
        q, (const TKV*)pool.k, (const TKV*)pool.v, row_pos, row_slot, page_table, o, md.nq, md.nkv,
        md.d, md.max_pages_per_traj);
  else
    attention_generic_kernel<TA, TKV, SWZ, false><<<grid, 64, 0, s>>>(
        q, (const TKV*)pool.k, (const TKV*)pool.v, row_pos, row_slot, page_table, o, md.nq, md.nkv,
        md.d, md.max_pages_per_traj);
}
template void launch_attention_generic<float, float, false>(hipStream_t, const float*, KvPool, const int32_t*, const int32_t*, const int32_t*, float*, const ModelDims&, int, bool);
template void launch_attention_generic<bf16_t, bf16_t, false>(hipStream_t, const bf16_t*, KvPool, const int32_t*, const int32_t*, const int32_t*, bf16_t*, const ModelDims&, int, bool);
template void launch_attention_generic<bf16_t, bf16_t, true>(hipStream_t, const bf16_t*, KvPool, const int32_t*, const int32_t*, const int32_t*, bf16_t*, const ModelDims&, int, bool);

template <typename TA>
void launch_swiglu(hipStream_t s, const float* gu, TA* m, int M, int I, bool atile) {
  if (M <= 0) return;
  dim3 grid((I + 255) / 256, M);
  if (atile) swiglu_kernel<TA, true><<<grid, 256, 0, s>>>(gu, m, I);
  else swiglu_kernel<TA, false><<<grid, 256, 0, s>>>(gu, m, I);
}
template void launch_swiglu<float>(hipStream_t, const float*, float*, int, int, bool);
template void launch_swiglu<bf16_t>(hipStream_t, const float*, bf16_t*, int, int, bool);

void launch_copy_pages(hipStream_t s, KvPool pool, const int32_t* pairs, int n_pairs,
                       size_t page_bytes) {
  if (n_pairs <= 0) return;
  copy_pages_kernel<<<dim3(n_pairs, 2), 256, 0, s>>>((char*)pool.k, (char*)pool.v, pairs, page_bytes);
}
void launch_page_table_update(hipStream_t s, int32_t* page_table, const int32_t* upd, int n,
                              int stride) {
  if (n <= 0) return;
  page_table_update_kernel<<<(n + 255) / 256, 256, 0, s>>>(page_table, upd, n, stride);
}
