// bf16 MFMA kernels for gfx950: weight-streaming GEMM, weight repack, paged GQA attention.
// They implement the same decoder pieces as the generic kernels (policy forward of the paper's
// Generate / Update steps, Section 2.3.2) for head_dim 128 and tile-aligned widths.
#include "kernels.h"

// =============================================================================================
// Weight repack: W[N,K] row-major -> [K/64 chunks][N/32 strips][4 k-blocks][64 lanes][8].  One
// (chunk, strip) cell is 4 KB: four 32x32x16 MFMA column operands in lane order
// (lane = n % 32 + 32 * ((k % 16) / 8), 8 consecutive k per lane).  Chunk-major order makes all
// workgroups that advance through K in step sweep HBM contiguously; a strip-major order puts
// every wave's stream at a multiple of K * 64 bytes and piles them onto a few memory channels.
// =============================================================================================
__global__ void repack_weight_kernel(const bf16_t* __restrict__ W, const bf16_t* __restrict__ Wu,
                                     bf16_t* __restrict__ Wp, int N, int K, int interleave16) {
  size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int NB = N / 32;
  size_t total = (size_t)NB * (K / 16) * 64;
  if (t >= total) return;
  int lane = (int)(t & 63);
  size_t blk = t >> 6;                 // ((chunk * NB + strip) * 4 + k-block in chunk)
  int kb4 = (int)(blk & 3);
  size_t cell = blk >> 2;
  int nb = (int)(cell % NB);
  int chunk = (int)(cell / NB);
  int n = nb * 32 + (lane & 31);
  int k = chunk * 64 + kb4 * 16 + (lane >> 5) * 8;
  const bf16_t* src;
  if (interleave16) {
    int grp = n >> 4;                       // even groups: gate rows, odd groups: up rows
    int srow = (grp >> 1) * 16 + (n & 15);
    src = ((grp & 1) ? Wu : W) + (size_t)srow * K + k;
  } else {
    src = W + (size_t)n * K + k;
  }
  *(uint4*)(Wp + t * 8) = *(const uint4*)src;
}

void launch_repack_weight(hipStream_t s, const bf16_t* W, const bf16_t* Wu, bf16_t* Wp, int N,
                          int K, bool interleave16) {
  size_t total = (size_t)(N / 32) * (K / 16) * 64;
  repack_weight_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(W, Wu, Wp, N, K,
                                                                        interleave16 ? 1 : 0);
}

// =============================================================================================
// GEMM  C[M,N] = A[M,K] * W[N,K]^T for weight streaming.  Workgroup = NW waves (2 or 4), tile
// 128 rows x 32*NW columns; wave w owns the 32-column strip NW*blockIdx.x + w for all 128 rows
// (4 accumulators of 32x32).  Per 64-k chunk the A tile (16 KB, already in operand order in HBM)
// is copied to LDS and shared by the waves; each wave streams its own weight cells straight from
// HBM into registers, D chunks ahead.  blockIdx.z selects a K-slice (split-K); every slice
// stores its own fp32 partial sum, which the consumer kernel adds in a fixed order (no atomics:
// results are bit-reproducible).
// MB = number of 32-row blocks of the tile that can hold rows (1, 2 or 4; the launcher picks the
// smallest that covers M when there is one row tile): only those blocks of the A chunk are
// fetched, staged and multiplied.  At decode sizes a workgroup's time follows the bytes its CU
// fetches, and the A chunk is half of them, so small batches gain most of what they leave out
// (rows <= 32: gate-up 30.7 -> 23.6 us, down 18.3 -> 13.0 us); results per row are unchanged.
// EPI_LSE (lm-head of the masked log-prob pass): the product is formed transposed (weights as the
// MFMA row operand; both operands have the same lane layout, so swapping them costs nothing), which
// puts 16 vocabulary entries of one batch row into the registers of a lane.  The epilogue reduces
// its 32-column strip per row to (max, sum of 2^((z - max) c)) and picks out the target token's
// logit; the logits themselves are never stored.
// EPI_STORE_MAX (lm-head of a decode step): EPI_STORE plus, per row, the maximum over the wave's 32
// columns (a butterfly over the 32 lanes of each half that halves the values a lane holds at every
// step), written to zt[row * (N / 32) + strip]: the sampler gets the row maximum it needs before
// any weight can be formed from V / 32 numbers per row instead of a pass over the logits.
// =============================================================================================
template <int EPI, int D, int NW, int MB>
__global__ __launch_bounds__(64 * NW) void gemm_mfma_kernel(const bf16_t* __restrict__ A,
                                                            const bf16_t* __restrict__ Wp,
                                                            void* __restrict__ Cv, int M, int N,
                                                            int K, int chunks_per_split,
                                                            const int32_t* __restrict__ tgt,
                                                            float* __restrict__ zt, float scale_c) {
  constexpr int NT = 64 * NW;        // threads
  constexpr int APT = 256 * MB / NT; // 16-byte pieces of the used part of an A chunk per thread
  __shared__ u32x4 As[2][1024];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nb = blockIdx.x * NW + wave;
  const bool active = nb * 32 < N;
  const int mt = blockIdx.y;
  const int nchunks = K >> 6;
  const int c0 = blockIdx.z * chunks_per_split;
  const int c1 = min(c0 + chunks_per_split, nchunks);
  const u32x4* Ag = (const u32x4*)(A + (size_t)mt * K * 128);       // tile: 128 rows x K
  // piece p of the used part of a chunk -> its offset in the chunk (k-block, row block, lane):
  // with MB < 4 only the first MB row blocks of every k-block are staged
  auto a_piece = [](int p) { return MB == 4 ? p : (p / (64 * MB)) * 256 + (p % (64 * MB)); };
  const int NB = N >> 5;
  const u32x4* Wg = (const u32x4*)Wp + (size_t)(active ? nb : 0) * 256;   // cell (chunk 0, strip nb)
  f32x16 acc[MB];
#pragma unroll
  for (int i = 0; i < MB; i++)
#pragma unroll
    for (int j = 0; j < 16; j++) acc[i][j] = 0.f;
  // D chunks of A (for the whole workgroup) and of this wave's weight strip are kept in flight.
  // Loads past the end of the K-slice are clamped to its last chunk (re-reads that hit in L2) so
  // that the pipeline has no conditional register definitions.  Stages are spelled out (no
  // arrays of stages) so that every buffer lives in registers.
  const int clast = c1 - 1;
  u32x4 a0[APT], a1[APT], a2[APT], a3[APT], b0[4], b1[4], b2[4], b3[4];
#define GEMM_LOAD(AR, BR, CHUNK)                                            \
  {                                                                         \
    const int cl_ = min((CHUNK), clast);                                    \
    _Pragma("unroll") for (int i = 0; i < APT; i++)                         \
      AR[i] = Ag[(size_t)cl_ * 1024 + a_piece(i * NT + tid)];               \
    _Pragma("unroll") for (int i = 0; i < 4; i++)                           \
      BR[i] = Wg[((size_t)cl_ * NB * 4 + i) * 64 + lane];                   \
    /* keep the scheduler from sinking these loads towards their use */     \
    __builtin_amdgcn_sched_barrier(0);                                      \
  }
#define GEMM_STAGE(S, AR, BR)                                               \
  if ((S) < D) {                                                            \
    const int cc = c + (S);                                                 \
    u32x4* buf = As[(S) & 1];                                               \
    /* past the end of the slice the weight operand is zeroed: the body stays branch free; \
       the masked copy also frees the staging registers before they are refilled */ \
    const unsigned keep = cc < c1 ? 0xffffffffu : 0u;                       \
    u32x4 bcur[4];                                                          \
    _Pragma("unroll") for (int i = 0; i < APT; i++) buf[a_piece(i * NT + tid)] = AR[i]; \
    _Pragma("unroll") for (int i = 0; i < 4; i++) bcur[i] = BR[i] & keep;   \
    __builtin_amdgcn_sched_barrier(0);                                      \
    __syncthreads();                                                        \
    GEMM_LOAD(AR, BR, cc + D)                                               \
    /* all 16 row operands of the chunk are requested from LDS before the first MFMA: with one \
       wave per SIMD nothing else hides the LDS latency */                  \
    u32x4 av[16];                                                           \
    _Pragma("unroll") for (int i = 0; i < 16; i++) if ((i & 3) < MB) av[i] = buf[i * 64 + lane]; \
    __builtin_amdgcn_sched_barrier(0);                                      \
    _Pragma("unroll") for (int kk = 0; kk < 4; kk++) {                      \
      bf16x8 b = __builtin_bit_cast(bf16x8, bcur[kk]);                      \
      _Pragma("unroll") for (int mb = 0; mb < MB; mb++) {                   \
        bf16x8 a = __builtin_bit_cast(bf16x8, av[kk * 4 + mb]);             \
        acc[mb] = EPI == EPI_LSE                                            \
                      ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[mb], 0, 0, 0) \
                      : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[mb], 0, 0, 0); \
      }                                                                     \
    }                                                                       \
  }
  GEMM_LOAD(a0, b0, c0)
  if (D > 1) GEMM_LOAD(a1, b1, c0 + 1)
  if (D > 2) GEMM_LOAD(a2, b2, c0 + 2)
  if (D > 3) GEMM_LOAD(a3, b3, c0 + 3)
  // the barrier inside a stage also orders its LDS store after every wave's reads of the same
  // buffer two chunks earlier (D is even, so stage parity equals chunk parity)
  for (int c = c0; c < c1; c += D) {
    GEMM_STAGE(0, a0, b0)
    GEMM_STAGE(1, a1, b1)
    GEMM_STAGE(2, a2, b2)
    GEMM_STAGE(3, a3, b3)
  }
#undef GEMM_LOAD
#undef GEMM_STAGE
  if (!active) return;
  if (EPI == EPI_LSE) {
    // acc[mb][i] = z[batch row mb*32 + lane%32][vocab nb*32 + (i/4)*8 + (lane/32)*4 + i%4]
    float2* P = (float2*)Cv;
#pragma unroll
    for (int mb = 0; mb < MB; mb++) {
      const int row = mt * 128 + mb * 32 + (lane & 31);
      float mx = acc[mb][0];
#pragma unroll
      for (int i = 1; i < 16; i++) mx = fmaxf(mx, acc[mb][i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      float sm = 0.f;
#pragma unroll
      for (int i = 0; i < 16; i++) sm += exp2f((acc[mb][i] - mx) * scale_c);
      sm += __shfl_xor(sm, 32, 64);
      if (row < M) {
        if (lane < 32) P[(size_t)row * NB + nb] = make_float2(mx, sm);
        const int t = tgt[row];
        if ((t >> 5) == nb && ((t >> 2) & 1) == (lane >> 5)) {
          const int isel = ((t & 31) >> 3) * 4 + (t & 3);
          float z = acc[mb][0];
#pragma unroll
          for (int i = 1; i < 16; i++) z = isel == i ? acc[mb][i] : z;
          zt[row] = z;
        }
      }
    }
    return;
  }
  const int col = nb * 32 + (lane & 31);
  float* Cp = (float*)Cv + (size_t)blockIdx.z * M * N;
  if (EPI == EPI_STORE_MAX) {
    // v[j], j = 16 mb + i, is the value of row mt*128 + 32 mb + (i>>2)*8 + (lane>>5)*4 + (i&3) in
    // this lane's column.  Step s pairs lanes L and L ^ (1 << s): of every two values the lane
    // with bit s clear keeps the even one, the other lane the odd one, and each takes the maximum
    // with what its partner held of the kept one.  After the five steps lane L holds the strip
    // maxima of the values j = 32 k + (L & 31).
    float v[16 * MB];
#pragma unroll
    for (int mb = 0; mb < MB; mb++)
#pragma unroll
      for (int i = 0; i < 16; i++) v[mb * 16 + i] = acc[mb][i];
    int n = 16 * MB;
#pragma unroll
    for (int st = 0; st < 5; st++) {
      const bool up = (lane >> st) & 1;
      if (n >= 2) {
        n >>= 1;
#pragma unroll
        for (int k = 0; k < 32; k++)
          if (k < n) {
            const float keep = up ? v[2 * k + 1] : v[2 * k];
            const float send = up ? v[2 * k] : v[2 * k + 1];
            v[k] = fmaxf(keep, __shfl_xor(send, 1 << st, 64));
          }
      } else {
        v[0] = fmaxf(v[0], __shfl_xor(v[0], 1 << st, 64));
      }
    }
    constexpr int NOUT = MB == 4 ? 2 : 1;
    const int jl = MB == 1 ? (lane & 15) : (lane & 31);
    if (MB > 1 || (lane & 16) == 0) {
#pragma unroll
      for (int k = 0; k < NOUT; k++) {
        const int j = 32 * k + jl, mb = j >> 4, i = j & 15;
        const int row = mt * 128 + mb * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
        if (row < M) zt[(size_t)row * NB + nb] = v[k];
      }
    }
  }
#pragma unroll
  for (int mb = 0; mb < MB; mb++) {
#pragma unroll
    for (int i = 0; i < 16; i++) {
      int row = mt * 128 + mb * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
      float v = acc[mb][i];
      if (EPI == EPI_SWIGLU) {
        float u = __shfl_xor(v, 16, 64);            // lanes 0..15 of a half: gate; 16..31: up
        if ((lane & 16) == 0 && row < M) {
          float y = v / (1.0f + __expf(-v)) * u;
          int j = nb * 16 + (lane & 15);
          ((bf16_t*)Cv)[atile_off(row, j, N >> 1)] = f2bf(y);
        }
      } else if (row < M) {
        __builtin_nontemporal_store(v, &Cp[(size_t)row * N + col]);   // leaves the L2 early instead of at the end of the kernel
      }
    }
  }
}

// =============================================================================================
// GEMM for many rows (chunked prefill, teacher-forced passes) and wide outputs: tile 256 x 256,
// 4 waves as 2 x 2, wave tile 128 x 128 (16 accumulators of 32x32).  Per 16-k step a wave reads 4
// row and 4 column operands from LDS for 16 MFMAs, so an operand byte fetched through the L1 feeds
// twice the MFMAs of the 128 x 128 kernel above.  Both operands are staged through LDS (double
// buffered, 2 x 64 KB).
// The loop is one steady stream: a chunk is 16 pieces of 16 bytes per thread, and every group of
// 4 MFMAs carries one global load (a piece 24 groups = 1.5 chunks ahead of the store that needs
// it, in a ring of 32 register slots), the LDS stores of the next chunk (all done by group 11),
// and two of the eight LDS operand reads of the next 16-k step.  The workgroup barrier sits in
// front of group 12: by then the next chunk is complete in the other buffer and this buffer has
// been read out, so groups 12-15 already fetch the next chunk's first operands and no LDS latency
// is exposed at the chunk boundary.  A burst of 16 loads per thread at the top of every chunk
// (all 256 workgroups at about the same time) instead of this even stream costs 17-26 %.
// sched_group_barrier pins the interleaving (MFMA, load, MFMA, stores, MFMA, reads, MFMA).
// XCD-aware tile numbering (xcd_tile256) is worth another 1.5-3 %.
// The k order per output element is that of the 128 x 128 kernel: results are bit-identical.
// Measured at 8192 rows (us, before -> after the steady stream): N = 6144 K = 2560 310 -> 266,
// N = 19456 K = 2560 1010 -> 843, N = 24576 K = 4096 1800 -> 1462, N = 4096 K = 12288 830 -> 656;
// N = 2560 stays with the kernel above (320 workgroups on 256 CUs).  K / 64 must be even; no
// split-K.
// =============================================================================================
// Tile of a workgroup: the hardware hands workgroups to the 8 XCDs round-robin by linear index
// and each XCD has its own L2.  XCD x works through a contiguous range of a sequence that walks
// groups of 4 row tiles column by column, so the 32 workgroups resident on an XCD cover a
// compact block of 4 x 8 tiles (12 distinct operand tiles per chunk instead of ~22).  A
// bijection for any tile counts.
__device__ __forceinline__ void xcd_tile256(int id, int tiles_m, int tiles_n, int* tm, int* tn) {
  constexpr int GM = 4;
  const int total = tiles_m * tiles_n;
  const int base = total >> 3, rem = total & 7, x = id & 7;
  const int vid = x * base + min(x, rem) + (id >> 3);
  const int per_group = GM * tiles_n, grp = vid / per_group, first = grp * GM;
  const int gm = min(GM, tiles_m - first), within = vid - grp * per_group;
  *tm = first + within % gm;
  *tn = within / gm;
}

template <int EPI>
__global__ __launch_bounds__(256) void gemm256_mfma_kernel(const bf16_t* __restrict__ A,
                                                      const bf16_t* __restrict__ Wp,
                                                      void* __restrict__ Cv, int M, int N, int K) {
  extern __shared__ u32x4 smem[];            // [2][A: 2048 | B: 2048] pieces of 16 bytes
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int NB = N >> 5;
  const int nchunks = K >> 6;
  const int mtiles128 = (M + 127) >> 7;
  int bx, by;
  xcd_tile256(blockIdx.y * gridDim.x + blockIdx.x, gridDim.y, gridDim.x, &by, &bx);
  const int mt0 = by * 2, mt1 = min(mt0 + 1, mtiles128 - 1);   // second half clamped (results dropped)
  const u32x4* Ag0 = (const u32x4*)(A + (size_t)mt0 * K * 128);
  const u32x4* Ag1 = (const u32x4*)(A + (size_t)mt1 * K * 128);
  const int strip0 = bx * 8;
  // weight pieces of this thread: 2048 pieces per chunk = 8 strips x 256; piece p = i * 256 + tid
  // strips past the end (N not a multiple of 256) are clamped to the last one; results dropped
  const int nvalid = min(8, NB - strip0);
  const int wbase = strip0 * 256 + tid;
  const u32x4* Wg = (const u32x4*)Wp;
  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < 4; b++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[a][b][e] = 0.f;
  // the 16 pieces of a thread and chunk: 0-3 rows 0-127, 4-7 rows 128-255, 8-15 the 8 strips;
  // chunks past the end are clamped to the last one (re-reads that hit in cache, never used)
  auto piece_src = [&](int chunk, int p) -> const u32x4* {
    const int cl = min(chunk, nchunks - 1);
    if (p < 4) return Ag0 + (size_t)cl * 1024 + p * 256 + tid;
    if (p < 8) return Ag1 + (size_t)cl * 1024 + (p - 4) * 256 + tid;
    return Wg + (size_t)cl * NB * 256 + wbase + min(p - 8, nvalid - 1) * 256;
  };
  auto piece_dst = [&](int buf, int p) -> u32x4* {
    return smem + buf * 4096 + (p < 8 ? p * 256 : 2048 + (p - 8) * 256) + tid;
  };
  constexpr int DIST = 24;                   // groups between a piece's load and the group of piece p's store
  u32x4 rs[32];                              // ring: the load of group T (counted from chunk 0) lands in slot T % 32
  u32x4 av[2][4], bv[2][4];
  {
    u32x4 t0[16];
#pragma unroll
    for (int p = 0; p < 16; p++) t0[p] = *piece_src(0, p);
#pragma unroll
    for (int q = 0; q < DIST; q++) rs[(q + 32 - DIST) & 31] = *piece_src(1 + (q >> 4), q & 15);
#pragma unroll
    for (int p = 0; p < 16; p++) *piece_dst(0, p) = t0[p];
  }
  __syncthreads();
  {
    const u32x4* as_ = smem + wm * 1024;
    const u32x4* bs_ = smem + 2048 + wn * 1024;
#pragma unroll
    for (int x = 0; x < 4; x++) { av[0][x] = as_[x * 64 + lane]; bv[0][x] = bs_[(x * 4) * 64 + lane]; }
  }
  for (int c = 0; c < nchunks; c += 2) {   // nchunks is even (checked by the launcher)
#pragma unroll
    for (int it2 = 0; it2 < 2; it2++) {
      const int i = c + it2;               // chunk being multiplied; it sits in LDS buffer it2
      const u32x4* as_cur = smem + it2 * 4096 + wm * 1024;
      const u32x4* bs_cur = smem + it2 * 4096 + 2048 + wn * 1024;
      const u32x4* as_nxt = smem + (1 - it2) * 4096 + wm * 1024;
      const u32x4* bs_nxt = smem + (1 - it2) * 4096 + 2048 + wn * 1024;
#pragma unroll
      for (int g = 0; g < 16; g++) {
        const int kk = g >> 2, a = g & 3;
        if (g == 12) __syncthreads();      // chunk i + 1 is complete in the other buffer; this one is read out
        rs[(16 * it2 + g) & 31] = *piece_src(i + 1 + ((g + DIST) >> 4), (g + DIST) & 15);
        // stores of chunk i + 1: pieces p with 3 p / 4 == g (16 pieces over groups 0-11)
#pragma unroll
        for (int p = 0; p < 16; p++)
          if ((3 * p) / 4 == g) *piece_dst(1 - it2, p) = rs[(16 * it2 + p + 32 - DIST) & 31];
        // operands of the next 16-k step
        if (kk < 3) {
          av[(kk + 1) & 1][a] = as_cur[((kk + 1) * 4 + a) * 64 + lane];
          bv[(kk + 1) & 1][a] = bs_cur[(a * 4 + kk + 1) * 64 + lane];
        } else {
          av[0][a] = as_nxt[a * 64 + lane];
          bv[0][a] = bs_nxt[(a * 4) * 64 + lane];
        }
#pragma unroll
        for (int b = 0; b < 4; b++)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av[kk & 1][a]),
                                                              __builtin_bit_cast(bf16x8, bv[kk & 1][b]),
                                                              acc[a][b], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // global load
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x200, 2, 0);   // LDS stores
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // LDS reads
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      }
    }
  }
  float* Cp = (float*)Cv;
#pragma unroll
  for (int b = 0; b < 4; b++) {
    const int nb = strip0 + wn * 4 + b;
    if (nb >= NB) continue;
    const int col = nb * 32 + (lane & 31);
#pragma unroll
    for (int a = 0; a < 4; a++) {
      const int mtile = wm == 0 ? mt0 : mt0 + 1;
      if (mtile >= mtiles128) continue;
#pragma unroll
      for (int i = 0; i < 16; i++) {
        int row = mtile * 128 + a * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
        float v = acc[a][b][i];
        if (EPI == EPI_SWIGLU) {
          float u = __shfl_xor(v, 16, 64);
          if ((lane & 16) == 0 && row < M) {
            float y = v / (1.0f + __expf(-v)) * u;
            int j = nb * 16 + (lane & 15);
            ((bf16_t*)Cv)[atile_off(row, j, N >> 1)] = f2bf(y);
          }
        } else if (row < M) {
          __builtin_nontemporal_store(v, &Cp[(size_t)row * N + col]);
        }
      }
    }
  }
}

static bool use_gemm256(int M, int N, int K, int epilogue, int splits) {
  const int tiles = ((M + 255) / 256) * ((N + 255) / 256);
  return splits == 1 && (epilogue == EPI_STORE || epilogue == EPI_SWIGLU) && N >= 4096 && N % 32 == 0 &&
         (K / 64) % 2 == 0 && K >= 128 && tiles >= 512;
}

static void launch_gemm256(hipStream_t s, const bf16_t* A, const bf16_t* Wp, void* C, int M, int N,
                           int K, int epilogue) {
  static bool attr_set = false;      // 128 KB of dynamic LDS need the opt-in once per process
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)gemm256_mfma_kernel<EPI_STORE>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, 131072);
    (void)hipFuncSetAttribute((const void*)gemm256_mfma_kernel<EPI_SWIGLU>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, 131072);
    attr_set = true;
  }
  dim3 grid((N + 255) / 256, (M + 255) / 256, 1);
  if (epilogue == EPI_STORE) gemm256_mfma_kernel<EPI_STORE><<<grid, 256, 131072, s>>>(A, Wp, C, M, N, K);
  else gemm256_mfma_kernel<EPI_SWIGLU><<<grid, 256, 131072, s>>>(A, Wp, C, M, N, K);
}

template <int D, int NW, int MB>
static void gemm_launch(hipStream_t s, dim3 grid, const bf16_t* A, const bf16_t* Wp, void* C, int M,
                        int N, int K, int epilogue, int cps) {
  if (epilogue == EPI_STORE)
    gemm_mfma_kernel<EPI_STORE, D, NW, MB><<<grid, 64 * NW, 0, s>>>(A, Wp, C, M, N, K, cps, nullptr, nullptr, 0.f);
  else
    gemm_mfma_kernel<EPI_SWIGLU, D, NW, MB><<<grid, 64 * NW, 0, s>>>(A, Wp, C, M, N, K, cps, nullptr, nullptr, 0.f);
}

// depth = chunks in flight per workgroup (2 or 4)
int launch_gemm_mfma_cfg(hipStream_t s, const bf16_t* A, const bf16_t* Wp, void* C, int M, int N,
                         int K, int epilogue, int splits, int nw, int depth) {
  if (M <= 0) return 0;
  int nchunks = K / 64;
  if (splits < 1 || epilogue == EPI_SWIGLU) splits = 1;
  if (splits > nchunks) splits = nchunks;
  if (nw == 4 && depth == 2 && use_gemm256(M, N, K, epilogue, splits)) {
    launch_gemm256(s, A, Wp, C, M, N, K, epilogue);
    return 1;
  }
  int cps = (nchunks + splits - 1) / splits;
  splits = (nchunks + cps - 1) / cps;
  dim3 grid((N + 32 * nw - 1) / (32 * nw), (M + 127) / 128, splits);
  const int mb = M <= 32 ? 1 : M <= 64 ? 2 : 4;    // row blocks in use (one row tile when < 4)
  if (nw == 2 && depth == 2) {
    if (mb == 1) gemm_launch<2, 2, 1>(s, grid, A, Wp, C, M, N, K, epilogue, cps);
    else if (mb == 2) gemm_launch<2, 2, 2>(s, grid, A, Wp, C, M, N, K, epilogue, cps);
    else gemm_launch<2, 2, 4>(s, grid, A, Wp, C, M, N, K, epilogue, cps);
  } else if (nw == 2) {
    gemm_launch<4, 2, 4>(s, grid, A, Wp, C, M, N, K, epilogue, cps);
  } else if (depth == 2) {
    if (mb == 1) gemm_launch<2, 4, 1>(s, grid, A, Wp, C, M, N, K, epilogue, cps);
    else if (mb == 2) gemm_launch<2, 4, 2>(s, grid, A, Wp, C, M, N, K, epilogue, cps);
    else gemm_launch<2, 4, 4>(s, grid, A, Wp, C, M, N, K, epilogue, cps);
  } else {
    gemm_launch<4, 4, 4>(s, grid, A, Wp, C, M, N, K, epilogue, cps);
  }
  return splits;
}

int launch_gemm_mfma(hipStream_t s, const bf16_t* A, const bf16_t* Wp, void* C, int M, int N,
                     int K, int epilogue, int splits, int nw) {
  // two chunks in flight: fewer registers, more resident workgroups (measured best at M = 128)
  return launch_gemm_mfma_cfg(s, A, Wp, C, M, N, K, epilogue, splits, nw, 2);
}

// lm-head of a decode step: logits[M, V] (fp32, row-major) and stripmax[M, V / 32].
void launch_lm_head_logits(hipStream_t s, const bf16_t* A, const bf16_t* Wp, float* logits, int M,
                           int V, int K, float* stripmax) {
  if (M <= 0) return;
  dim3 grid((V + 127) / 128, (M + 127) / 128, 1);
  const int cps = K / 64;
  if (M <= 32)
    gemm_mfma_kernel<EPI_STORE_MAX, 2, 4, 1><<<grid, 256, 0, s>>>(A, Wp, logits, M, V, K, cps, nullptr, stripmax, 0.f);
  else if (M <= 64)
    gemm_mfma_kernel<EPI_STORE_MAX, 2, 4, 2><<<grid, 256, 0, s>>>(A, Wp, logits, M, V, K, cps, nullptr, stripmax, 0.f);
  else
    gemm_mfma_kernel<EPI_STORE_MAX, 2, 4, 4><<<grid, 256, 0, s>>>(A, Wp, logits, M, V, K, cps, nullptr, stripmax, 0.f);
}

// One workgroup per row: combine the per-strip (max, sum) pairs in a fixed order and write
// log softmax(z / T)[target] = (z_t - max) c ln2 - ln sum, c = log2(e) / T.
__global__ __launch_bounds__(256) void lse_finish_kernel(const float2* __restrict__ P,
                                                         const float* __restrict__ zt, int NB,
                                                         float scale_c, float* __restrict__ lp) {
  __shared__ float red[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  const float2* p = P + (size_t)row * NB;
  float mx = -3.0e38f;
  for (int j = tid; j < NB; j += 256) mx = fmaxf(mx, p[j].x);
  mx = wave_max(mx);
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sm = 0.f;
  for (int j = tid; j < NB; j += 256) {
    float2 v = p[j];
    sm += v.y * exp2f((v.x - mx) * scale_c);
  }
  sm = wave_sum(sm);
  if ((tid & 63) == 0) red[tid >> 6] = sm;
  __syncthreads();
  if (tid == 0) {
    float S = (red[0] + red[1]) + (red[2] + red[3]);
    lp[row] = (zt[row] - mx) * scale_c * 0.6931471805599453f - logf(S);
  }
}

void launch_lm_head_logprob(hipStream_t s, const bf16_t* A, const bf16_t* Wp, int M, int V, int K,
                            const int32_t* tgt, float scale_c, float* part, float* zt, float* lp) {
  if (M <= 0) return;
  dim3 grid((V + 127) / 128, (M + 127) / 128, 1);
  gemm_mfma_kernel<EPI_LSE, 2, 4, 4><<<grid, 256, 0, s>>>(A, Wp, part, M, V, K, K / 64, tgt, zt, scale_c);
  lse_finish_kernel<<<M, 256, 0, s>>>((const float2*)part, zt, V / 32, scale_c, lp);
}

// =============================================================================================
// Paged GQA attention, one workgroup (4 waves) per (work item, kv head, context split).
// The MFMA column index n = G * r + hq carries query row r of the item and query head hq of the kv
// head's group of G = n_q / n_kv heads (G a power of two <= 16, r < 16 / G), so decode (1 row) and
// chunked prefill (16 / G rows) share the kernel.
// Per 16-token page:  S^T[token, n] = K[token, :] . Q[n, :]   (4 x mfma 16x16x32, K straight from
// the page in operand order), online softmax per column, O^T[d, n] += V^T[d, token] P^T[token, n]
// (8 x mfma 16x16x16; the score accumulator layout is exactly the P operand layout).
// The item's page range is split over the 4 waves; partial (max, sum, O) are merged in fixed order
// through LDS and, when a row's context was cut into several items, through a scratch buffer and a
// second kernel.
// =============================================================================================
#define ATT_NEG (-1.0e30f)

// One page of the online-softmax loop; see the kernels below for the variables they use.
// Two flavours of the page load.  The decode kernel reads a trajectory's own pages once per step:
// those loads carry the non-temporal hint (measured 8-10 % more bandwidth than plain loads).  Pages
// shared with other trajectories of the step (a forked prompt) keep plain loads so that the group
// finds them in L2, and so does the prefill kernel, which re-reads pages across waves and items.
// The choice is made per wave, outside the page loop: inside it the compiler would merge the two
// loads into one and drop the hint.
// kpool / vpool are byte pointers; a (page, kv head) block is BLK bytes (4096: bf16, 2048: 8-bit
// cache) that a wave reads as NLD 16-byte slots per lane (head_off = kv head * BLK + lane * 16).
#define ATT_LOAD_PLAIN(KR, VR, PAGEID)                                        \
  {                                                                           \
    const size_t base_ = (size_t)(PAGEID) * nkv * BLK + head_off;             \
    _Pragma("unroll") for (int c = 0; c < NLD; c++) {                         \
      KR[c] = *(const u32x4*)(kpool + base_ + c * 1024);                      \
      VR[c] = *(const u32x4*)(vpool + base_ + c * 1024);                      \
    }                                                                         \
  }
#define ATT_LOAD_STREAM(KR, VR, PAGEID)                                       \
  {                                                                           \
    const size_t base_ = (size_t)(PAGEID) * nkv * BLK + head_off;             \
    _Pragma("unroll") for (int c = 0; c < NLD; c++) {                         \
      KR[c] = __builtin_nontemporal_load((const u32x4*)(kpool + base_ + c * 1024)); \
      VR[c] = __builtin_nontemporal_load((const u32x4*)(vpool + base_ + c * 1024)); \
    }                                                                         \
  }
// Operand register i of a page buffer: the 16-byte slot itself (bf16 cache), or half a raw slot
// of the 8-bit cache widened to bf16 (exact) just before use, so that no widened page stays live.
template <bool FP8, int N>
__device__ __forceinline__ u32x4 att_operand(const u32x4 (&R)[N], int i) {
  if constexpr (FP8) {
    uint32_t a, b, c, d;
    e4m3x4_to_bf16(R[i >> 1][2 * (i & 1)], &a, &b);
    e4m3x4_to_bf16(R[i >> 1][2 * (i & 1) + 1], &c, &d);
    return (u32x4){a, b, c, d};
  } else {
    return R[i];
  }
}
#define ATT_PAGE(KR, VR, PG)                                                  \
  {                                                                           \
    f32x4 S = (f32x4){0.f, 0.f, 0.f, 0.f};                                    \
    _Pragma("unroll") for (int c = 0; c < 4; c++)                             \
      S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, att_operand<FP8>(KR, c)), \
                                                  __builtin_bit_cast(bf16x8, qreg[c]), S, 0, 0, 0); \
    float sv[4], mx = ATT_NEG;                                                \
    bool vis[4];                                                              \
    _Pragma("unroll") for (int i = 0; i < 4; i++) {                           \
      int tg = (PG) * RL_PAGE + 4 * g + i;                                    \
      vis[i] = colvalid && tg <= mypos && (PG) < pg1;                         \
      sv[i] = vis[i] ? S[i] * scale2 : ATT_NEG;                               \
      mx = fmaxf(mx, sv[i]);                                                  \
    }                                                                         \
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));                                   \
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));                                   \
    float mn = fmaxf(m, mx);                                                  \
    float alpha = exp2f(m - mn);                                              \
    float ps = 0.f;                                                           \
    s16x4 pb;                                                                 \
    _Pragma("unroll") for (int i = 0; i < 4; i++) {                           \
      float p = vis[i] ? exp2f(sv[i] - mn) : 0.f;                             \
      ps += p;                                                                \
      pb[i] = (short)f2bf(p);                                                 \
    }                                                                         \
    l = l * alpha + ps;                                                       \
    m = mn;                                                                   \
    _Pragma("unroll") for (int jp = 0; jp < 4; jp++) {                        \
      s16x4 v0, v1;                                                           \
      const u32x4 vr_ = att_operand<FP8>(VR, jp);                             \
      v0[0] = (short)(vr_[0] & 0xffff); v0[1] = (short)(vr_[0] >> 16);        \
      v0[2] = (short)(vr_[1] & 0xffff); v0[3] = (short)(vr_[1] >> 16);        \
      v1[0] = (short)(vr_[2] & 0xffff); v1[1] = (short)(vr_[2] >> 16);        \
      v1[2] = (short)(vr_[3] & 0xffff); v1[3] = (short)(vr_[3] >> 16);        \
      _Pragma("unroll") for (int i = 0; i < 4; i++) { acc[2 * jp][i] *= alpha; acc[2 * jp + 1][i] *= alpha; } \
      acc[2 * jp] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v0, pb, acc[2 * jp], 0, 0, 0); \
      acc[2 * jp + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v1, pb, acc[2 * jp + 1], 0, 0, 0); \
    }                                                                         \
  }
// Order of a page step of the decode kernel: (2 loads, 1 MFMA) x 4, everything else after.
#define ATT_SPREAD                                                            \
  __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);                          \
  __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          \
  __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);                          \
  __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          \
  __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);                          \
  __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          \
  __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);                          \
  __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
// The decode kernel's page loop (uses pt, pg0, pg1, pglast, head_off, kpool, vpool, nkv and the
// buffers kA, vA, kB, vB of the enclosing kernel); LOAD is one of the two load macros.
#define ATT_PAGE_LOOP(LOAD)                                                   \
  if (pg0 < pg1) {                                                            \
    int id_cur = pt[pg0];                                                     \
    int id_nxt = pt[min(pg0 + 1, pglast)];                                    \
    LOAD(kA, vA, id_cur)                                                      \
    for (int pg = pg0; pg < pg1; pg += 2) {                                   \
      /* page pg is in A; request the table entry of pg+2 (first: the counter of outstanding \
         loads is in order, and its consumer must not wait for the page behind it), then pg+1 -> B. \
         The eight loads of a page are issued two at a time between the four score MFMAs of the \
         page being consumed (ATT_SPREAD) rather than in one burst: +0.5-2 % bandwidth. */ \
      int id_n2 = pt[min(pg + 2, pglast)];                                    \
      __builtin_amdgcn_sched_barrier(0);                                      \
      LOAD(kB, vB, id_nxt)                                                    \
      ATT_PAGE(kA, vA, pg)                                                \
      ATT_SPREAD                                                              \
      __builtin_amdgcn_sched_barrier(0);                                      \
      /* page pg+1 is in B; request the table entry of pg+3, then pg+2 -> A */ \
      id_nxt = pt[min(pg + 3, pglast)];                                       \
      LOAD(kA, vA, id_n2)                                                     \
      ATT_PAGE(kB, vB, pg + 1)                                            \
      ATT_SPREAD                                                              \
      __builtin_amdgcn_sched_barrier(0);                                      \
    }                                                                         \
  }

// The same loop three pages deep (buffers A-C; two pages in flight while one is consumed), used
// with the 8-bit cache: its pages are half as large, and one of them in flight per wave no longer
// covers the memory latency.
#define ATT_PAGE_LOOP3(LOAD)                                                  \
  if (pg0 < pg1) {                                                            \
    int i0 = pt[pg0], i1 = pt[min(pg0 + 1, pglast)], i2 = pt[min(pg0 + 2, pglast)]; \
    LOAD(kA, vA, i0)                                                          \
    LOAD(kB, vB, i1)                                                          \
    for (int pg = pg0; pg < pg1; pg += 3) {                                   \
      const int j0 = pt[min(pg + 3, pglast)], j1 = pt[min(pg + 4, pglast)];   \
      const int j2 = pt[min(pg + 5, pglast)];                                 \
      LOAD(kC, vC, i2)                                                        \
      __builtin_amdgcn_sched_barrier(0);                                      \
      ATT_PAGE(kA, vA, pg)                                                \
      __builtin_amdgcn_sched_barrier(0);                                      \
      LOAD(kA, vA, j0)                                                        \
      __builtin_amdgcn_sched_barrier(0);                                      \
      ATT_PAGE(kB, vB, pg + 1)                                            \
      __builtin_amdgcn_sched_barrier(0);                                      \
      LOAD(kB, vB, j1)                                                        \
      __builtin_amdgcn_sched_barrier(0);                                      \
      ATT_PAGE(kC, vC, pg + 2)                                            \
      __builtin_amdgcn_sched_barrier(0);                                      \
      i2 = j2;                                                                \
    }                                                                         \
  }

// row_stride: floats between the outputs of two MFMA columns of one part
__device__ __forceinline__ void attn_merge_store(const float* __restrict__ pm,
                                                 const float* __restrict__ pl,
                                                 const float* __restrict__ pacc, int nparts,
                                                 size_t part_stride_ml, size_t part_stride_acc,
                                                 int row_stride, int n, int d0, float* m_out,
                                                 float* l_out, float* o8) {
  float mt = ATT_NEG;
  for (int w = 0; w < nparts; w++) mt = fmaxf(mt, pm[w * part_stride_ml + n]);
  float L = 0.f;
#pragma unroll
  for (int e = 0; e < 8; e++) o8[e] = 0.f;
  for (int w = 0; w < nparts; w++) {
    float f = exp2f(pm[w * part_stride_ml + n] - mt);
    L += f * pl[w * part_stride_ml + n];
    const float* a = pacc + w * part_stride_acc + (size_t)n * row_stride + d0;
#pragma unroll
    for (int e = 0; e < 8; e++) o8[e] += f * a[e];
  }
  *m_out = mt;
  *l_out = L;
}

template <bool FP8>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void attention_mfma_kernel(
    const bf16_t* __restrict__ q, const char* __restrict__ kpool, const char* __restrict__ vpool,
    const AttnItem* __restrict__ items, const int32_t* __restrict__ rowlist,
    const int32_t* __restrict__ page_table, bf16_t* __restrict__ o, float* __restrict__ scratch,
    int nq, int nkv, int gshift, int pt_stride, float scale2) {
  // a column's 128 outputs are padded to 132 floats: with a stride of 128 the 16 lanes that hold
  // one token group's 16 columns would all store into the same 4 banks
  constexpr int AST = 132;
  __shared__ __align__(16) float s_acc[4 * 16 * AST];
  __shared__ float s_m[4 * 16];
  __shared__ float s_l[4 * 16];
  // blockIdx.x = item * nkv + kvh: consecutive workgroups go round-robin to the 8 XCDs, so with
  // kv head fastest all trajectories of one kv head share an XCD (for nkv = 8) and trajectories
  // that share prompt pages (a forked group, adjacent items) find each other's pages in that L2.
  const int item_idx = blockIdx.x / nkv;
  const AttnItem it = items[item_idx];
  const int kvh = blockIdx.x - item_idx * nkv;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 4, n = lane & 15, r = n >> gshift, hq = n & ((1 << gshift) - 1);
  const bool colvalid = r < it.nrows;
  // shared-prefix items: every page of the range lies before every member's position
  const bool gather = (it.gather & 1) != 0;
  const int mypos = gather ? 0x3fffffff : it.pos0 + r;
  const int qrow = !colvalid ? 0 : (gather ? rowlist[it.row0 + r] : it.row0 + r);
  const int per = (it.pg_hi - it.pg_lo + 3) >> 2;
  const int pg0 = it.pg_lo + wave * per, pg1 = min(pg0 + per, it.pg_hi);
  const int32_t* pt = page_table + (size_t)it.slot * pt_stride;

  u32x4 qreg[4];
#pragma unroll
  for (int c = 0; c < 4; c++) {
    qreg[c] = (u32x4){0u, 0u, 0u, 0u};
    if (colvalid)
      qreg[c] = *(const u32x4*)(q + ((size_t)qrow * nq + ((kvh << gshift) + hq)) * 128 + c * 32 + g * 8);
  }
  f32x4 acc[8];
#pragma unroll
  for (int j = 0; j < 8; j++) acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m = ATT_NEG, l = 0.f;

  // Two page buffers (A, B) alternate: while one page is consumed the next one is already on its
  // way, and the page-table entry after that has been requested.  Loads past the end of this
  // wave's range are clamped to its last page (a re-read that hits in cache) so that nothing in
  // the loop defines registers conditionally; sched_barrier keeps the loads where they are
  // written, ahead of the arithmetic.
  const int pglast = max(pg1 - 1, pg0);
  constexpr int NLD = FP8 ? 2 : 4, BLK = FP8 ? 2048 : 4096;
  const size_t head_off = (size_t)kvh * BLK + lane * 16;
  u32x4 kA[NLD], vA[NLD], kB[NLD], vB[NLD];
  // a wave whose share of the pages starts behind the trajectory's shared leading pages streams
  if constexpr (FP8) {
    u32x4 kC[NLD], vC[NLD];
    if (pg0 >= (it.gather >> 8)) {
      ATT_PAGE_LOOP3(ATT_LOAD_STREAM)
    } else {
      ATT_PAGE_LOOP3(ATT_LOAD_PLAIN)
    }
  } else {
    if (pg0 >= (it.gather >> 8)) {
      ATT_PAGE_LOOP(ATT_LOAD_STREAM)
    } else {
      ATT_PAGE_LOOP(ATT_LOAD_PLAIN)
    }
  }
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);
  // wave partials -> LDS: acc[jb][i] is O^T[d = 16 jb + 4 g + i][column n]
#pragma unroll
  for (int jb = 0; jb < 8; jb++) *(f32x4*)&s_acc[(wave * 16 + n) * AST + jb * 16 + g * 4] = acc[jb];
  if (g == 0) { s_m[wave * 16 + n] = m; s_l[wave * 16 + n] = l; }
  __syncthreads();
  // 256 threads: column cn = tid / 16, dims d0 .. d0+7
  const int cn = tid >> 4, d0 = (tid & 15) * 8;
  float mt, L, o8[8];
  attn_merge_store(s_m, s_l, s_acc, 4, 16, 16 * AST, AST, cn, d0, &mt, &L, o8);
  const int cr = cn >> gshift, chq = cn & ((1 << gshift) - 1);
  if (it.part < 0) {
    if (cr < it.nrows) {
      float inv = 1.0f / L;
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 4; e++)
        w[e] = (uint32_t)f2bf(o8[2 * e] * inv) | ((uint32_t)f2bf(o8[2 * e + 1] * inv) << 16);
      *(uint4*)(o + atile_off(it.row0 + cr, ((kvh << gshift) + chq) * 128 + d0, nq * 128)) =
          make_uint4(w[0], w[1], w[2], w[3]);
    }
  } else {
    float* dst = scratch + ((size_t)it.part * nkv + kvh) * (16 * 130);
#pragma unroll
    for (int e = 0; e < 8; e++) dst[cn * 128 + d0 + e] = o8[e];
    if ((tid & 15) == 0) { dst[16 * 128 + cn] = mt; dst[16 * 128 + 16 + cn] = L; }
  }
}

// Two consecutive pages (32 keys) of the LDS-staged prefill kernel for the CB column blocks of a
// wave.  kb / vb point at the first page's key / value block in LDS, the second page's blocks lie
// BLK bytes behind them.  Scores: 4 x mfma 16x16x32 per page and column block.  The two pages
// share one softmax update, and P (32 keys x 16 columns) meets the two pages' values in one
// 16x16x32 MFMA per 16 output dims: operand slot 8 g + i of lane group g is key 4 g + i of the
// first page for i < 4 and key 4 g + i - 4 of the second page otherwise, on both operands.
template <int CB, bool FP8, bool MASKED>
__device__ __forceinline__ void prefill_pair(const char* kb, const char* vb, int pg,
                                             const u32x4 (&qreg)[CB][4], f32x4 (&acc)[CB][8],
                                             float (&m)[CB], float (&l)[CB], const int (&mypos)[CB],
                                             int g, int lane, float scale2) {
  constexpr int BLK = FP8 ? 2048 : 4096, NLD = BLK / 1024;
  f32x4 S[CB][2];
#pragma unroll
  for (int pp = 0; pp < 2; pp++) {
    u32x4 raw[NLD];
#pragma unroll
    for (int c = 0; c < NLD; c++) raw[c] = *(const u32x4*)(kb + pp * BLK + c * 1024 + lane * 16);
#pragma unroll
    for (int cb = 0; cb < CB; cb++) S[cb][pp] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; c++) {
      const u32x4 kr = att_operand<FP8>(raw, c);
#pragma unroll
      for (int cb = 0; cb < CB; cb++)
        S[cb][pp] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kr),
                                                            __builtin_bit_cast(bf16x8, qreg[cb][c]),
                                                            S[cb][pp], 0, 0, 0);
    }
  }
  bf16x8 P[CB];
#pragma unroll
  for (int cb = 0; cb < CB; cb++) {
    bool vis[8];
    float mx = ATT_NEG;
#pragma unroll
    for (int i = 0; i < 8; i++) {
      vis[i] = !MASKED || (pg + (i >> 2)) * RL_PAGE + 4 * g + (i & 3) <= mypos[cb];
      mx = fmaxf(mx, vis[i] ? S[cb][i >> 2][i & 3] : ATT_NEG);
    }
    // m (in scaled units: score * scale2, scale2 > 0) is the reference point of the exponents, not
    // necessarily the running maximum: it only moves, to the column's maximum so far, when some
    // score of the wave lies more than kLazy above it.  Every term then stays below 2^kLazy, the
    // ratio acc / l does not depend on m, and the common case needs neither the reduction over
    // the column's four lanes nor a rescaling of the accumulators.
    constexpr float kLazy = 8.0f;
    if (__any(mx * scale2 > m[cb] + kLazy)) {
      mx = quad_max(mx);
      const float mn = fmaxf(m[cb], mx * scale2);
      const float alpha = exp2f(m[cb] - mn);
      l[cb] *= alpha;
#pragma unroll
      for (int j = 0; j < 8; j++)
#pragma unroll
        for (int i = 0; i < 4; i++) acc[cb][j][i] *= alpha;
      m[cb] = mn;
    }
    const float mn = m[cb];
    float p[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
      p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[cb][i >> 2][i & 3], scale2, -mn));
      if (MASKED) p[i] = vis[i] ? p[i] : 0.f;
    }
    l[cb] += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
    P[cb] = (bf16x8){(__bf16)p[0], (__bf16)p[1], (__bf16)p[2], (__bf16)p[3],
                     (__bf16)p[4], (__bf16)p[5], (__bf16)p[6], (__bf16)p[7]};
  }
  if constexpr (FP8) {
    u32x4 raw0[NLD], raw1[NLD];
#pragma unroll
    for (int c = 0; c < NLD; c++) {
      raw0[c] = *(const u32x4*)(vb + c * 1024 + lane * 16);
      raw1[c] = *(const u32x4*)(vb + BLK + c * 1024 + lane * 16);
    }
#pragma unroll
    for (int jb = 0; jb < 8; jb++) {
      uint32_t a0, b0, a1, b1;
      e4m3x4_to_bf16(raw0[jb >> 2][jb & 3], &a0, &b0);
      e4m3x4_to_bf16(raw1[jb >> 2][jb & 3], &a1, &b1);
      const bf16x8 vo = __builtin_bit_cast(bf16x8, ((u32x4){a0, b0, a1, b1}));
#pragma unroll
      for (int cb = 0; cb < CB; cb++)
        acc[cb][jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vo, P[cb], acc[cb][jb], 0, 0, 0);
    }
  } else {
    // the lane's 4 tokens of 16 output dims are 8 bytes in each page's block: two 8-byte reads
    // make the 32-key operand without any register shuffling
    uint2 v0[8], v1[8];
#pragma unroll
    for (int jb = 0; jb < 8; jb++) {
      v0[jb] = *(const uint2*)(vb + (jb >> 1) * 1024 + lane * 16 + (jb & 1) * 8);
      v1[jb] = *(const uint2*)(vb + BLK + (jb >> 1) * 1024 + lane * 16 + (jb & 1) * 8);
    }
#pragma unroll
    for (int jb = 0; jb < 8; jb++) {
      const bf16x8 vo = __builtin_bit_cast(bf16x8, ((u32x4){v0[jb].x, v0[jb].y, v1[jb].x, v1[jb].y}));
#pragma unroll
      for (int cb = 0; cb < CB; cb++)
        acc[cb][jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vo, P[cb], acc[cb][jb], 0, 0, 0);
    }
  }
}

// Chunked prefill with the pages staged through LDS: one workgroup per (item of up to
// 4 * CB * 16/G rows, kv head) as above, but a page's keys / values are fetched once per
// workgroup (not once per wave) into a double-buffered LDS stage of NP pages, in the pool's
// operand order, and the four waves read their operands from there (linear 16-byte reads, no bank
// conflicts).  Pages are consumed in pairs (prefill_pair).  One barrier per stage: the loads of
// stage s + 1 are issued before the barrier of stage s and written to the other buffer after the
// stage's arithmetic, which every wave can only reach once all waves have left stage s - 1.
// Page indices past the item's last page are clamped to it (their keys are masked: they lie
// behind every row of the item); the pool is cleared at load, so such blocks hold finite values.
template <int CB, bool FP8>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attention_prefill_lds_kernel(
    const bf16_t* __restrict__ q, const char* __restrict__ kpool, const char* __restrict__ vpool,
    const AttnItem* __restrict__ items, const int32_t* __restrict__ page_table,
    bf16_t* __restrict__ o, int nq, int nkv, int gshift, int pt_stride, float scale2) {
  constexpr int NP = 4;
  constexpr int BLK = FP8 ? 2048 : 4096;
  constexpr int STAGE = 2 * NP * BLK;            // NP key blocks, then NP value blocks
  constexpr int U = STAGE / 4096;                // 16-byte loads per thread and stage
  __shared__ __align__(16) char s_kv[2 * STAGE];
  const int item_idx = blockIdx.x / nkv;
  const AttnItem it = items[item_idx];
  const int kvh = blockIdx.x - item_idx * nkv;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 4, n = lane & 15, hq = n & ((1 << gshift) - 1);
  const int rpb = 16 >> gshift;                       // rows per column block
  const int wrow0 = wave * CB * rpb;                  // first row of this wave within the item
  const int wave_rows = min(it.nrows - wrow0, CB * rpb);
  const int pg1 = wave_rows > 0 ? (it.pos0 + wrow0 + wave_rows - 1) / RL_PAGE + 1 : 0;
  const int item_pg1 = (it.pos0 + it.nrows - 1) / RL_PAGE + 1;
  const int pglast = item_pg1 - 1;
  const int nst = (item_pg1 + NP - 1) / NP;
  const int32_t* pt = page_table + (size_t)it.slot * pt_stride;
  u32x4 qreg[CB][4];
  f32x4 acc[CB][8];
  float m[CB], l[CB];
  int mypos[CB];
#pragma unroll
  for (int cb = 0; cb < CB; cb++) {
    const int r = wrow0 + cb * rpb + (n >> gshift);
    // columns past the item's rows get position -1: every key of a masked pair is masked for them
    mypos[cb] = r < it.nrows ? it.pos0 + r : -1;
#pragma unroll
    for (int c = 0; c < 4; c++) {
      qreg[cb][c] = (u32x4){0u, 0u, 0u, 0u};
      if (r < it.nrows)
        qreg[cb][c] = *(const u32x4*)(q + ((size_t)(it.row0 + r) * nq + ((kvh << gshift) + hq)) * 128 + c * 32 + g * 8);
    }
#pragma unroll
    for (int j = 0; j < 8; j++) acc[cb][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    m[cb] = ATT_NEG;
    l[cb] = 0.f;
  }
  // pages that end at or before the wave's first row are visible to all of its rows: no masking
  const int full_pages = wave_rows > 0 ? (it.pos0 + wrow0 + 1) / RL_PAGE : 0;
  u32x4 stg[U];
  auto fetch = [&](int s) {
    int id[NP];
#pragma unroll
    for (int p = 0; p < NP; p++) id[p] = pt[min(s * NP + p, pglast)];
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int byte = u * 4096 + tid * 16;
      const int blk = byte / BLK, off = byte % BLK;
      const bool isv = blk >= NP;
      const int p = isv ? blk - NP : blk;
      int pid = id[0];
#pragma unroll
      for (int x = 1; x < NP; x++) pid = p == x ? id[x] : pid;
      const char* src = (isv ? vpool : kpool) + ((size_t)pid * nkv + kvh) * BLK + off;
      stg[u] = *(const u32x4*)src;
    }
  };
  auto stash = [&](int b) {
#pragma unroll
    for (int u = 0; u < U; u++) *(u32x4*)(s_kv + b * STAGE + u * 4096 + tid * 16) = stg[u];
  };
  if (nst > 0) {
    fetch(0);
    stash(0);
  }
  for (int s = 0; s < nst; s++) {
    if (s + 1 < nst) fetch(s + 1);
    __syncthreads();
    const char* buf = s_kv + (s & 1) * STAGE;
#pragma unroll
    for (int j = 0; j < NP / 2; j++) {
      const int pg = s * NP + 2 * j;
      const char* kb = buf + 2 * j * BLK;
      const char* vb = buf + (NP + 2 * j) * BLK;
      if (pg + 1 < full_pages)
        prefill_pair<CB, FP8, false>(kb, vb, pg, qreg, acc, m, l, mypos, g, lane, scale2);
      else if (pg < pg1)
        prefill_pair<CB, FP8, true>(kb, vb, pg, qreg, acc, m, l, mypos, g, lane, scale2);
    }
    if (s + 1 < nst) stash((s + 1) & 1);
  }
#pragma unroll
  for (int cb = 0; cb < CB; cb++) {
    const float lt = quad_sum(l[cb]);
    const int r = wrow0 + cb * rpb + (n >> gshift);
    if (r < it.nrows) {
      // acc[jb][i] is O[row r][head hq][d = 16 jb + 4 g + i]: four consecutive dims = one 8-byte store
      const float inv = 1.0f / lt;
      const size_t base = atile_off(it.row0 + r, ((kvh << gshift) + hq) * 128 + 4 * g, nq * 128);
#pragma unroll
      for (int jb = 0; jb < 8; jb++) {
        uint2 w;
        w.x = (uint32_t)f2bf(acc[cb][jb][0] * inv) | ((uint32_t)f2bf(acc[cb][jb][1] * inv) << 16);
        w.y = (uint32_t)f2bf(acc[cb][jb][2] * inv) | ((uint32_t)f2bf(acc[cb][jb][3] * inv) << 16);
        *(uint2*)(o + base + (size_t)jb * (4 * 64 * 8)) = w;
      }
    }
  }
}

// grid (n_merges, nkv), block 256: merge the parts of one (row, kv head) in a fixed order: the
// shared-prefix parts first (the row is row `sr` of those items), then the row's own parts.
__global__ __launch_bounds__(256) void attention_merge_kernel(const float* __restrict__ scratch,
                                                              const AttnMerge* __restrict__ merges,
                                                              bf16_t* __restrict__ o, int nq,
                                                              int nkv, int gshift) {
  const AttnMerge mg = merges[blockIdx.x];
  const int kvh = blockIdx.y, tid = threadIdx.x;
  const size_t stride = (size_t)nkv * (16 * 130);
  const int cn = tid >> 4, d0 = (tid & 15) * 8;
  if ((cn >> gshift) != 0) return;   // decode rows: one query row, columns 0 .. G-1
  const int total = mg.snparts + mg.nparts;
  const int scol = (mg.sr << gshift) + cn;
  // part w: slot and column holding this row's head cn
  auto src_of = [&](int w, int* col) -> const float* {
    const bool sh = w < mg.snparts;
    *col = sh ? scol : cn;
    const int slot = sh ? mg.sfirst + w : mg.first + (w - mg.snparts);
    return scratch + ((size_t)slot * nkv + kvh) * (16 * 130);
  };
  float mt = ATT_NEG;
  for (int w = 0; w < total; w++) {
    int col;
    const float* src = src_of(w, &col);
    mt = fmaxf(mt, src[16 * 128 + col]);
  }
  float L = 0.f, o8[8];
#pragma unroll
  for (int e = 0; e < 8; e++) o8[e] = 0.f;
  for (int w = 0; w < total; w++) {
    int col;
    const float* src = src_of(w, &col);
    const float f = exp2f(src[16 * 128 + col] - mt);
    L += f * src[16 * 128 + 16 + col];
    const float* a = src + (size_t)col * 128 + d0;
#pragma unroll
    for (int e = 0; e < 8; e++) o8[e] += f * a[e];
  }
  const float inv = 1.0f / L;
  uint32_t wv[4];
#pragma unroll
  for (int e = 0; e < 4; e++)
    wv[e] = (uint32_t)f2bf(o8[2 * e] * inv) | ((uint32_t)f2bf(o8[2 * e + 1] * inv) << 16);
  *(uint4*)(o + atile_off(mg.row, ((kvh << gshift) + cn) * 128 + d0, nq * 128)) =
      make_uint4(wv[0], wv[1], wv[2], wv[3]);
}

void launch_attention_mfma(hipStream_t s, const bf16_t* q, KvPool pool, const AttnItem* items,
                           int n_items, const AttnMerge* merges, int n_merges,
                           const int32_t* rowlist, const int32_t* page_table, bf16_t* o,
                           float* scratch, const ModelDims& md, bool prefill) {
  if (n_items <= 0) return;
  float scale2 = 1.4426950408889634f / sqrtf((float)md.d);
  int gshift = 0;
  while ((1 << gshift) < md.nq / md.nkv) gshift++;
  const char* kp = (const char*)pool.k;
  const char* vp = (const char*)pool.v;
  const dim3 grid(n_items * md.nkv);
  if (prefill) {
    if (md.kv_fp8)
      attention_prefill_lds_kernel<RL_PREFILL_CB, true><<<grid, 256, 0, s>>>(
          q, kp, vp, items, page_table, o, md.nq, md.nkv, gshift, md.max_pages_per_traj, scale2);
    else
      attention_prefill_lds_kernel<RL_PREFILL_CB, false><<<grid, 256, 0, s>>>(
          q, kp, vp, items, page_table, o, md.nq, md.nkv, gshift, md.max_pages_per_traj, scale2);
    return;
  }
  if (md.kv_fp8)
    attention_mfma_kernel<true><<<grid, 256, 0, s>>>(q, kp, vp, items, rowlist, page_table, o, scratch,
                                                     md.nq, md.nkv, gshift, md.max_pages_per_traj, scale2);
  else
    attention_mfma_kernel<false><<<grid, 256, 0, s>>>(q, kp, vp, items, rowlist, page_table, o, scratch,
                                                      md.nq, md.nkv, gshift, md.max_pages_per_traj, scale2);
  if (n_merges > 0)
    attention_merge_kernel<<<dim3(n_merges, md.nkv), 256, 0, s>>>(scratch, merges, o, md.nq, md.nkv,
                                                                  gshift);
}
