// fp16 MFMA GEMMs for gfx950 (wave64, v_mfma_f32_32x32x16_f16): the tiled projection kernel,
// the output projection fused with the row arg-max, and the small-M decoder-step kernel.
//
// C[M,N] = A[M,K] * Wt[N,K]^T.  Both operands are K-contiguous, so an MFMA fragment (8
// consecutive k of one row) is one 16-byte LDS read.  Weights are laid out as Wt at load time
// (the paper moves its transposes out of the matrix multiplications to the start of decoding,
// Sec. 3.3 "Graph Optimization").
//
// Tile: 128 x 128 x 64 per workgroup of 4 waves (2 x 2), each wave 64 x 64 = 2 x 2 MFMA blocks;
// the next K-slab is prefetched into registers while the current one is multiplied.  Workgroup
// ids are mapped to tiles XCD-aware: ids are dealt round-robin to the 8 XCDs (each with its own
// L2), so every XCD gets its own slice of the longer tile dimension and walks the shorter one
// fastest - an operand tile is then pulled into one L2 only.
//
// Split precision: an activation a is carried as head + tail, hi = fp16(a), lo = fp16(a - hi)
// (about 22 significant bits; the MFMA keeps fp16 subnormal inputs, so the tail needs no
// scaling).  Both halves are multiplied with the same weight fragment into one fp32
// accumulator: two MFMA passes instead of the 16x slower fp32 MFMA.  The greedy arg-max needs
// this: a single fp16 rounding of the decoder state flips about 1 % of sentences.
//   A_F16    A is one fp16 plane
//   A_PLANES A is two fp16 planes (head, tail) written by the producing kernel
//   A_F32    A is fp32 and is split while it is staged into LDS
#include "nt_kernels.h"

namespace nt {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_LD = BK + 8;  // halfs per LDS row: 144 B keeps 16-byte alignment and is bank-conflict free

// Accumulate the 128x128 tile at (m0, n0) over the whole K.
// acc[mb][nb][v] is C[row = wm*64 + mb*32 + (v/4)*8 + (lane/32)*4 + v%4][col = wn*64 + nb*32 + lane%32].
// Rows beyond M / N re-read the last valid row (never stored), which keeps the loads branch-free.
// SWAP exchanges the operand roles of the MFMA, which transposes every 32x32 block: then
// acc[mb][nb][v] is C[row = wm*64 + mb*32 + lane%32][col = wn*64 + nb*32 + (v/4)*8 + (lane/32)*4 + v%4],
// i.e. a lane owns one row and its registers run along the columns.
template <int AMODE, bool SWAP = false>
__device__ __forceinline__ void mainloop(const void *A, const void *A2, long lda, int M, const _Float16 *Wt, int N,
                                         int K, int m0, int n0, _Float16 *sAhi, _Float16 *sAlo, _Float16 *sB,
                                         floatx16 (&acc)[2][2], const int *row_map = nullptr) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, g = lane >> 5;
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;
  // registers holding the next K-slab
  constexpr int NRA = (AMODE == A_F16) ? 4 : 8;
  u32x4 ra[NRA], rb[4];  // native vectors: HIP's uint4 struct is not reliably kept in registers here
  // A rows of this thread's four fp16 chunks (optionally gathered through row_map)
  long arow[4];
  if constexpr (AMODE != A_F32) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int row = (tid + 256 * i) >> 3;
      const int m = (m0 + row < M) ? m0 + row : M - 1;
      arow[i] = (long)(row_map ? row_map[m] : m) * lda;
    }
  }
  auto load_slab = [&](int k0) {
    if constexpr (AMODE == A_F32) {
      const float *Af = (const float *)A;
#pragma unroll
      for (int i = 0; i < 8; i++) {
        const int c = tid + 256 * i, row = c >> 4, kc = c & 15;
        const int m = (m0 + row < M) ? m0 + row : M - 1;
        ra[i] = *(const u32x4 *)(Af + (long)m * lda + k0 + kc * 4);
      }
    } else {
      const _Float16 *Ah = (const _Float16 *)A, *Al = (const _Float16 *)A2;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int kc = (tid + 256 * i) & 7;
        ra[i] = *(const u32x4 *)(Ah + arow[i] + k0 + kc * 8);
        if constexpr (AMODE == A_PLANES) ra[NRA - 4 + i] = *(const u32x4 *)(Al + arow[i] + k0 + kc * 8);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
      const int n = (n0 + row < N) ? n0 + row : N - 1;
      rb[i] = *(const u32x4 *)(Wt + (long)n * K + k0 + kc * 8);
    }
  };
  auto store_slab = [&]() {
    if constexpr (AMODE == A_F32) {
#pragma unroll
      for (int i = 0; i < 8; i++) {
        const int c = tid + 256 * i, row = c >> 4, kc = c & 15;
        const float f[4] = {__uint_as_float(ra[i][0]), __uint_as_float(ra[i][1]), __uint_as_float(ra[i][2]),
                            __uint_as_float(ra[i][3])};
        half4 hi, lo;
#pragma unroll
        for (int j = 0; j < 4; j++) {
          hi[j] = (_Float16)f[j];
          lo[j] = (_Float16)(f[j] - (float)hi[j]);
        }
        *(half4 *)(sAhi + row * LDS_LD + kc * 4) = hi;
        *(half4 *)(sAlo + row * LDS_LD + kc * 4) = lo;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        *(u32x4 *)(sAhi + row * LDS_LD + kc * 8) = ra[i];
        if constexpr (AMODE == A_PLANES) *(u32x4 *)(sAlo + row * LDS_LD + kc * 8) = ra[NRA - 4 + i];
      }
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
      *(u32x4 *)(sB + row * LDS_LD + kc * 8) = rb[i];
    }
  };
  load_slab(0);
  const int nk = K / BK;
  for (int kt = 0; kt < nk; kt++) {
    __syncthreads();  // the previous slab (or the previous user of the LDS tiles) is done
    store_slab();
    if (kt + 1 < nk) load_slab((kt + 1) * BK);
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < BK / 16; ks++) {
      half8 a[2], al[2], b[2];
#pragma unroll
      for (int mb = 0; mb < 2; mb++) {
        const int off = (wm * 64 + mb * 32 + li) * LDS_LD + ks * 16 + g * 8;
        a[mb] = *(const half8 *)(sAhi + off);
        if constexpr (AMODE != A_F16) al[mb] = *(const half8 *)(sAlo + off);
      }
#pragma unroll
      for (int nb = 0; nb < 2; nb++) b[nb] = *(const half8 *)(sB + (wn * 64 + nb * 32 + li) * LDS_LD + ks * 16 + g * 8);
#pragma unroll
      for (int mb = 0; mb < 2; mb++)
#pragma unroll
        for (int nb = 0; nb < 2; nb++) {
          if constexpr (SWAP) {
            acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(b[nb], a[mb], acc[mb][nb], 0, 0, 0);
            if constexpr (AMODE != A_F16)
              acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(b[nb], al[mb], acc[mb][nb], 0, 0, 0);
          } else {
            acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[mb], b[nb], acc[mb][nb], 0, 0, 0);
            if constexpr (AMODE != A_F16)
              acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al[mb], b[nb], acc[mb][nb], 0, 0, 0);
          }
        }
    }
  }
}

// Epilogue of NB 32 x 32 accumulator blocks of one wave: block i has its origin at row mb0[i], column nb0[i] (both
// uniform over the wave); lane (g, li) holds, in acc[i][v], the element at row (v/4)*8 + g*4 + v%4, column li of it.
// When all blocks lie inside the matrix the code is straight-line: a block's 16 residual values are requested before
// the stores of the block before it, and every store is issued without waiting for the one before it.  (With a guard
// around each store the compiler waits for the memory counter to reach zero before every store, i.e. for the
// acknowledgement of the previous one.)  Addresses are a uniform 64-bit base plus a 32-bit lane offset.  Blocks that
// stick out of the matrix take the path that checks every element.
template <int NB, bool C_F32>
__device__ __forceinline__ void blocks_epilogue(const floatx16 *acc, const int *mb0, const int *nb0, int g, int li,
                                                bool inside, int M, int N, const GemmEpilogue &e) {
  constexpr int CE = C_F32 ? 4 : 2;
  auto finish = [&](float a, float bias, float sc, float r) -> float {
    float val = (a + bias) * sc;
    if (e.relu) val = fmaxf(val, 0.f);
    return val + r;
  };
  auto put = [&](char *at_, float val) {
    if (C_F32) {
      *(float *)at_ = val;
    } else {
      const _Float16 hi = (_Float16)val;
      *(_Float16 *)at_ = hi;
      if (e.dst_lo_offset) *((_Float16 *)at_ + e.dst_lo_offset) = (_Float16)(val - (float)hi);
    }
  };
  if (inside) {
    float bias[NB], sc[NB];
#pragma unroll
    for (int i = 0; i < NB; i++) {
      const int n = nb0[i] + li;
      bias[i] = e.bias ? e.bias[n] : 0.f;
      sc[i] = (n < e.scale_cols) ? e.scale : 1.f;
    }
    auto store_block = [&](int i, const float *res) {
      const bool first = nb0[i] < e.n_split;  // n_split is a multiple of 32: a block never straddles the destinations
      char *dst = (char *)(first ? e.dst0 : e.dst1);
      const long ld = first ? e.ld0 : e.ld1;
      char *dblock = dst + ((long)mb0[i] * ld + (first ? nb0[i] : nb0[i] - e.n_split)) * CE;
      unsigned dlane = (unsigned)((g * 4 * ld + li) * CE);
      asm volatile("" : "+v"(dlane));
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int r = (v >> 2) * 8 + (v & 3);
        put(dblock + (dlane + (unsigned)(r * ld * CE)), finish(acc[i][v], bias[i], sc[i], res ? res[v] : 0.f));
      }
    };
    if (e.resid) {
      float res[2][16];
      auto request = [&](int i) {
        const char *rblock = (const char *)e.resid + ((long)mb0[i] * e.ldr + nb0[i]) * 4;
        unsigned rlane = (unsigned)((g * 4 * e.ldr + li) * 4);
        asm volatile("" : "+v"(rlane));
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const int r = (v >> 2) * 8 + (v & 3);
          res[i & 1][v] = *(const float *)(rblock + (rlane + (unsigned)(r * e.ldr * 4)));
        }
      };
      request(0);
#pragma unroll
      for (int i = 0; i < NB; i++) {
        __builtin_amdgcn_sched_barrier(0);
        if (i + 1 < NB) request(i + 1);
        __builtin_amdgcn_sched_barrier(0);
        store_block(i, res[i & 1]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NB; i++) store_block(i, nullptr);
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < NB; i++) {
    const int n = nb0[i] + li;
    if (n >= N) continue;
    const float bias = e.bias ? e.bias[n] : 0.f;
    const float sc = (n < e.scale_cols) ? e.scale : 1.f;
    const bool first = n < e.n_split;
    char *dst = (char *)(first ? e.dst0 : e.dst1);
    const long ld = first ? e.ld0 : e.ld1;
    const int nc = first ? n : n - e.n_split;
#pragma unroll
    for (int v = 0; v < 16; v++) {
      const int m = mb0[i] + (v >> 2) * 8 + g * 4 + (v & 3);
      if (m >= M) continue;
      put(dst + ((long)m * ld + nc) * CE, finish(acc[i][v], bias, sc, e.resid ? e.resid[(long)m * e.ldr + n] : 0.f));
    }
  }
}

// Workgroup id -> (m tile, n tile), XCD-aware.  Returns false for the padding ids of the grid.
__device__ __forceinline__ bool tile_of(int id, int tiles_m, int tiles_n, int &mt, int &nt_) {
  const int xcd = id & 7, j = id >> 3;
  if (tiles_m >= tiles_n) {  // long M (encoder): an A tile stays in one L2, Wt is small
    mt = (j / tiles_n) * 8 + xcd;
    nt_ = j % tiles_n;
    return mt < tiles_m;
  }
  nt_ = (j / tiles_m) * 8 + xcd;  // long N (output projection): a Wt tile stays in one L2
  mt = j % tiles_m;
  return nt_ < tiles_n;
}
static int tile_grid(int tiles_m, int tiles_n) {
  return tiles_m >= tiles_n ? ((tiles_m + 7) / 8) * 8 * tiles_n : ((tiles_n + 7) / 8) * 8 * tiles_m;
}

template <int AMODE, bool C_F32>
__global__ __launch_bounds__(256) void gemm_kernel(const void *A, const void *A2, long lda, const _Float16 *Wt, int M,
                                                   int N, int K, GemmEpilogue e) {
  __shared__ __attribute__((aligned(16))) _Float16 sAhi[BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) _Float16 sAlo[AMODE != A_F16 ? BM * LDS_LD : 8];
  __shared__ __attribute__((aligned(16))) _Float16 sB[BN * LDS_LD];
  int mt, nt_;
  if (!tile_of(blockIdx.x, (M + BM - 1) / BM, (N + BN - 1) / BN, mt, nt_)) return;
  const int m0 = mt * BM, n0 = nt_ * BN;
  floatx16 acc[2][2];
  mainloop<AMODE>(A, A2, lda, M, Wt, N, K, m0, n0, sAhi, sAlo, sB, acc);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, g = lane >> 5;
  const int wmu = __builtin_amdgcn_readfirstlane(wm), wnu = __builtin_amdgcn_readfirstlane(wn);
  int mb0[4], nb0[4];
#pragma unroll
  for (int mb = 0; mb < 2; mb++)
#pragma unroll
    for (int nb = 0; nb < 2; nb++) {
      mb0[mb * 2 + nb] = m0 + wmu * 64 + mb * 32;
      nb0[mb * 2 + nb] = n0 + wnu * 64 + nb * 32;
    }
  const bool inside = m0 + wmu * 64 + 64 <= M && n0 + wnu * 64 + 64 <= N && e.n_split % 32 == 0;
  blocks_epilogue<4, C_F32>(&acc[0][0], mb0, nb0, g, li, inside, M, N, e);
}

// ---------------------------------------------------------------------------------------
// Mid-size variant: 64 x 64 tiles (4 waves, one 32 x 32 MFMA block each) with the K-slabs
// prefetched three deep into registers.  Used when the 128 x 128 grid would leave most of the
// 256 CUs idle (decoder projections with a few thousand rows, short encoder batches): four times
// the workgroups, and the deep prefetch takes the global-load latency out of the K loop.
// ---------------------------------------------------------------------------------------
constexpr int MID = 64, MID_PD = 3;

template <int AMODE, bool C_F32>
__global__ __launch_bounds__(256) void gemm_mid_kernel(const void *A, const void *A2, long lda, const _Float16 *Wt,
                                                       int M, int N, int K, GemmEpilogue e) {
  __shared__ __attribute__((aligned(16))) _Float16 sAhi[MID * LDS_LD];
  __shared__ __attribute__((aligned(16))) _Float16 sAlo[AMODE != A_F16 ? MID * LDS_LD : 8];
  __shared__ __attribute__((aligned(16))) _Float16 sB[MID * LDS_LD];
  int mt, nt_;
  if (!tile_of(blockIdx.x, (M + MID - 1) / MID, (N + MID - 1) / MID, mt, nt_)) return;
  const int m0 = mt * MID, n0 = nt_ * MID;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, g = lane >> 5;
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; v++) acc[v] = 0.f;
  // per slab and thread: fp32 A 64x64 -> 4 chunks of 16 B; fp16 planes 64x64 -> 2 chunks each; Wt 64x64 -> 2
  constexpr int NRA = (AMODE == A_F32) ? 4 : (AMODE == A_PLANES ? 4 : 2);
  u32x4 ra[MID_PD][NRA], rb[MID_PD][2];
  auto load_slab = [&](int slot, int k0) {
    if constexpr (AMODE == A_F32) {
      const float *Af = (const float *)A;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int c = tid + 256 * i, row = c >> 4, kc = c & 15;
        const int m = (m0 + row < M) ? m0 + row : M - 1;
        ra[slot][i] = *(const u32x4 *)(Af + (long)m * lda + k0 + kc * 4);
      }
    } else {
      const _Float16 *Ah = (const _Float16 *)A, *Al = (const _Float16 *)A2;
#pragma unroll
      for (int i = 0; i < 2; i++) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        const int m = (m0 + row < M) ? m0 + row : M - 1;
        ra[slot][i] = *(const u32x4 *)(Ah + (long)m * lda + k0 + kc * 8);
        if constexpr (AMODE == A_PLANES) ra[slot][NRA - 2 + i] = *(const u32x4 *)(Al + (long)m * lda + k0 + kc * 8);
      }
    }
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
      const int n = (n0 + row < N) ? n0 + row : N - 1;
      rb[slot][i] = *(const u32x4 *)(Wt + (long)n * K + k0 + kc * 8);
    }
  };
  auto store_slab = [&](int slot) {
    if constexpr (AMODE == A_F32) {
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int c = tid + 256 * i, row = c >> 4, kc = c & 15;
        half4 hi, lo;
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const float f = __uint_as_float(ra[slot][i][j]);
          hi[j] = (_Float16)f;
          lo[j] = (_Float16)(f - (float)hi[j]);
        }
        *(half4 *)(sAhi + row * LDS_LD + kc * 4) = hi;
        *(half4 *)(sAlo + row * LDS_LD + kc * 4) = lo;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 2; i++) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        *(u32x4 *)(sAhi + row * LDS_LD + kc * 8) = ra[slot][i];
        if constexpr (AMODE == A_PLANES) *(u32x4 *)(sAlo + row * LDS_LD + kc * 8) = ra[slot][NRA - 2 + i];
      }
    }
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
      *(u32x4 *)(sB + row * LDS_LD + kc * 8) = rb[slot][i];
    }
  };
  const int nk = K / BK;
#pragma unroll
  for (int p = 0; p < MID_PD; p++)
    if (p < nk) load_slab(p, p * BK);
  for (int kt = 0; kt < nk; kt += MID_PD) {
#pragma unroll
    for (int p = 0; p < MID_PD; p++) {  // unrolled so that the register slots are static
      if (kt + p < nk) {
        __syncthreads();
        store_slab(p);
        if (kt + p + MID_PD < nk) load_slab(p, (kt + p + MID_PD) * BK);
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < BK / 16; ks++) {
          const int offa = (wm * 32 + li) * LDS_LD + ks * 16 + g * 8, offb = (wn * 32 + li) * LDS_LD + ks * 16 + g * 8;
          const half8 a = *(const half8 *)(sAhi + offa), b = *(const half8 *)(sB + offb);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
          if constexpr (AMODE != A_F16) {
            const half8 al = *(const half8 *)(sAlo + offa);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, b, acc, 0, 0, 0);
          }
        }
      }
    }
  }
  const int mb0 = m0 + __builtin_amdgcn_readfirstlane(wm) * 32, nb0 = n0 + __builtin_amdgcn_readfirstlane(wn) * 32;
  const bool inside = mb0 + 32 <= M && nb0 + 32 <= N && e.n_split % 32 == 0;
  blocks_epilogue<1, C_F32>(&acc, &mb0, &nb0, g, li, inside, M, N, e);
}

hipError_t launch_gemm(int a_mode, bool c_f32, const void *A, const void *A_lo, long lda, const _Float16 *Wt, int M,
                       int N, int K, const GemmEpilogue &e, hipStream_t s, const _Float16 *Wp, bool tail) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (a_mode == A_PLANES && Wp && gemm_stream_supported(N, K) && e.n_split % 32 == 0)
    return launch_gemm_stream(c_f32, (const _Float16 *)A, (const _Float16 *)A_lo, lda, Wp, M, N, K, e, s, tail);
  if (a_mode == A_PLANES && Wp && c_f32 && gemm_stream_k_supported(N, K) && e.n_split % 32 == 0)
    return launch_gemm_stream_k(c_f32, (const _Float16 *)A, (const _Float16 *)A_lo, lda, Wp, M, N, K, e, s, tail);
  const int big_tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const bool mid = big_tiles < 2 * 256;  // fewer than two 128x128 tiles per CU: use the 64x64 variant
  dim3 grid(mid ? tile_grid((M + MID - 1) / MID, (N + MID - 1) / MID) : tile_grid((M + BM - 1) / BM, (N + BN - 1) / BN)),
      block(256);
#define NT_GEMM_CASE(MODE, CF)                                                                                  \
  if (a_mode == MODE && c_f32 == CF) {                                                                          \
    if (mid)                                                                                                    \
      hipLaunchKernelGGL((gemm_mid_kernel<MODE, CF>), grid, block, 0, s, A, A_lo, lda, Wt, M, N, K, e);         \
    else                                                                                                        \
      hipLaunchKernelGGL((gemm_kernel<MODE, CF>), grid, block, 0, s, A, A_lo, lda, Wt, M, N, K, e);             \
    return hipGetLastError();                                                                                   \
  }
  NT_GEMM_CASE(A_F16, false) NT_GEMM_CASE(A_F16, true) NT_GEMM_CASE(A_PLANES, false) NT_GEMM_CASE(A_PLANES, true)
  NT_GEMM_CASE(A_F32, false) NT_GEMM_CASE(A_F32, true)
#undef NT_GEMM_CASE
  return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------
// Output projection + arg-max (the log-softmax of the output layer is not needed for greedy
// search, Sec. 3.3 "Graph Optimization"; here the logits themselves never reach HBM either).
//
// Key = (order-preserving bits of the fp32 logit) << 32 | (0xFFFFFFFF - v): the maximum key is the
// largest logit and, among equal logits, the lowest id.  Max over keys is associative and
// commutative, so the result does not depend on the tiling: deterministic without atomics.
// ---------------------------------------------------------------------------------------
constexpr int VOCAB_TILES_TARGET_WGS = 1024;

static int vocab_tiles_per_wg(int M, int N) {
  int mt = (M + BM - 1) / BM, nt_ = (N + BN - 1) / BN;
  int tpw = (int)(((long)mt * nt_ + VOCAB_TILES_TARGET_WGS - 1) / VOCAB_TILES_TARGET_WGS);
  if (tpw < 1) tpw = 1;
  if (tpw > 10) tpw = 10;
  return tpw;
}

int vocab_argmax_partials_tiled(int M, int N) {
  int nt_ = (N + BN - 1) / BN, tpw = vocab_tiles_per_wg(M, N);
  return 2 * ((nt_ + tpw - 1) / tpw);
}

// Two variants of one kernel.
//  CERT = false ("exact"): logits from the head/tail plane pair of h.  Either every row m < M is
//    processed and per-strip partial keys go to pk[m * n_partials + p], or (row_map != nullptr) the
//    rows row_map[0 .. *count) are gathered and each result is folded into final_key[slot] with a
//    64-bit atomic max (order-independent, hence still deterministic).
//  CERT = true ("single pass"): logits from the head plane only; besides the partial keys the
//    runner-up logit of every strip goes to ps, so that the caller can certify the arg-max (see
//    argmax_select_kernel).
// Workgroup id -> (strip of vocabulary tiles, m slot), XCD-aware with the strips split over the XCDs;
// a workgroup walks m tiles m_slot, m_slot + m_par, ...
template <bool CERT>
__global__ __launch_bounds__(256) void vocab_argmax_kernel(const _Float16 *h, const _Float16 *h_lo, long ldh,
                                                           const _Float16 *Wt, int M, int N, int K, int tiles_per_wg,
                                                           int n_partials, int m_par, unsigned long long *pk, float *ps,
                                                           const int *row_map, const int *count,
                                                           unsigned long long *final_key) {
  __shared__ __attribute__((aligned(16))) _Float16 sAhi[BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) _Float16 sAlo[CERT ? 8 : BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) _Float16 sB[BN * LDS_LD];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, g = lane >> 5;
  const int strips = n_partials / 2;
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  const int strip = (j / m_par) * 8 + xcd, m_slot = j % m_par;
  if (strip >= strips) return;
  if (count) M = *count;  // number of gathered rows, decided on the device
  const int n_tiles = (N + BN - 1) / BN;
  for (int m0 = m_slot * BM; m0 < M; m0 += m_par * BM) {
    // The MFMA blocks are transposed (SWAP): a lane owns two rows (one per mb) and its accumulator
    // registers run along the vocabulary, so the reduction over the vocabulary stays inside the lane:
    // running largest logit, its column and the runner-up, over all tiles of the strip.
    float rmax[2] = {-INFINITY, -INFINITY}, rsec[2] = {-INFINITY, -INFINITY};
    int ridx[2] = {0, 0};
    for (int tt = 0; tt < tiles_per_wg; tt++) {
      const int tile = strip * tiles_per_wg + tt;
      if (tile >= n_tiles) break;  // uniform over the workgroup
      const int n0 = tile * BN;
      floatx16 acc[2][2];
      mainloop<CERT ? A_F16 : A_PLANES, true>(h, h_lo, ldh, M, Wt, N, K, m0, n0, sAhi, sAlo, sB, acc, row_map);
      const bool full = n0 + BN <= N;
#pragma unroll
      for (int mb = 0; mb < 2; mb++)
#pragma unroll
        for (int nb = 0; nb < 2; nb++)
#pragma unroll
          for (int v = 0; v < 16; v++) {  // columns ascend with (nb, v): on equal logits the lower column stays
            const int n = n0 + wn * 64 + nb * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
            const float val = (full || n < N) ? acc[mb][nb][v] : -INFINITY;
            if (CERT) rsec[mb] = fmaxf(rsec[mb], fminf(rmax[mb], val));
            const bool gt = val > rmax[mb];
            rmax[mb] = gt ? val : rmax[mb];
            ridx[mb] = gt ? n : ridx[mb];
          }
    }
#pragma unroll
    for (int mb = 0; mb < 2; mb++) {
      // the two lane groups hold interleaved columns of the same row: merge them
      unsigned long long key = (rmax[mb] == -INFINITY) ? 0ull : argmax_key(rmax[mb], ridx[mb]);
      float second = rsec[mb];
      const unsigned long long okey = shfl_xor_u64(key, 32);
      const float osec = __shfl_xor(second, 32, 64);
      const bool take = okey > key;
      const unsigned long long loser = take ? key : okey;
      if (CERT) second = fmaxf(fmaxf(second, osec), loser ? key_value(loser) : -INFINITY);
      key = take ? okey : key;
      const int m = m0 + wm * 64 + mb * 32 + li;
      if (g == 0 && m < M) {
        if (final_key) {
          atomicMax(final_key + m, key);
        } else {
          pk[(long)m * n_partials + strip * 2 + wn] = key;
          if (CERT) ps[(long)m * n_partials + strip * 2 + wn] = second;
        }
      }
    }
  }
}

hipError_t launch_vocab_argmax_tiled(const _Float16 *h, const _Float16 *h_lo, long ldh, const _Float16 *Wt, int M, int N,
                                     int K, unsigned long long *pk, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  const int tpw = vocab_tiles_per_wg(M, N), np = vocab_argmax_partials_tiled(M, N);
  const int tiles_m = (M + BM - 1) / BM, strips = np / 2;
  dim3 grid(((strips + 7) / 8) * 8 * tiles_m), block(256);
  hipLaunchKernelGGL(vocab_argmax_kernel<false>, grid, block, 0, s, h, h_lo, ldh, Wt, M, N, K, tpw, np, tiles_m, pk,
                     (float *)nullptr, (const int *)nullptr, (const int *)nullptr, (unsigned long long *)nullptr);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Certified single-pass arg-max.  With h = hi + lo, the head-only logit l'(v) = hi . w_v differs
// from the head+tail logit by at most |lo . w_v| <= ||lo|| * max_v ||w_v||.  If the head-only
// winner leads the runner-up by more than twice that bound (plus a little slack for the fp32
// accumulation order) it is also the winner of the head+tail logits, and the second MFMA pass is
// not needed.  The few rows that fail the test (about 2 % with flat random logits) are collected
// and recomputed with both planes by the gathered variant of the kernel above.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void argmax_select_kernel(const unsigned long long *pk, const float *ps, int n_partials,
                                                            int rows, const float *lo_norm, float w_norm_max,
                                                            int32_t *tok, int32_t *slot_of_row, int32_t *list,
                                                            int32_t *count, unsigned long long *final_key,
                                                            unsigned long long *need_mask) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  unsigned long long best = 0ull;
  float second = -INFINITY;
  for (int i = lane; i < n_partials; i += 64) {
    const unsigned long long k = pk[(long)r * n_partials + i];
    const float s2 = ps[(long)r * n_partials + i];
    const bool take = k > best;
    const unsigned long long loser = take ? best : k;
    second = fmaxf(fmaxf(second, s2), loser ? key_value(loser) : -INFINITY);
    best = take ? k : best;
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const unsigned long long ob = shfl_xor_u64(best, m);
    const float os = __shfl_xor(second, m, 64);
    const bool take = ob > best;
    const unsigned long long loser = take ? best : ob;
    second = fmaxf(fmaxf(second, os), loser ? key_value(loser) : -INFINITY);
    best = take ? ob : best;
  }
  const float gap = key_value(best) - second;
  const float bound = 2.f * lo_norm[r] * w_norm_max + 1e-4f;
  // Ranges of the vocabulary (one per partial) that can hold the arg-max of the head+tail logits: a head-only
  // logit more than `bound` below the best one cannot win.  Bit p of the mask stands for partial p (up to 64).
  unsigned long long mask = 0ull;
  if (n_partials <= 64) {
    const float floor_ = key_value(best) - bound;
    const bool cand = lane < n_partials && pk[(long)r * n_partials + lane] != 0ull &&
                      key_value(pk[(long)r * n_partials + lane]) >= floor_;
    mask = __ballot(cand);
  } else {
    mask = ~0ull;
  }
  if (lane != 0) return;
  tok[r] = (int32_t)(0xFFFFFFFFu - (unsigned int)best);
  if (gap > bound) {
    slot_of_row[r] = -1;
  } else {
    const int sl = atomicAdd(count, 1);  // which slot a row gets does not affect its result
    slot_of_row[r] = sl;
    list[sl] = r;
    final_key[sl] = 0ull;
    need_mask[sl] = mask;
  }
}

hipError_t launch_argmax_select(const unsigned long long *pk, const float *ps, int n_partials, int M, const float *lo_norm,
                                float w_norm_max, int32_t *tok, int32_t *slot_of_row, int32_t *list, int32_t *count,
                                unsigned long long *final_key, unsigned long long *need_mask, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  hipLaunchKernelGGL(argmax_select_kernel, dim3((M + 3) / 4), dim3(256), 0, s, pk, ps, n_partials, M, lo_norm, w_norm_max,
                     tok, slot_of_row, list, count, final_key, need_mask);
  return hipGetLastError();
}

hipError_t launch_vocab_argmax_certified_tiled(const _Float16 *h, const _Float16 *h_lo, long ldh, const _Float16 *Wt, int M,
                                               int N, int K, const float *lo_norm, float w_norm_max,
                                               unsigned long long *pk, float *ps, int32_t *tok, int32_t *slot_of_row,
                                               int32_t *list, int32_t *count, unsigned long long *final_key,
                                               unsigned long long *need_mask, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  const int tpw = vocab_tiles_per_wg(M, N), np = vocab_argmax_partials_tiled(M, N);
  const int tiles_m = (M + BM - 1) / BM, strips = np / 2;
  hipLaunchKernelGGL(vocab_argmax_kernel<true>, dim3(((strips + 7) / 8) * 8 * tiles_m), dim3(256), 0, s, h, h_lo, ldh, Wt,
                     M, N, K, tpw, np, tiles_m, pk, ps, (const int *)nullptr, (const int *)nullptr,
                     (unsigned long long *)nullptr);
  hipError_t e = launch_argmax_select(pk, ps, np, M, lo_norm, w_norm_max, tok, slot_of_row, list, count, final_key,
                                      need_mask, s);
  if (e != hipSuccess) return e;
  // recompute of the uncertified rows: one vocabulary tile per workgroup, every workgroup walks all
  // gathered m tiles (normally one); the row count is read on the device
  const int n_tiles = (N + BN - 1) / BN;
  hipLaunchKernelGGL(vocab_argmax_kernel<false>, dim3(((n_tiles + 7) / 8) * 8), dim3(256), 0, s, h, h_lo, ldh, Wt, M, N, K,
                     1, 2 * n_tiles, 1, (unsigned long long *)nullptr, (float *)nullptr, (const int *)list,
                     (const int *)count, final_key);
  return hipGetLastError();
}

}  // namespace nt

// ---------------------------------------------------------------------------------------
// Skinny GEMM for the decoder step (M = active rows, a few tens to a few hundreds).
//
// At these sizes a projection moves ~1 MB and the tiled kernel above spends its time in a chain
// of dependent K-slab loads on a handful of workgroups.  Here a workgroup owns a 32 x 32 output
// tile and issues the loads of its whole operand panel (32 rows of A and of Wt over KC columns)
// at once: one memory round trip, every lane with 24 independent 16-byte loads in flight, and
// (M/32)*(N/32) workgroups instead of (M/128)*(N/128).  The four waves split K, multiply their
// quarter with split-precision MFMAs and the partial tiles are summed through LDS in a fixed
// order (deterministic).
//
// Optional prologue: A = LayerNorm(A) with fp32 statistics (needs K == KC: the whole row is in
// the panel), which removes the separate LayerNorm launches of the decoder step.
// ---------------------------------------------------------------------------------------
namespace nt {

template <int KC>
struct SkinnyCfg {
  static constexpr int LD = KC + 8;                       // halfs per LDS row
  static constexpr int PANEL = 32 * LD;                   // halfs per operand panel
  static constexpr size_t LDS = (size_t)3 * PANEL * 2 + 4 * 32 * 33 * 4;
};

__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

template <int KC, bool C_F32>
__global__ __launch_bounds__(256) void skinny_gemm_kernel(const float *A, long lda, const _Float16 *Wt, int M, int N,
                                                          int K, const float *ln_g, const float *ln_b, LnEps ln_eps,
                                                          GemmEpilogue e) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_sk[];
  using Cfg = SkinnyCfg<KC>;
  constexpr int LD = Cfg::LD;
  _Float16 *sAhi = (_Float16 *)smem_sk, *sAlo = sAhi + Cfg::PANEL, *sW = sAlo + Cfg::PANEL;
  float *sRed = (float *)(sW + Cfg::PANEL);  // [4][32][33]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, g = lane >> 5;
  const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  constexpr int CPL = KC / 256;  // float4 chunks per lane per row (wave covers a row: 64 lanes x 4 floats x CPL)

  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; v++) acc[v] = 0.f;

  for (int k0 = 0; k0 < K; k0 += KC) {
    // ---- issue every load of the panel: wave w owns rows 8w .. 8w+7 of A ----
    float4 ra[8][CPL];
#pragma unroll
    for (int r = 0; r < 8; r++) {
      const int m = m0 + wave * 8 + r;
#pragma unroll
      for (int c = 0; c < CPL; c++)
        ra[r][c] = (m < M) ? *(const float4 *)(A + (long)m * lda + k0 + c * 256 + lane * 4) : make_float4(0, 0, 0, 0);
    }
    uint4 rw[KC / 64];
#pragma unroll
    for (int i = 0; i < KC / 64; i++) {
      const int c = tid + 256 * i, row = c / (KC / 8), kc = c % (KC / 8);
      const int n = n0 + row;
      rw[i] = (n < N) ? *(const uint4 *)(Wt + (long)n * K + k0 + kc * 8) : make_uint4(0, 0, 0, 0);
    }
    if (k0 > 0) __syncthreads();  // previous panel fully consumed
    // ---- optional LayerNorm of the rows, then head/tail split into LDS ----
    float4 gg[CPL], bb[CPL];
    if (ln_g) {
#pragma unroll
      for (int c = 0; c < CPL; c++) {
        gg[c] = *(const float4 *)(ln_g + c * 256 + lane * 4);
        bb[c] = *(const float4 *)(ln_b + c * 256 + lane * 4);
      }
    }
#pragma unroll
    for (int r = 0; r < 8; r++) {
      if (ln_g) {
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < CPL; c++) s += ra[r][c].x + ra[r][c].y + ra[r][c].z + ra[r][c].w;
        const float mean = wave_sum_f(s) / (float)KC;
        float q = 0.f;
#pragma unroll
        for (int c = 0; c < CPL; c++) {
          float4 &x = ra[r][c];
          x.x -= mean; x.y -= mean; x.z -= mean; x.w -= mean;
          q += ln_term(x.x, ln_eps.l1) + ln_term(x.y, ln_eps.l1) + ln_term(x.z, ln_eps.l1) + ln_term(x.w, ln_eps.l1);
        }
        const float rstd = ln_rscale(wave_sum_f(q) / (float)KC, ln_eps);
#pragma unroll
        for (int c = 0; c < CPL; c++) {
          float4 &x = ra[r][c];
          x.x = gg[c].x * (x.x * rstd) + bb[c].x;
          x.y = gg[c].y * (x.y * rstd) + bb[c].y;
          x.z = gg[c].z * (x.z * rstd) + bb[c].z;
          x.w = gg[c].w * (x.w * rstd) + bb[c].w;
        }
      }
#pragma unroll
      for (int c = 0; c < CPL; c++) {
        const float f[4] = {ra[r][c].x, ra[r][c].y, ra[r][c].z, ra[r][c].w};
        half4 hi, lo;
#pragma unroll
        for (int j = 0; j < 4; j++) {
          hi[j] = (_Float16)f[j];
          lo[j] = (_Float16)(f[j] - (float)hi[j]);
        }
        const int off = (wave * 8 + r) * LD + c * 256 + lane * 4;
        *(half4 *)(sAhi + off) = hi;
        *(half4 *)(sAlo + off) = lo;
      }
    }
#pragma unroll
    for (int i = 0; i < KC / 64; i++) {
      const int c = tid + 256 * i, row = c / (KC / 8), kc = c % (KC / 8);
      *(uint4 *)(sW + row * LD + kc * 8) = rw[i];
    }
    __syncthreads();
    // ---- wave w multiplies its quarter of the panel ----
#pragma unroll
    for (int ks = 0; ks < KC / 64; ks++) {
      const int off = li * LD + wave * (KC / 4) + ks * 16 + g * 8;
      const half8 a = *(const half8 *)(sAhi + off), al = *(const half8 *)(sAlo + off), b = *(const half8 *)(sW + off);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, b, acc, 0, 0, 0);
    }
  }
  // ---- sum the four K-quarters in a fixed order, then the epilogue ----
#pragma unroll
  for (int v = 0; v < 16; v++) {
    const int row = (v >> 2) * 8 + g * 4 + (v & 3);
    sRed[(wave * 32 + row) * 33 + li] = acc[v];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; j++) {
    const int idx = tid + 256 * j, row = idx >> 5, col = idx & 31;
    const int m = m0 + row, n = n0 + col;
    if (m >= M || n >= N) continue;
    float val = sRed[(0 * 32 + row) * 33 + col] + sRed[(1 * 32 + row) * 33 + col] + sRed[(2 * 32 + row) * 33 + col] +
                sRed[(3 * 32 + row) * 33 + col];
    if (e.bias) val += e.bias[n];
    if (n < e.scale_cols) val *= e.scale;
    if (e.relu) val = fmaxf(val, 0.f);
    if (e.resid) val += e.resid[(long)m * e.ldr + n];
    const bool first = n < e.n_split;
    char *dst = (char *)(first ? e.dst0 : e.dst1);
    const long ld = first ? e.ld0 : e.ld1;
    const int nc = first ? n : n - e.n_split;
    if (C_F32)
      ((float *)dst)[(long)m * ld + nc] = val;
    else
      ((_Float16 *)dst)[(long)m * ld + nc] = (_Float16)val;
  }
}

template <int KC>
static hipError_t skinny_launch(const float *A, long lda, const _Float16 *Wt, int M, int N, int K, const float *ln_g,
                                const float *ln_b, LnEps ln_eps, const GemmEpilogue &e, hipStream_t s) {
  static bool configured = false;
  const size_t lds = SkinnyCfg<KC>::LDS;
  if (!configured) {
    hipError_t err = hipFuncSetAttribute((const void *)skinny_gemm_kernel<KC, true>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err != hipSuccess) return err;
    configured = true;
  }
  dim3 grid((N + 31) / 32, (M + 31) / 32), block(256);
  hipLaunchKernelGGL((skinny_gemm_kernel<KC, true>), grid, block, lds, s, A, lda, Wt, M, N, K, ln_g, ln_b, ln_eps, e);
  return hipGetLastError();
}

bool skinny_gemm_supported(int K, bool with_ln) {
  if (with_ln) return K == 256 || K == 512;
  return K % 256 == 0;
}

hipError_t launch_skinny_gemm(const float *A, long lda, const _Float16 *Wt, int M, int N, int K, const float *ln_g,
                              const float *ln_b, LnEps ln_eps, const GemmEpilogue &e, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (K % 512 == 0) return skinny_launch<512>(A, lda, Wt, M, N, K, ln_g, ln_b, ln_eps, e, s);
  if (K % 256 == 0) return skinny_launch<256>(A, lda, Wt, M, N, K, ln_g, ln_b, ln_eps, e, s);
  return hipErrorInvalidValue;
}

}  // namespace nt
