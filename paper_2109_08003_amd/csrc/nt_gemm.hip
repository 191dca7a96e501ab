// fp16 MFMA GEMM for gfx950 (wave64, v_mfma_f32_32x32x16_f16) and the output projection fused
// with the row arg-max.
//
// C[M,N] = A[M,K] * Wt[N,K]^T.  Both operands are K-contiguous, so an MFMA fragment (8
// consecutive k of one row) is one 16-byte LDS read.  Weights are laid out as Wt at load time
// (the paper moves its transposes out of the matrix multiplications to the start of decoding,
// Sec. 3.3 "Graph Optimization").
//
// Tile: 128 x 128 x 64 per workgroup of 4 waves (2 x 2), each wave 64 x 64 = 2 x 2 MFMA blocks.
// Global -> register prefetch of the next K-slab overlaps the MFMAs of the current one.
//
// fp32 A operand ("split" mode, used on the decoder side): a = hi + lo with hi = fp16(a) and
// lo = fp16((a - hi) * 2^11); two MFMA passes share the weight fragment and accumulate
// separately, result = acc_hi + acc_lo * 2^-11.  The tail is pre-scaled so that it stays in
// fp16's normal range.  This keeps ~22 bits of the activations at fp16 MFMA rate, which the
// greedy arg-max needs: a single fp16 rounding of the decoder state flips ~1 % of sentences.
#include "nt_kernels.h"

namespace nt {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_LD = BK + 8;  // halfs per LDS row: 144 B, keeps 16-byte alignment, spreads banks
constexpr float LO_SCALE = 2048.f, LO_INV = 1.f / 2048.f;

template <bool A_F32>
struct Tile {
  // registers holding the next K-slab
  uint4 ra[A_F32 ? 8 : 4];
  uint4 rb[4];
};

template <bool A_F32>
__device__ __forceinline__ void load_slab(Tile<A_F32> &t, const void *A, long lda, int M, const _Float16 *Wt,
                                          int N, int K, int m0, int n0, int k0, int tid) {
  if (A_F32) {
    const float *Af = (const float *)A;
#pragma unroll
    for (int i = 0; i < 8; i++) {
      int c = tid + 256 * i, row = c >> 4, kc = c & 15;
      int m = m0 + row;
      t.ra[i] = (m < M) ? *(const uint4 *)(Af + (long)m * lda + k0 + kc * 4) : make_uint4(0, 0, 0, 0);
    }
  } else {
    const _Float16 *Ah = (const _Float16 *)A;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      int c = tid + 256 * i, row = c >> 3, kc = c & 7;
      int m = m0 + row;
      t.ra[i] = (m < M) ? *(const uint4 *)(Ah + (long)m * lda + k0 + kc * 8) : make_uint4(0, 0, 0, 0);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int c = tid + 256 * i, row = c >> 3, kc = c & 7;
    int n = n0 + row;
    t.rb[i] = (n < N) ? *(const uint4 *)(Wt + (long)n * K + k0 + kc * 8) : make_uint4(0, 0, 0, 0);
  }
}

template <bool A_F32>
__device__ __forceinline__ void store_slab(const Tile<A_F32> &t, _Float16 *sAhi, _Float16 *sAlo, _Float16 *sB,
                                           int tid) {
  if (A_F32) {
#pragma unroll
    for (int i = 0; i < 8; i++) {
      int c = tid + 256 * i, row = c >> 4, kc = c & 15;
      float f[4];
      *(uint4 *)f = t.ra[i];
      half4 hi, lo;
#pragma unroll
      for (int j = 0; j < 4; j++) {
        hi[j] = (_Float16)f[j];
        lo[j] = (_Float16)((f[j] - (float)hi[j]) * LO_SCALE);
      }
      *(half4 *)(sAhi + row * LDS_LD + kc * 4) = hi;
      *(half4 *)(sAlo + row * LDS_LD + kc * 4) = lo;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      int c = tid + 256 * i, row = c >> 3, kc = c & 7;
      *(uint4 *)(sAhi + row * LDS_LD + kc * 8) = t.ra[i];
    }
  }
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int c = tid + 256 * i, row = c >> 3, kc = c & 7;
    *(uint4 *)(sB + row * LDS_LD + kc * 8) = t.rb[i];
  }
}

// Accumulate the 128x128 tile at (m0, n0) over the whole K into acc (and acc_lo in split mode).
// acc[mb][nb][v] is C[row = wm*64 + mb*32 + (v/4)*8 + (lane/32)*4 + v%4][col = wn*64 + nb*32 + lane%32].
template <bool A_F32>
__device__ __forceinline__ void mainloop(const void *A, long lda, int M, const _Float16 *Wt, int N, int K, int m0,
                                         int n0, _Float16 *sAhi, _Float16 *sAlo, _Float16 *sB,
                                         floatx16 (&acc)[2][2], floatx16 (&acc_lo)[2][2]) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, g = lane >> 5;
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        acc[i][j][v] = 0.f;
        if (A_F32) acc_lo[i][j][v] = 0.f;
      }
  Tile<A_F32> t;
  load_slab<A_F32>(t, A, lda, M, Wt, N, K, m0, n0, 0, tid);
  __syncthreads();  // previous users of the LDS tiles are done
  store_slab<A_F32>(t, sAhi, sAlo, sB, tid);
  __syncthreads();
  const int nk = K / BK;
  for (int kt = 0; kt < nk; kt++) {
    if (kt + 1 < nk) load_slab<A_F32>(t, A, lda, M, Wt, N, K, m0, n0, (kt + 1) * BK, tid);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ks++) {
      half8 a[2], al[2], b[2];
#pragma unroll
      for (int mb = 0; mb < 2; mb++) {
        int off = (wm * 64 + mb * 32 + li) * LDS_LD + ks * 16 + g * 8;
        a[mb] = *(const half8 *)(sAhi + off);
        if (A_F32) al[mb] = *(const half8 *)(sAlo + off);
      }
#pragma unroll
      for (int nb = 0; nb < 2; nb++) b[nb] = *(const half8 *)(sB + (wn * 64 + nb * 32 + li) * LDS_LD + ks * 16 + g * 8);
#pragma unroll
      for (int mb = 0; mb < 2; mb++)
#pragma unroll
        for (int nb = 0; nb < 2; nb++) {
          acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[mb], b[nb], acc[mb][nb], 0, 0, 0);
          if (A_F32) acc_lo[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al[mb], b[nb], acc_lo[mb][nb], 0, 0, 0);
        }
    }
    __syncthreads();
    if (kt + 1 < nk) {
      store_slab<A_F32>(t, sAhi, sAlo, sB, tid);
      __syncthreads();
    }
  }
}

template <bool A_F32, bool C_F32>
__global__ __launch_bounds__(256) void gemm_kernel(const void *A, long lda, const _Float16 *Wt, int M, int N, int K,
                                                   GemmEpilogue e) {
  __shared__ __attribute__((aligned(16))) _Float16 sAhi[BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) _Float16 sAlo[A_F32 ? BM * LDS_LD : 8];
  __shared__ __attribute__((aligned(16))) _Float16 sB[BN * LDS_LD];
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  floatx16 acc[2][2], acc_lo[2][2];
  mainloop<A_F32>(A, lda, M, Wt, N, K, m0, n0, sAhi, sAlo, sB, acc, acc_lo);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, g = lane >> 5;
#pragma unroll
  for (int nb = 0; nb < 2; nb++) {
    const int n = n0 + wn * 64 + nb * 32 + li;
    if (n >= N) continue;
    const float bias = e.bias ? e.bias[n] : 0.f;
    const float sc = (n < e.scale_cols) ? e.scale : 1.f;
    const bool first = n < e.n_split;
    char *dst = (char *)(first ? e.dst0 : e.dst1);
    const long ld = first ? e.ld0 : e.ld1;
    const int nc = first ? n : n - e.n_split;
#pragma unroll
    for (int mb = 0; mb < 2; mb++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int m = m0 + wm * 64 + mb * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
        if (m >= M) continue;
        float val = acc[mb][nb][v];
        if (A_F32) val += acc_lo[mb][nb][v] * LO_INV;
        val = (val + bias) * sc;
        if (e.relu) val = fmaxf(val, 0.f);
        if (e.resid) val += e.resid[(long)m * e.ldr + n];
        if (C_F32)
          ((float *)dst)[(long)m * ld + nc] = val;
        else
          ((_Float16 *)dst)[(long)m * ld + nc] = (_Float16)val;
      }
  }
}

hipError_t launch_gemm(bool a_f32, bool c_f32, const void *A, long lda, const _Float16 *Wt, int M, int N, int K,
                       const GemmEpilogue &e, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM), block(256);
  if (a_f32 && c_f32)
    hipLaunchKernelGGL((gemm_kernel<true, true>), grid, block, 0, s, A, lda, Wt, M, N, K, e);
  else if (!a_f32 && c_f32)
    hipLaunchKernelGGL((gemm_kernel<false, true>), grid, block, 0, s, A, lda, Wt, M, N, K, e);
  else if (!a_f32 && !c_f32)
    hipLaunchKernelGGL((gemm_kernel<false, false>), grid, block, 0, s, A, lda, Wt, M, N, K, e);
  else
    hipLaunchKernelGGL((gemm_kernel<true, false>), grid, block, 0, s, A, lda, Wt, M, N, K, e);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Output projection + arg-max (the log-softmax of the output layer is not needed for greedy
// search, Sec. 3.3 "Graph Optimization"; here the logits themselves never reach HBM either).
//
// Key = (order-preserving bits of the fp32 logit) << 32 | (0xFFFFFFFF - v): the maximum key is the
// largest logit and, among equal logits, the lowest id.  Max over keys is associative and
// commutative, so the result does not depend on the tiling: deterministic without atomics.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long argmax_key(float val, int v) {
  unsigned int b = __float_as_uint(val);
  b = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
  return ((unsigned long long)b << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned int)v);
}

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long x, int mask) {
  unsigned int lo = (unsigned int)x, hi = (unsigned int)(x >> 32);
  lo = __shfl_xor(lo, mask, 64);
  hi = __shfl_xor(hi, mask, 64);
  return ((unsigned long long)hi << 32) | lo;
}

template <int HALF>
__device__ __forceinline__ void butterfly_step(unsigned long long (&k)[32], int lane) {
  const bool upper = (lane & HALF) != 0;
#pragma unroll
  for (int i = 0; i < HALF; i++) {
    unsigned long long a = k[i], b = k[i + HALF];
    unsigned long long send = upper ? a : b, keep = upper ? b : a;
    unsigned long long recv = shfl_xor_u64(send, HALF);
    k[i] = keep > recv ? keep : recv;
  }
}

constexpr int VOCAB_TILES_TARGET_WGS = 1024;

static int vocab_tiles_per_wg(int M, int N) {
  int mt = (M + BM - 1) / BM, nt_ = (N + BN - 1) / BN;
  int tpw = (int)(((long)mt * nt_ + VOCAB_TILES_TARGET_WGS - 1) / VOCAB_TILES_TARGET_WGS);
  if (tpw < 1) tpw = 1;
  if (tpw > 8) tpw = 8;
  return tpw;
}

int vocab_argmax_partials(int M, int N) {
  int nt_ = (N + BN - 1) / BN, tpw = vocab_tiles_per_wg(M, N);
  return 2 * ((nt_ + tpw - 1) / tpw);
}

__global__ __launch_bounds__(256) void vocab_argmax_kernel(const float *h, long ldh, const _Float16 *Wt, int M, int N,
                                                           int K, int tiles_per_wg, int n_partials,
                                                           unsigned long long *pk) {
  __shared__ __attribute__((aligned(16))) _Float16 sAhi[BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) _Float16 sAlo[BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) _Float16 sB[BN * LDS_LD];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, g = lane >> 5;
  const int m0 = blockIdx.y * BM;
  const int n_tiles = (N + BN - 1) / BN;
  unsigned long long best = 0ull;
  for (int tt = 0; tt < tiles_per_wg; tt++) {
    const int tile = blockIdx.x * tiles_per_wg + tt;
    if (tile >= n_tiles) break;  // uniform over the workgroup
    const int n0 = tile * BN;
    floatx16 acc[2][2], acc_lo[2][2];
    mainloop<true>(h, ldh, M, Wt, N, K, m0, n0, sAhi, sAlo, sB, acc, acc_lo);
    unsigned long long keys[32];
#pragma unroll
    for (int mb = 0; mb < 2; mb++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        unsigned long long k = 0ull;
#pragma unroll
        for (int nb = 0; nb < 2; nb++) {
          const int n = n0 + wn * 64 + nb * 32 + li;
          const float val = acc[mb][nb][v] + acc_lo[mb][nb][v] * LO_INV;
          const unsigned long long c = (n < N) ? argmax_key(val, n) : 0ull;
          k = c > k ? c : k;
        }
        keys[mb * 16 + v] = k;
      }
    // reduce over the 32 column lanes; afterwards lane li holds slot li (mb = li/16, v = li%16)
    butterfly_step<16>(keys, lane);
    butterfly_step<8>(keys, lane);
    butterfly_step<4>(keys, lane);
    butterfly_step<2>(keys, lane);
    butterfly_step<1>(keys, lane);
    best = keys[0] > best ? keys[0] : best;
  }
  const int mb = li >> 4, v = li & 15;
  const int m = m0 + wm * 64 + mb * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
  if (m < M) pk[(long)m * n_partials + blockIdx.x * 2 + wn] = best;
}

hipError_t launch_vocab_argmax(const float *h, long ldh, const _Float16 *Wt, int M, int N, int K,
                               unsigned long long *pk, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  const int tpw = vocab_tiles_per_wg(M, N), np = vocab_argmax_partials(M, N);
  dim3 grid(np / 2, (M + BM - 1) / BM), block(256);
  hipLaunchKernelGGL(vocab_argmax_kernel, grid, block, 0, s, h, ldh, Wt, M, N, K, tpw, np, pk);
  return hipGetLastError();
}

}  // namespace nt
