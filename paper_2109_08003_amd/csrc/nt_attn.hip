// Attention kernels for gfx950.
//
// enc_attention: padded-batch encoder self-attention, one workgroup per (32 queries, head,
// sentence).  Scores Q K^T and the product P V run on v_mfma_f32_32x32x16_f16; the softmax is
// fp32 in LDS (the paper converts to full precision around the softmax, Sec. 3.1 "FP16
// Inference"; the 1/sqrt(d_k) scale was already applied to the query by the projection).
// Keys beyond the sentence length get -inf before the row maximum, hence weight exactly 0.
//
// attn_decode: one query per (row, head) against a key/value cache - the incremental decoder's
// self-attention (fp32 cache, t+1 keys) and cross-attention (fp16 cache, len keys).  Pure HBM
// streaming: every key and value is read once, coalesced 16/32 bytes per lane, with an online
// softmax in registers and a butterfly merge across key groups and waves.
//
// Relative position keys (Sec. 2.1, clip distance c): score_ij += q_i . rk[clamp(j-i,-c,c)+c].
#include <math.h>

#include <type_traits>

#include "nt_kernels.h"

namespace nt {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------------------
// encoder attention
// ---------------------------------------------------------------------------------------
constexpr int QT = 32;        // queries per workgroup
constexpr int MAX_CLIP = 16;  // relative-position clip distance supported
constexpr float LO_SCALE = 2048.f, LO_INV = 1.f / 2048.f;

static inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

// F32 mode keeps q, k, v, the probabilities and the context at ~22 bits through the fp16 MFMA
// units: every operand x is split into hi = fp16(x) and lo = fp16((x - hi) * 2^11), and a
// product a.b is evaluated as a_hi.b_hi + (a_lo.b_hi + a_hi.b_lo) * 2^-11 with the two parts in
// separate fp32 accumulators.
size_t enc_attention_lds_bytes(int S, int dh, bool f32) {
  const int SP = round_up(S, 32), n = f32 ? 2 : 1;
  return (size_t)n * QT * (dh + 8) * 2 + (size_t)QT * (SP + 1) * 4 + (size_t)n * QT * (SP + 8) * 2 +
         (size_t)QT * (2 * MAX_CLIP + 1) * 4;
}

__device__ __forceinline__ void split8(const float *f, half8 &hi, half8 &lo) {
#pragma unroll
  for (int e = 0; e < 8; e++) {
    hi[e] = (_Float16)f[e];
    lo[e] = (_Float16)((f[e] - (float)hi[e]) * LO_SCALE);
  }
}

template <int DH, bool F32>
__global__ __launch_bounds__(256) void enc_attention_kernel(const void *qkv_, const int32_t *len, void *ctx_,
                                                            long ctx_lo_offset, int S, int d, const float *rk,
                                                            int clip) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  typedef typename std::conditional<F32, float, _Float16>::type T;
  const T *qkv = (const T *)qkv_;
  _Float16 *ctx = (_Float16 *)ctx_;  // F32: head plane, tail plane ctx_lo_offset elements later
  const int SP = (S + 31) / 32 * 32;
  constexpr int QLD = DH + 8;
  constexpr int NQ = F32 ? 2 : 1;
  const int SLD = SP + 1, PLD = SP + 8;
  _Float16 *sQh = (_Float16 *)smem;  // [QT][QLD]; reused for the V block in phase 3
  _Float16 *sQl = sQh + (F32 ? QT * QLD : 0);
  float *sS = (float *)(smem + (size_t)NQ * QT * QLD * 2);
  _Float16 *sPh = (_Float16 *)((unsigned char *)sS + (size_t)QT * SLD * 4);
  _Float16 *sPl = sPh + (F32 ? QT * PLD : 0);
  float *sR = (float *)((unsigned char *)sPh + (size_t)NQ * QT * PLD * 2);  // [QT][2*MAX_CLIP+1] q . rk

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, g = lane >> 5;
  const int b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * QT;
  const int L = len[b];  // already clamped to [1,S]
  const long row0 = (long)b * S;
  const long ld = 3L * d;
  const int hoff = h * DH;

  if (q0 >= L) {  // padding queries: defined output, no work
    for (int i = tid; i < QT * DH; i += 256) {
      int r = i / DH, c = i % DH;
      if (q0 + r < S) {
        ctx[(row0 + q0 + r) * d + hoff + c] = (_Float16)0.f;
        if (F32) ctx[(row0 + q0 + r) * d + hoff + c + ctx_lo_offset] = (_Float16)0.f;
      }
    }
    return;
  }
  const int nkb = (L + 31) / 32;

  // stage the query tile (rows beyond S re-read the last row; they are never stored)
  for (int i = tid; i < QT * (DH / 8); i += 256) {
    int r = i / (DH / 8), c = i % (DH / 8);
    int qr = min(q0 + r, S - 1);
    const T *src = qkv + (row0 + qr) * ld + hoff + c * 8;
    if (F32) {
      float f[8];
      *(float4 *)f = *(const float4 *)src;
      *(float4 *)(f + 4) = *(const float4 *)(src + 4);
      half8 hi, lo;
      split8(f, hi, lo);
      *(half8 *)(sQh + r * QLD + c * 8) = hi;
      *(half8 *)(sQl + r * QLD + c * 8) = lo;
    } else {
      *(uint4 *)(sQh + r * QLD + c * 8) = *(const uint4 *)src;
    }
  }
  __syncthreads();

  if (rk) {  // q . rk for the 2*clip+1 relative offsets
    const int nrel = 2 * clip + 1;
    for (int i = tid; i < QT * nrel; i += 256) {
      int r = i / nrel, o = i % nrel;
      float acc = 0.f;
      for (int e = 0; e < DH; e++) {
        float qv = (float)sQh[r * QLD + e];
        if (F32) qv += (float)sQl[r * QLD + e] * LO_INV;
        acc += qv * rk[o * DH + e];
      }
      sR[r * (2 * MAX_CLIP + 1) + o] = acc;
    }
    __syncthreads();
  }

  // phase 1: scores.  Each lane streams its key row straight from global memory, 32 consecutive
  // k per 64-wide chunk (every key element is used once per query tile, so LDS would add
  // nothing); lane group g takes k in [c*64 + g*32, +32) and the query fragment uses the same
  // assignment.
  for (int kb = wave; kb < nkb; kb += 4) {
    floatx16 acc, accx;
#pragma unroll
    for (int v = 0; v < 16; v++) acc[v] = accx[v] = 0.f;
    const int key = min(kb * 32 + li, S - 1);
    const T *kp = qkv + (row0 + key) * ld + d + hoff + g * 32;
#pragma unroll 2
    for (int c = 0; c < DH / 64; c++) {
      half8 kh[4], kl[4];
      if (F32) {
        float f[32];
#pragma unroll
        for (int u = 0; u < 8; u++) *(float4 *)(f + 4 * u) = *(const float4 *)(kp + c * 64 + u * 4);
#pragma unroll
        for (int u = 0; u < 4; u++) split8(f + 8 * u, kh[u], kl[u]);
      } else {
#pragma unroll
        for (int u = 0; u < 4; u++) kh[u] = *(const half8 *)(kp + c * 64 + u * 8);
      }
#pragma unroll
      for (int u = 0; u < 4; u++) {
        const int qo = li * QLD + c * 64 + g * 32 + u * 8;
        half8 a = *(const half8 *)(sQh + qo);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, kh[u], acc, 0, 0, 0);
        if (F32) {
          half8 al = *(const half8 *)(sQl + qo);
          accx = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, kh[u], accx, 0, 0, 0);
          accx = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, kl[u], accx, 0, 0, 0);
        }
      }
    }
    const int j = kb * 32 + li;
#pragma unroll
    for (int v = 0; v < 16; v++) {
      const int i = (v >> 2) * 8 + g * 4 + (v & 3);
      float s = acc[v];
      if (F32) s += accx[v] * LO_INV;
      if (rk) {
        int rel = j - (q0 + i);
        rel = max(-clip, min(clip, rel));
        s += sR[i * (2 * MAX_CLIP + 1) + rel + clip];
      }
      sS[i * SLD + j] = (j < L) ? s : -INFINITY;
    }
  }
  __syncthreads();

  // phase 2: fp32 softmax, 8 threads per query row
  {
    const int i = tid >> 3, sub = tid & 7, nk = nkb * 32;
    float mx = -INFINITY;
    for (int j = sub; j < nk; j += 8) mx = fmaxf(mx, sS[i * SLD + j]);
#pragma unroll
    for (int m = 4; m >= 1; m >>= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    float sum = 0.f;
    for (int j = sub; j < nk; j += 8) {
      float e = F32 ? expf(sS[i * SLD + j] - mx) : __expf(sS[i * SLD + j] - mx);
      sS[i * SLD + j] = e;
      sum += e;
    }
#pragma unroll
    for (int m = 4; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, 64);
    const float inv = 1.f / sum;
    for (int j = sub; j < nk; j += 8) {
      const float pv = sS[i * SLD + j] * inv;
      const _Float16 hi = (_Float16)pv;
      sPh[i * PLD + j] = hi;
      if (F32) sPl[i * PLD + j] = (_Float16)((pv - (float)hi) * LO_SCALE);
    }
  }

  // phase 3: context = P V.  The V block is staged in LDS in its natural [key][col] layout and
  // the MFMA operand (8 keys of one column) is gathered with 16-bit LDS reads.
  constexpr int NCB = (DH >= 128) ? DH / 128 : 1;  // 32-column blocks per wave
  constexpr int ACTIVE = (DH / 32 < 4) ? DH / 32 : 4;
  floatx16 o[NCB], ox[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; cb++)
#pragma unroll
    for (int v = 0; v < 16; v++) o[cb][v] = ox[cb][v] = 0.f;
  _Float16 *sVh = sQh, *sVl = sQl;
  for (int kb = 0; kb < nkb; kb++) {
    __syncthreads();  // sQ / previous V block no longer read; sP complete (first pass)
    for (int i = tid; i < 32 * (DH / 8); i += 256) {
      int r = i / (DH / 8), c = i % (DH / 8);
      int key = min(kb * 32 + r, S - 1);
      const T *src = qkv + (row0 + key) * ld + 2 * d + hoff + c * 8;
      if (F32) {
        float f[8];
        *(float4 *)f = *(const float4 *)src;
        *(float4 *)(f + 4) = *(const float4 *)(src + 4);
        half8 hi, lo;
        split8(f, hi, lo);
        *(half8 *)(sVh + r * QLD + c * 8) = hi;
        *(half8 *)(sVl + r * QLD + c * 8) = lo;
      } else {
        *(uint4 *)(sVh + r * QLD + c * 8) = *(const uint4 *)src;
      }
    }
    __syncthreads();
    if (wave < ACTIVE) {
#pragma unroll
      for (int ks = 0; ks < 2; ks++) {
        const int po = li * PLD + kb * 32 + ks * 16 + g * 8;
        half8 a = *(const half8 *)(sPh + po), al;
        if (F32) al = *(const half8 *)(sPl + po);
#pragma unroll
        for (int cb = 0; cb < NCB; cb++) {
          const int col = (wave * NCB + cb) * 32 + li;
          half8 bv, bl;
#pragma unroll
          for (int e = 0; e < 8; e++) {
            bv[e] = sVh[(ks * 16 + g * 8 + e) * QLD + col];
            if (F32) bl[e] = sVl[(ks * 16 + g * 8 + e) * QLD + col];
          }
          o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bv, o[cb], 0, 0, 0);
          if (F32) {
            ox[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bv, ox[cb], 0, 0, 0);
            ox[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bl, ox[cb], 0, 0, 0);
          }
        }
      }
    }
  }
  if (wave < ACTIVE) {
#pragma unroll
    for (int cb = 0; cb < NCB; cb++) {
      const int col = (wave * NCB + cb) * 32 + li;
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int q = q0 + (v >> 2) * 8 + g * 4 + (v & 3);
        float val = o[cb][v];
        if (F32) val += ox[cb][v] * LO_INV;
        if (q >= S) continue;
        if (q >= L) val = 0.f;
        const _Float16 hi = (_Float16)val;
        ctx[(row0 + q) * d + hoff + col] = hi;
        if (F32) ctx[(row0 + q) * d + hoff + col + ctx_lo_offset] = (_Float16)(val - (float)hi);
      }
    }
  }
}

template <int DH, bool F32>
static hipError_t enc_attention_launch(const void *qkv, const int32_t *len, void *ctx, long ctx_lo_offset, int B, int S,
                                       int d, int heads, const float *rk, int clip, hipStream_t s) {
  static size_t configured = 0;
  size_t lds = enc_attention_lds_bytes(S, DH, F32);
  if (lds > configured) {
    hipError_t e = hipFuncSetAttribute((const void *)enc_attention_kernel<DH, F32>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = lds;
  }
  dim3 grid((S + QT - 1) / QT, heads, B), block(256);
  hipLaunchKernelGGL((enc_attention_kernel<DH, F32>), grid, block, lds, s, qkv, len, ctx, ctx_lo_offset, S, d, rk, clip);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Wave-per-tile variant for sentences of up to 32*NKB tokens (fp32 inputs, no relative keys).
//
// One wave owns 32 queries of one (sentence, head) and runs the whole attention in registers:
// no LDS, no workgroup barrier, four independent waves per workgroup.  The score blocks are
// computed transposed (A operand = key rows, B operand = query rows), so a lane owns one query
// and its accumulator registers run over the keys: the softmax reduction stays inside the lane
// plus one exchange between the two lane groups, and the probabilities are already laid out as
// the A operand of the P V product (the MFMA contraction index may be permuted freely as long as
// both operands use the same assignment, so V is gathered with the matching key order).
// Split precision as above: head + tail for q, k, v and the probabilities, three MFMAs per
// product into one accumulator (the MFMA keeps fp16 subnormals, the tails need no scaling).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void split8u(const float *f, half8 &hi, half8 &lo) {
#pragma unroll
  for (int e = 0; e < 8; e++) {
    hi[e] = (_Float16)f[e];
    lo[e] = (_Float16)(f[e] - (float)hi[e]);
  }
}

// QK16: the scaled query and the key come as plain fp16 from qk16 [B*S, 2d] (q | k) and the value as fp32 from
// qkv = v [B*S, d]; one MFMA per score product.
template <int DH, int NKB, bool QK16>
__global__ __launch_bounds__(256, NKB == 1 ? 3 : NKB == 2 ? 2 : 1) void enc_attention_wave_kernel(const float *qkv, const _Float16 *qk16, const int32_t *len, _Float16 *ctx,
                                                                 long ctx_lo_offset, int B, int S, int d, int heads,
                                                                 int q_tiles) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, li = lane & 31, g = lane >> 5;
  const long unit = (long)blockIdx.x * 4 + wave;  // uniform over the wave, and known to be: addresses below are a
                                                   // uniform 64-bit base plus a 32-bit lane offset
  if (unit >= (long)B * heads * q_tiles) return;
  const int qt = (int)(unit % q_tiles), h = (int)((unit / q_tiles) % heads), b = (int)(unit / ((long)q_tiles * heads));
  const int L = __builtin_amdgcn_readfirstlane(len[b]), q0 = qt * 32;
  const long row0 = (long)b * S, ld = QK16 ? (long)d : 3L * d;  // row stride of the fp32 array (v alone, or q|k|v)
  const int hoff = h * DH;
  if (q0 >= L) {  // padding queries: defined output, no work
    for (int i = lane; i < 32 * DH; i += 64) {
      const int r = i / DH, c = i % DH;
      if (q0 + r < S) {
        ctx[(row0 + q0 + r) * d + hoff + c] = (_Float16)0.f;
        ctx[(row0 + q0 + r) * d + hoff + c + ctx_lo_offset] = (_Float16)0.f;
      }
    }
    return;
  }
  const int nkb = (L + 31) / 32;  // <= NKB, checked by the launcher through S

  // ---- scores, transposed: sc[kb][v] = q_(q0+li) . k_(kb*32 + (v/4)*8 + g*4 + v%4) ----
  floatx16 sc[NKB];
#pragma unroll
  for (int kb = 0; kb < NKB; kb++)
#pragma unroll
    for (int v = 0; v < 16; v++) sc[kb][v] = 0.f;
  if constexpr (QK16) {
    const _Float16 *qp16 = qk16 + (row0 + min(q0 + li, L - 1)) * (2L * d) + hoff + g * 32;
#pragma nounroll
    for (int c = 0; c < DH / 64; c++) {
      half8 qh[4];
#pragma unroll
      for (int u = 0; u < 4; u++) qh[u] = *(const half8 *)(qp16 + c * 64 + u * 8);  // one 64-byte half line
#pragma unroll
      for (int kb = 0; kb < NKB; kb++) {
        if (kb < nkb) {
          const _Float16 *kp16 = qk16 + (row0 + min(kb * 32 + li, L - 1)) * (2L * d) + d + hoff + g * 32 + c * 64;
          half8 kh[4];
#pragma unroll
          for (int u = 0; u < 4; u++) kh[u] = *(const half8 *)(kp16 + u * 8);
#pragma unroll
          for (int u = 0; u < 4; u++) sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kh[u], qh[u], sc[kb], 0, 0, 0);
        }
      }
    }
  }
  const float *qp = qkv + (row0 + min(q0 + li, L - 1)) * ld + hoff + g * 32;
  // A lane takes its 32 consecutive values of a 64-wide slice (one whole 128-byte line) in one go: taking them in
  // two halves, the second half a loop iteration later, was measured to fetch 17 % more from HBM (the line is
  // evicted in between) for no gain in time.
#pragma nounroll
  for (int c = 0; c < (QK16 ? 0 : DH / 64); c++) {
    float f[32];
#pragma unroll
    for (int u = 0; u < 8; u++) *(float4 *)(f + 4 * u) = *(const float4 *)(qp + c * 64 + u * 4);
    half8 qh[4], ql[4];
#pragma unroll
    for (int u = 0; u < 4; u++) split8u(f + 8 * u, qh[u], ql[u]);
#pragma unroll
    for (int kb = 0; kb < NKB; kb++) {
      if (kb < nkb) {
        const float *kp = qkv + (row0 + min(kb * 32 + li, L - 1)) * ld + d + hoff + g * 32 + c * 64;
#pragma unroll
        for (int u = 0; u < 8; u++) *(float4 *)(f + 4 * u) = *(const float4 *)(kp + u * 4);
#pragma unroll
        for (int u = 0; u < 4; u++) {
          half8 kh, kl;
          split8u(f + 8 * u, kh, kl);
          sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kh, qh[u], sc[kb], 0, 0, 0);
          sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kl, qh[u], sc[kb], 0, 0, 0);
          sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kh, ql[u], sc[kb], 0, 0, 0);
        }
      }
    }
  }

  // ---- fp32 softmax over the keys: in-lane, then one exchange between the lane groups ----
  float mx = -INFINITY;
#pragma unroll
  for (int kb = 0; kb < NKB; kb++)
#pragma unroll
    for (int v = 0; v < 16; v++) {
      const int key = kb * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
      sc[kb][v] = (kb < nkb && key < L) ? sc[kb][v] : -INFINITY;  // masked keys get weight exactly 0
      mx = fmaxf(mx, sc[kb][v]);
    }
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  float sum = 0.f;
#pragma unroll
  for (int kb = 0; kb < NKB; kb++)
#pragma unroll
    for (int v = 0; v < 16; v++) {
      sc[kb][v] = expf(sc[kb][v] - mx);
      sum += sc[kb][v];
    }
  sum += __shfl_xor(sum, 32, 64);
  const float inv = 1.f / sum;
  // probabilities as A-operand fragments: k-step ks of block kb uses registers ks*8 .. ks*8+7
  half8 ph[NKB][2], pl[NKB][2];
#pragma unroll
  for (int kb = 0; kb < NKB; kb++)
#pragma unroll
    for (int ks = 0; ks < 2; ks++) {
      float f[8];
#pragma unroll
      for (int e = 0; e < 8; e++) f[e] = sc[kb][ks * 8 + e] * inv;
      split8u(f, ph[kb][ks], pl[kb][ks]);
    }

  // ---- context = P V, one 32-column block at a time ----
  // With two key blocks the V values of the next block are requested before the MFMAs and stores of the current one
  // (with one block nothing is gained and the registers of the third wave per SIMD are exceeded; beyond two the
  // registers do not allow it).
  const char *vbase = (const char *)(qkv + row0 * ld + (QK16 ? 0 : 2 * d) + hoff);
  char *obase = (char *)(ctx + row0 * d + hoff);
  constexpr bool PREFETCH = NKB == 2;
  float fv[PREFETCH ? 2 : 1][NKB][2][8];
  auto request = [&](int cb, int slot) {
    // the block's base stays one opaque scalar pair: otherwise every one of the 16 addresses becomes a 64-bit
    // induction variable of its own
    const char *vb = vbase + cb * 128;
    asm volatile("" : "+s"(vb));
#pragma unroll
    for (int kb = 0; kb < NKB; kb++) {
      if (kb < nkb) {
#pragma unroll
        for (int ks = 0; ks < 2; ks++)
#pragma unroll
          for (int e = 0; e < 8; e++) {  // same key order as the probability registers
            const int key = min(kb * 32 + (2 * ks + (e >> 2)) * 8 + g * 4 + (e & 3), L - 1);
            fv[slot][kb][ks][e] = *(const float *)(vb + (unsigned)((key * (int)ld + li) * 4));
          }
      }
    }
  };
  auto block = [&](int cb, int slot) {
    char *ob = obase + cb * 64;
    asm volatile("" : "+s"(ob));
    floatx16 o;
#pragma unroll
    for (int v = 0; v < 16; v++) o[v] = 0.f;
#pragma unroll
    for (int kb = 0; kb < NKB; kb++) {
      if (kb < nkb) {
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
          half8 vh, vl;
          split8u(fv[slot][kb][ks], vh, vl);
          o = __builtin_amdgcn_mfma_f32_32x32x16_f16(ph[kb][ks], vh, o, 0, 0, 0);
          o = __builtin_amdgcn_mfma_f32_32x32x16_f16(pl[kb][ks], vh, o, 0, 0, 0);
          o = __builtin_amdgcn_mfma_f32_32x32x16_f16(ph[kb][ks], vl, o, 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int v = 0; v < 16; v++) {
      const int q = q0 + (v >> 2) * 8 + g * 4 + (v & 3);
      if (q >= S) continue;
      const float val = (q < L) ? o[v] : 0.f;
      const _Float16 hi = (_Float16)val;
      char *at_ = ob + (unsigned)((q * d + li) * 2);
      *(_Float16 *)at_ = hi;
      *((_Float16 *)at_ + ctx_lo_offset) = (_Float16)(val - (float)hi);
    }
  };
  if constexpr (PREFETCH) {
    static_assert((DH / 32) % 2 == 0, "the two slots alternate over an even number of column blocks");
    request(0, 0);
#pragma nounroll
    for (int cb = 0; cb < DH / 32; cb += 2) {
      request(cb + 1, 1);
      block(cb, 0);
      if (cb + 2 < DH / 32) request(cb + 2, 0);
      block(cb + 1, 1);
    }
  } else {
#pragma nounroll
    for (int cb = 0; cb < DH / 32; cb++) {
      request(cb, 0);
      block(cb, 0);
    }
  }
}

template <int DH, bool QK16 = false>
static hipError_t enc_attention_wave_launch(const float *qkv, const int32_t *len, _Float16 *ctx, long ctx_lo_offset,
                                            int B, int S, int d, int heads, hipStream_t s, const _Float16 *qk16 = nullptr) {
  const int q_tiles = (S + 31) / 32;
  const long units = (long)B * heads * q_tiles;
  dim3 grid((unsigned)((units + 3) / 4)), block(256);
#define NT_WAVE_CASE(NKB)                                                                                          \
  case NKB:                                                                                                        \
    hipLaunchKernelGGL((enc_attention_wave_kernel<DH, NKB, QK16>), grid, block, 0, s, qkv, qk16, len, ctx, ctx_lo_offset, \
                       B, S, d, heads, q_tiles);                                                                   \
    break;
  switch (q_tiles) {
    NT_WAVE_CASE(1)
    NT_WAVE_CASE(2)
    NT_WAVE_CASE(3)
    NT_WAVE_CASE(4)
    default: return hipErrorInvalidValue;
  }
#undef NT_WAVE_CASE
  return hipGetLastError();
}

bool enc_attention_qk16_supported(int S, int d, int heads, const float *rk) {
  return !rk && S <= 128 && heads == 1 && d == 512;
}

hipError_t launch_enc_attention_qk16(const _Float16 *qk, const float *v, const int32_t *len, void *ctx, long ctx_lo_offset,
                                     int B, int S, int d, int heads, hipStream_t s) {
  if (B <= 0 || S <= 0) return hipSuccess;
  if (!enc_attention_qk16_supported(S, d, heads, nullptr)) return hipErrorInvalidValue;
  return enc_attention_wave_launch<512, true>(v, len, (_Float16 *)ctx, ctx_lo_offset, B, S, d, heads, s, qk);
}

hipError_t launch_enc_attention(const void *qkv, bool f32, const int32_t *len, void *ctx, long ctx_lo_offset, int B,
                                int S, int d, int heads, const float *rk, int clip, hipStream_t s) {
  if (B <= 0 || S <= 0) return hipSuccess;
  if (clip > MAX_CLIP) return hipErrorInvalidValue;
  if (f32 && !rk && S <= 128) {  // register-resident wave-per-tile kernel
    switch (d / heads) {
      case 64: return enc_attention_wave_launch<64>((const float *)qkv, len, (_Float16 *)ctx, ctx_lo_offset, B, S, d, heads, s);
      case 128: return enc_attention_wave_launch<128>((const float *)qkv, len, (_Float16 *)ctx, ctx_lo_offset, B, S, d, heads, s);
      case 256: return enc_attention_wave_launch<256>((const float *)qkv, len, (_Float16 *)ctx, ctx_lo_offset, B, S, d, heads, s);
      case 512: return enc_attention_wave_launch<512>((const float *)qkv, len, (_Float16 *)ctx, ctx_lo_offset, B, S, d, heads, s);
      default: return hipErrorInvalidValue;
    }
  }
#define NT_ATTN_CASE(DH)                                                                                   \
  case DH:                                                                                                 \
    return f32 ? enc_attention_launch<DH, true>(qkv, len, ctx, ctx_lo_offset, B, S, d, heads, rk, clip, s) \
               : enc_attention_launch<DH, false>(qkv, len, ctx, 0, B, S, d, heads, rk, clip, s);
  switch (d / heads) {
    NT_ATTN_CASE(64)
    NT_ATTN_CASE(128)
    NT_ATTN_CASE(256)
    NT_ATTN_CASE(512)
    default: return hipErrorInvalidValue;
  }
#undef NT_ATTN_CASE
}

// ---------------------------------------------------------------------------------------
// single-query attention against a cache
// ---------------------------------------------------------------------------------------
struct Partial {
  float m, l, acc[8];
};

__device__ __forceinline__ void merge(Partial &a, const Partial &b) {
  const float mn = fmaxf(a.m, b.m);
  const float ca = (a.m == -INFINITY) ? 0.f : __expf(a.m - mn);
  const float cb = (b.m == -INFINITY) ? 0.f : __expf(b.m - mn);
  a.l = a.l * ca + b.l * cb;
#pragma unroll
  for (int e = 0; e < 8; e++) a.acc[e] = a.acc[e] * ca + b.acc[e] * cb;
  a.m = mn;
}

template <bool F32>
__device__ __forceinline__ void load8(const void *p, float (&o)[8]) {
  if (F32) {
    const float4 *f = (const float4 *)p;
    float4 a = f[0], b = f[1];
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
  } else {
    half8 hv = *(const half8 *)p;
#pragma unroll
    for (int e = 0; e < 8; e++) o[e] = (float)hv[e];
  }
}

// IND: query rows address the cache through `origin` (rows < 0 are skipped), and with kv_new the newest key/value
// pair of a row is taken from there and stored into the cache on the way.
template <int DH, bool KV_F32, bool IND>
__global__ __launch_bounds__(256) void attn_decode_kernel(const float *q, const void *kv, long row_stride,
                                                          const int32_t *len, int n_keys, int rows, int d, int heads,
                                                          const float *rk, int clip, int qpos, float *ctx,
                                                          long ctx_lo_offset, const int32_t *origin,
                                                          const float *kv_new) {
  constexpr int LPK = DH / 8;              // lanes per key
  constexpr int G = 64 / LPK;              // keys per wave iteration
  constexpr int WPP = (DH >= 256) ? 4 : 1; // waves per (row, head) pair
  constexpr int ESZ = KV_F32 ? 4 : 2;
  __shared__ Partial sPart[4][LPK > 64 ? 1 : LPK];
  __shared__ float sQR[4][2 * MAX_CLIP + 1];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const long pair = (WPP == 4) ? (long)blockIdx.x : (long)blockIdx.x * 4 + wave;
  const int wip = (WPP == 4) ? wave : 0;
  const bool valid = pair < (long)rows * heads;
  const int r = valid ? (int)(pair / heads) : 0, h = valid ? (int)(pair % heads) : 0;
  int rc = r;  // cache row
  if (IND) rc = valid ? origin[r] : -1;
  const int nk = (valid && rc >= 0) ? (len ? len[rc] : n_keys) : 0;
  if (IND && rc < 0) rc = 0;
  const int grp = lane / LPK, sub = lane % LPK;

  float qv[8];
  {
    const float4 *qp = (const float4 *)(q + (long)r * d + h * DH + sub * 8);
    float4 a = qp[0], b = qp[1];
    qv[0] = a.x; qv[1] = a.y; qv[2] = a.z; qv[3] = a.w;
    qv[4] = b.x; qv[5] = b.y; qv[6] = b.z; qv[7] = b.w;
  }
  if (rk) {  // q . rk[o] for every relative offset, one offset per LPK-lane group at a time
    const int nrel = 2 * clip + 1;
    for (int o = grp; o < nrel; o += G) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; e++) s += qv[e] * rk[o * DH + sub * 8 + e];
#pragma unroll
      for (int m = LPK / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
      if (sub == 0) sQR[wave][o] = s;
    }
    __syncthreads();
  }

  Partial p;
  p.m = -INFINITY;
  p.l = 0.f;
#pragma unroll
  for (int e = 0; e < 8; e++) p.acc[e] = 0.f;
  const char *base = (const char *)kv + ((long)rc * row_stride + h * DH + sub * 8) * ESZ;
  for (int j = wip * G + grp; j < nk; j += WPP * G) {
    const char *kp = base + (long)j * 2 * d * ESZ;
    float kx[8], vx[8];
    if (IND && KV_F32 && kv_new && j == nk - 1) {  // the pair computed in this step: use it and append it to the cache
      const char *np_ = (const char *)(kv_new + (long)r * 2 * d + h * DH + sub * 8);
      load8<true>(np_, kx);
      load8<true>(np_ + (long)d * 4, vx);
      float4 *ck = (float4 *)const_cast<char *>(kp), *cv = (float4 *)const_cast<char *>(kp + (long)d * 4);
      ck[0] = make_float4(kx[0], kx[1], kx[2], kx[3]);
      ck[1] = make_float4(kx[4], kx[5], kx[6], kx[7]);
      cv[0] = make_float4(vx[0], vx[1], vx[2], vx[3]);
      cv[1] = make_float4(vx[4], vx[5], vx[6], vx[7]);
    } else {
      load8<KV_F32>(kp, kx);
      load8<KV_F32>(kp + (long)d * ESZ, vx);
    }
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 8; e++) s += qv[e] * kx[e];
#pragma unroll
    for (int m = LPK / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
    if (rk) {
      int rel = max(-clip, min(clip, j - qpos));
      s += sQR[wave][rel + clip];
    }
    const float mn = fmaxf(p.m, s);
    const float corr = (p.m == -INFINITY) ? 0.f : __expf(p.m - mn);
    const float w = __expf(s - mn);
    p.l = p.l * corr + w;
#pragma unroll
    for (int e = 0; e < 8; e++) p.acc[e] = p.acc[e] * corr + w * vx[e];
    p.m = mn;
  }
  // merge the key groups of this wave
#pragma unroll
  for (int mask = LPK; mask < 64; mask <<= 1) {
    Partial o;
    o.m = __shfl_xor(p.m, mask, 64);
    o.l = __shfl_xor(p.l, mask, 64);
#pragma unroll
    for (int e = 0; e < 8; e++) o.acc[e] = __shfl_xor(p.acc[e], mask, 64);
    merge(p, o);
  }
  if (WPP == 4) {
    if (lane < LPK) sPart[wave][lane] = p;
    __syncthreads();
    if (wave == 0 && lane < LPK) {
#pragma unroll
      for (int w = 1; w < 4; w++) merge(p, sPart[w][lane]);
    }
    if (wave != 0) return;
  }
  if (valid && lane < LPK) {
    const float inv = (p.l > 0.f) ? 1.f / p.l : 0.f;
    const long at_ = (long)r * d + h * DH + sub * 8;
    if (ctx_lo_offset == 0) {
      float4 *o = (float4 *)(ctx + at_);
      o[0] = make_float4(p.acc[0] * inv, p.acc[1] * inv, p.acc[2] * inv, p.acc[3] * inv);
      o[1] = make_float4(p.acc[4] * inv, p.acc[5] * inv, p.acc[6] * inv, p.acc[7] * inv);
    } else {  // head/tail pair of fp16 planes for a projection that reads planes
      typedef _Float16 half8v __attribute__((ext_vector_type(8)));
      half8v hi, lo;
#pragma unroll
      for (int e = 0; e < 8; e++) {
        const float val = p.acc[e] * inv;
        hi[e] = (_Float16)val;
        lo[e] = (_Float16)(val - (float)hi[e]);
      }
      *(half8v *)((_Float16 *)ctx + at_) = hi;
      *(half8v *)((_Float16 *)ctx + at_ + ctx_lo_offset) = lo;
    }
  }
}

template <int DH>
static hipError_t attn_decode_launch(const float *q, const void *kv, bool kv_f32, long row_stride, const int32_t *len,
                                     int n_keys, int rows, int d, int heads, const float *rk, int clip, int qpos,
                                     float *ctx, long ctx_lo_offset, const int32_t *origin, const float *kv_new,
                                     hipStream_t s) {
  const long pairs = (long)rows * heads;
  const unsigned grid = (DH >= 256) ? (unsigned)pairs : (unsigned)((pairs + 3) / 4);
#define NT_ATTN_DECODE(F32, IND)                                                                                       \
  hipLaunchKernelGGL((attn_decode_kernel<DH, F32, IND>), dim3(grid), dim3(256), 0, s, q, kv, row_stride, len, n_keys, \
                     rows, d, heads, rk, clip, qpos, ctx, ctx_lo_offset, origin, kv_new)
  if (kv_f32 && origin) NT_ATTN_DECODE(true, true);
  else if (kv_f32) NT_ATTN_DECODE(true, false);
  else if (origin) NT_ATTN_DECODE(false, true);
  else NT_ATTN_DECODE(false, false);
#undef NT_ATTN_DECODE
  return hipGetLastError();
}

hipError_t launch_attn_decode(const float *q, const void *kv, bool kv_f32, long row_stride, const int32_t *len,
                              int n_keys, int rows, int d, int heads, const float *rk, int clip, int qpos,
                              float *ctx, hipStream_t s, long ctx_lo_offset, const int32_t *origin,
                              const float *kv_new) {
  if (rows <= 0) return hipSuccess;
  if (clip > MAX_CLIP) return hipErrorInvalidValue;
  if (kv_new && (!origin || !kv_f32 || len)) return hipErrorInvalidValue;
  switch (d / heads) {
    case 64: return attn_decode_launch<64>(q, kv, kv_f32, row_stride, len, n_keys, rows, d, heads, rk, clip, qpos, ctx, ctx_lo_offset, origin, kv_new, s);
    case 128: return attn_decode_launch<128>(q, kv, kv_f32, row_stride, len, n_keys, rows, d, heads, rk, clip, qpos, ctx, ctx_lo_offset, origin, kv_new, s);
    case 256: return attn_decode_launch<256>(q, kv, kv_f32, row_stride, len, n_keys, rows, d, heads, rk, clip, qpos, ctx, ctx_lo_offset, origin, kv_new, s);
    case 512: return attn_decode_launch<512>(q, kv, kv_f32, row_stride, len, n_keys, rows, d, heads, rk, clip, qpos, ctx, ctx_lo_offset, origin, kv_new, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace nt
