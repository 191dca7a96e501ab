// Single-query attention against 16-bit integer key/value caches (gfx950): the decoder's self- and cross-attention
// for single-head models of width 256 / 512.
//
// The two attention steps of the decoder are pure streams: every cached key and value is read once per step and used
// for one multiply-add, so their time is the bytes they move.  The caches therefore hold 16 bits per element - and
// they hold them as integers with one fp32 scale per vector (absmax / 32767), not as fp16: a key or value vector is
// the output of a projection of LayerNorm-ed activations, its elements are of one magnitude, and a 15-bit fixed-point
// grid over that range has an rms error of about 3e-5 of the vector's spread where fp16's 11 significant bits leave
// 2.8e-4 of every element.  The query, the scores, the softmax and the context stay fp32 (Sec. 3.1 "FP16 Inference":
// full precision around the softmax).  Same spirit as the paper's integer matrices (Sec. 3.2), applied to the data
// that bounds the decoder instead.
//
// Layout: cache row c (a sentence), position p: keys at kv[((c * row_positions + p) * 2) * d], values d elements
// later; scales at sc[(c * row_positions + p) * 2 + {0: key, 1: value}].
//
// A wave owns a query row (or, for small batches, four waves share it and merge); lane l holds elements
// l * NE .. l * NE + NE - 1 of every vector, so a wave instruction reads one whole vector, fully coalesced.  Keys are
// taken four at a time: the partial dot products of a lane are reduced with a reduce-scatter butterfly (seven
// exchanges for four keys instead of six per key), the scores become wave-uniform, and the online softmax rescales
// once per block.
//
// Self-attention: the newest key/value pair arrives as fp32 from the projection (kv_new), is used at full precision,
// and is appended to the cache in integer form by this kernel.
#include <math.h>

#include "nt_kernels.h"

namespace nt {

// Keys per block.  Four, with the block's vectors requested right before their use, keeps the kernel at 80-100
// registers: measured on the whole job (four pipeline lanes) +1.2 % over blocks of eight with the next block
// requested ahead (220-250 registers), which is faster alone; blocks of two in 64 registers were no faster on the job
// either (the kernel's waves start as the workgroups of the other lanes' kernels end, and more of them fit sooner
// when they are small).
constexpr int A16_NK = 4;

bool attn_i16_supported(int d, int heads, int clip) { return heads == 1 && clip == 0 && (d == 256 || d == 512); }

__device__ __forceinline__ float a16_wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}
__device__ __forceinline__ float a16_wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}

// x (NE elements per lane, one vector per wave) -> integer codes at dst, scale at *sc
template <int NE>
__device__ __forceinline__ void a16_quantize_store(const float (&x)[NE], short *dst, float *sc, int lane) {
  typedef short shortNE __attribute__((ext_vector_type(NE)));
  float amax = 0.f;
#pragma unroll
  for (int e = 0; e < NE; e++) amax = fmaxf(amax, fabsf(x[e]));
  amax = a16_wave_max(amax);
  const float scale = amax > 0.f ? amax / 32767.f : 1.f;
  const float inv = 1.f / scale;
  shortNE qv;
#pragma unroll
  for (int e = 0; e < NE; e++) {
    float c = rintf(x[e] * inv);
    c = fminf(fmaxf(c, -32767.f), 32767.f);
    qv[e] = (short)(int)c;
  }
  *(shortNE *)(dst + lane * NE) = qv;
  if (lane == 0) *sc = scale;
}

// fp32 rows [M][2 d] (key | value of one position each) -> integer cache + scales
template <int NE>
__global__ __launch_bounds__(256) void quantize_kv_i16_kernel(const float *x, long M, short *cache, float *sc) {
  constexpr int D = NE * 64;
  const int lane = threadIdx.x & 63;
  const long m = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= M) return;
#pragma unroll
  for (int which = 0; which < 2; which++) {
    float v[NE];
    const float *src = x + (m * 2 + which) * D + lane * NE;
#pragma unroll
    for (int e = 0; e < NE; e += 4) {
      typedef float f32x4 __attribute__((ext_vector_type(4)));
      const f32x4 t = __builtin_nontemporal_load((const f32x4 *)(src + e));  // read once
      v[e] = t[0], v[e + 1] = t[1], v[e + 2] = t[2], v[e + 3] = t[3];
    }
    a16_quantize_store<NE>(v, cache + (m * 2 + which) * D, sc + m * 2 + which, lane);
  }
}

hipError_t launch_quantize_kv_i16(const float *x, long M, int d, short *cache, float *sc, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  const dim3 grid((unsigned)((M + 3) / 4)), block(256);
  if (d == 512) hipLaunchKernelGGL(quantize_kv_i16_kernel<8>, grid, block, 0, s, x, M, cache, sc);
  else if (d == 256) hipLaunchKernelGGL(quantize_kv_i16_kernel<4>, grid, block, 0, s, x, M, cache, sc);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

template <int NE>
struct A16Partial {
  float m, l, acc[NE];
};

// NE: elements per lane (d / 64).  WPP: waves per query row (1: a wave per row, four rows per workgroup; 4: the
// four waves of a workgroup share the row's keys).  SELF: the last of n_keys keys comes from kv_new and is appended.
// IND: query row r uses cache row origin[r] (< 0: no row, zero context).
template <int NE, int WPP, bool SELF, bool IND>
__global__ __launch_bounds__(256) void attn_decode_i16_kernel(AttnI16Args a) {
  constexpr int NK = A16_NK, D = NE * 64;
  typedef short shortNE __attribute__((ext_vector_type(NE)));
  __shared__ A16Partial<NE> sPart[WPP == 4 ? 4 : 1][WPP == 4 ? 64 : 1];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long row = (WPP == 4) ? (long)blockIdx.x : (long)blockIdx.x * 4 + wave;
  const int wip = (WPP == 4) ? wave : 0;
  const bool valid = row < a.rows;
  const int r = valid ? (int)row : 0;
  int rc = r;
  if (IND) rc = valid ? a.origin[r] : -1;
  const bool live = valid && rc >= 0;
  rc = __builtin_amdgcn_readfirstlane(live ? rc : 0);
  const int n_total = __builtin_amdgcn_readfirstlane(live ? (SELF ? a.n_keys : a.len[rc]) : 0);
  const int n_cached = SELF ? (n_total > 0 ? n_total - 1 : 0) : n_total;

  float q[NE];
  {
    const float *qp = a.q + (long)r * D + lane * NE;
#pragma unroll
    for (int e = 0; e < NE; e += 4) {
      const float4 t = *(const float4 *)(qp + e);
      q[e] = t.x, q[e + 1] = t.y, q[e + 2] = t.z, q[e + 3] = t.w;
    }
  }
  const long pos0 = (long)rc * a.row_positions;  // first position of this cache row
  float m = -INFINITY, l = 0.f, acc[NE];
#pragma unroll
  for (int e = 0; e < NE; e++) acc[e] = 0.f;

  // the pair computed in this step: used as it is, and appended to the cache in integer form
  auto new_key = [&]() {
    if (!(SELF && live && wip == 0 && n_total > 0)) return;
    float kx[NE], vx[NE];
    const float *np_ = a.kv_new + (long)r * 2 * D + lane * NE;
#pragma unroll
    for (int e = 0; e < NE; e += 4) {
      const float4 t = *(const float4 *)(np_ + e), u = *(const float4 *)(np_ + D + e);
      kx[e] = t.x, kx[e + 1] = t.y, kx[e + 2] = t.z, kx[e + 3] = t.w;
      vx[e] = u.x, vx[e + 1] = u.y, vx[e + 2] = u.z, vx[e + 3] = u.w;
    }
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < NE; e++) s += q[e] * kx[e];
    m = a16_wave_sum(s);
    l = 1.f;
#pragma unroll
    for (int e = 0; e < NE; e++) acc[e] = vx[e];
    const long p = pos0 + (n_total - 1);
    a16_quantize_store<NE>(kx, a.kv + p * 2 * D, a.sc + p * 2, lane);
    a16_quantize_store<NE>(vx, a.kv + p * 2 * D + D, a.sc + p * 2 + 1, lane);
  };

  // ---- the cached keys, NK at a time; positions past the end repeat the last one and get weight 0 ----
  struct Block {
    shortNE k[NK], v[NK];
    float ks[NK], vs[NK];
  };
  auto load = [&](int j0, Block &b) {
#pragma unroll
    for (int i = 0; i < NK; i++) {
      const int j = j0 + i < n_cached ? j0 + i : n_cached - 1;
      const long p = pos0 + j;
      const short *kp = a.kv + p * 2 * D + lane * NE;
      b.k[i] = *(const shortNE *)kp;
      b.v[i] = *(const shortNE *)(kp + D);
      b.ks[i] = a.sc[p * 2];
      b.vs[i] = a.sc[p * 2 + 1];
    }
  };
  auto compute = [&](int j0, const Block &b) {
    float p[NK];
#pragma unroll
    for (int i = 0; i < NK; i++) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < NE; e++) s += q[e] * (float)b.k[i][e];
      p[i] = s;
    }
    // reduce-scatter: after the exchanges over the top lane bits a lane holds the sum over those bits of the key
    // numbered by them; the remaining exchanges complete it.  Lanes (64 / NK) i .. (64 / NK) (i + 1) - 1 then hold
    // the dot product of key i.
    float r1;
    if constexpr (NK == 8) {
      float r4[4], r2[2];
      {
        const bool up = lane & 32;
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const float send = up ? p[i] : p[i + 4], keep = up ? p[i + 4] : p[i];
          r4[i] = keep + __shfl_xor(send, 32, 64);
        }
      }
      {
        const bool up = lane & 16;
#pragma unroll
        for (int i = 0; i < 2; i++) {
          const float send = up ? r4[i] : r4[i + 2], keep = up ? r4[i + 2] : r4[i];
          r2[i] = keep + __shfl_xor(send, 16, 64);
        }
      }
      {
        const bool up = lane & 8;
        const float send = up ? r2[0] : r2[1], keep = up ? r2[1] : r2[0];
        r1 = keep + __shfl_xor(send, 8, 64);
      }
    } else {
      static_assert(NK == 4, "blocks of 4 or 8 keys");
      float r2[2];
      {
        const bool up = lane & 32;
#pragma unroll
        for (int i = 0; i < 2; i++) {
          const float send = up ? p[i] : p[i + 2], keep = up ? p[i + 2] : p[i];
          r2[i] = keep + __shfl_xor(send, 32, 64);
        }
      }
      {
        const bool up = lane & 16;
        const float send = up ? r2[0] : r2[1], keep = up ? r2[1] : r2[0];
        r1 = keep + __shfl_xor(send, 16, 64);
      }
      r1 += __shfl_xor(r1, 8, 64);
    }
    r1 += __shfl_xor(r1, 4, 64);
    r1 += __shfl_xor(r1, 2, 64);
    r1 += __shfl_xor(r1, 1, 64);
    float s[NK], bm = -INFINITY;
#pragma unroll
    for (int i = 0; i < NK; i++) {
      s[i] = __uint_as_float((unsigned)__builtin_amdgcn_readlane((int)__float_as_uint(r1), (64 / NK) * i)) * b.ks[i];
      if (j0 + i >= n_cached) s[i] = -INFINITY;
      bm = fmaxf(bm, s[i]);
    }
    const float mn = fmaxf(m, bm);  // j0 < n_cached: at least one finite score
    const float corr = (m == -INFINITY) ? 0.f : __expf(m - mn);
    float w[NK], wsum = 0.f;
#pragma unroll
    for (int i = 0; i < NK; i++) {
      w[i] = __expf(s[i] - mn);  // exp(-inf) = 0 for the positions past the end
      wsum += w[i];
      w[i] *= b.vs[i];
    }
    l = l * corr + wsum;
#pragma unroll
    for (int e = 0; e < NE; e++) {
      float t = acc[e] * corr;
#pragma unroll
      for (int i = 0; i < NK; i++) t += w[i] * (float)b.v[i][e];
      acc[e] = t;
    }
    m = mn;
  };
  {
    Block A;
    new_key();
    for (int j0 = wip * NK; j0 < n_cached; j0 += WPP * NK) {
      load(j0, A);
      compute(j0, A);
    }
  }
  if (WPP == 4) {
    A16Partial<NE> &mine = sPart[wave][lane];
    mine.m = m;
    mine.l = l;
#pragma unroll
    for (int e = 0; e < NE; e++) mine.acc[e] = acc[e];
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int w = 1; w < 4; w++) {
      const A16Partial<NE> &o = sPart[w][lane];
      const float mn = fmaxf(m, o.m);
      const float ca = (m == -INFINITY) ? 0.f : __expf(m - mn);
      const float cb = (o.m == -INFINITY) ? 0.f : __expf(o.m - mn);
      l = l * ca + o.l * cb;
#pragma unroll
      for (int e = 0; e < NE; e++) acc[e] = acc[e] * ca + o.acc[e] * cb;
      m = mn;
    }
  }
  if (!valid) return;
  const float inv = (l > 0.f) ? 1.f / l : 0.f;
  const long at_ = (long)r * D + lane * NE;
  if (a.ctx_lo_offset == 0) {
#pragma unroll
    for (int e = 0; e < NE; e += 4)
      *(float4 *)(a.ctx + at_ + e) = make_float4(acc[e] * inv, acc[e + 1] * inv, acc[e + 2] * inv, acc[e + 3] * inv);
  } else {  // head/tail pair of fp16 planes for a projection that reads planes
    typedef _Float16 halfNE __attribute__((ext_vector_type(NE)));
    halfNE hi, lo;
#pragma unroll
    for (int e = 0; e < NE; e++) {
      const float val = acc[e] * inv;
      hi[e] = (_Float16)val;
      lo[e] = (_Float16)(val - (float)hi[e]);
    }
    *(halfNE *)((_Float16 *)a.ctx + at_) = hi;
    *(halfNE *)((_Float16 *)a.ctx + at_ + a.ctx_lo_offset) = lo;
  }
}

template <int NE, bool SELF>
static hipError_t a16_launch(const AttnI16Args &a, hipStream_t s) {
  // a wave per row keeps every SIMD busy once there are a few rows per SIMD; below that the four waves of a
  // workgroup share a row's keys
  // (up to 4,096 rows the shared form was measured as fast alone and slower with other kernels beside it)
  const bool shared = (a.shape_rows > 0 ? a.shape_rows : a.rows) < 1024;
  const unsigned grid = shared ? (unsigned)a.rows : (unsigned)((a.rows + 3) / 4);
#define NT_A16(WPP_, IND_) hipLaunchKernelGGL((attn_decode_i16_kernel<NE, WPP_, SELF, IND_>), dim3(grid), dim3(256), 0, s, a)
  if (shared && a.origin) NT_A16(4, true);
  else if (shared) NT_A16(4, false);
  else if (a.origin) NT_A16(1, true);
  else NT_A16(1, false);
#undef NT_A16
  return hipGetLastError();
}

hipError_t launch_attn_decode_i16(const AttnI16Args &a, hipStream_t s) {
  if (a.rows <= 0) return hipSuccess;
  const bool self = a.kv_new != nullptr;
  if ((self && a.len) || (!self && !a.len) || (a.d != 256 && a.d != 512)) return hipErrorInvalidValue;
  if (a.d == 512) return self ? a16_launch<8, true>(a, s) : a16_launch<8, false>(a, s);
  return self ? a16_launch<4, true>(a, s) : a16_launch<4, false>(a, s);
}

}  // namespace nt
