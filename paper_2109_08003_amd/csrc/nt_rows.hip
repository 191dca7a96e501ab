// Row-wise kernels: embedding gather + sinusoidal positions, LayerNorm, the start-of-step kernel
// of the decoder (arg-max reduction of the previous step + embedding + LayerNorm), and helpers.
// One wave64 per row; a row of d <= 1024 values lives in at most 16 registers per lane and
// every reduction is a wavefront butterfly (no LDS).  Statistics are fp32: mean first, then the
// biased variance of the centred values.
#include "nt_kernels.h"

namespace nt {

constexpr int MAX_PER_LANE = 16;  // d <= 1024

// The kernels are compiled for the row lengths in use (NE = d / 64 elements per lane: 4, 8, 16) and once for any
// other length (NE = 0: the count is a run-time value and every element is guarded).  The fixed counts matter for
// more than the loop overhead: loads and stores of a wave complete in order on one counter, and around guarded
// accesses the compiler waits for that counter to reach zero, so that every store would wait for the acknowledgement
// of the one before it.
#define NT_FOR_LANE_ELEMS(i) \
  _Pragma("unroll") for (int i = 0; i < (NE ? NE : MAX_PER_LANE); i++) if (NE || i < ne)
static int ne_case(int d) { return (d == 256 || d == 512 || d == 1024) ? d / 64 : 0; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    unsigned int lo = __shfl_xor((unsigned int)x, m, 64), hi = __shfl_xor((unsigned int)(x >> 32), m, 64);
    unsigned long long o = ((unsigned long long)hi << 32) | lo;
    x = o > x ? o : x;
  }
  return x;
}

// lane holds elements lane + 64*i, i < ne
template <int NE>
__device__ __forceinline__ void row_layer_norm(float (&v)[MAX_PER_LANE], int ne, int d, LnEps eps, int lane,
                                               const float *gamma, const float *beta) {
  float ga[MAX_PER_LANE], be[MAX_PER_LANE];
  NT_FOR_LANE_ELEMS(i) {
    ga[i] = gamma[lane + 64 * i];
    be[i] = beta[lane + 64 * i];
  }
  float s = 0.f;
  NT_FOR_LANE_ELEMS(i) s += v[i];
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
  NT_FOR_LANE_ELEMS(i) {
    const float c = v[i] - mean;
    q += ln_term(c, eps.l1);
  }
  const float rstd = ln_rscale(wave_sum(q) / (float)d, eps);
  NT_FOR_LANE_ELEMS(i) v[i] = ga[i] * ((v[i] - mean) * rstd) + be[i];
}

template <int NE>
__global__ __launch_bounds__(256) void embed_src_kernel(const int32_t *src, const int32_t *len, int32_t *len_out, int B,
                                                        int S, int d, int vocab, int pad_id, const _Float16 *E,
                                                        const float *pe, float *x, int32_t *flags) {
  const int lane = threadIdx.x & 63;
  const long r = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= (long)B * S) return;
  const int b = (int)(r / S), pos = (int)(r % S);
  if (pos == 0 && lane == 0) {
    int L = len[b];
    if (L < 1 || L > S) {
      flags[0] = 1;
      L = L < 1 ? 1 : S;
    }
    len_out[b] = L;
  }
  int id = src[r];
  int L = len[b];
  if (pos >= L) id = pad_id;  // padding carries no meaning; make it deterministic
  if (id < 0 || id >= vocab) {
    if (lane == 0) flags[0] = 1;
    id = pad_id;
  }
  const float sc = sqrtf((float)d);
  const _Float16 *e = E + (long)id * d;
  const float *p = pe + (long)pos * d;
  float *o = x + r * d;
  if (NE) {
    float v[MAX_PER_LANE];
    const int ne = NE;
    NT_FOR_LANE_ELEMS(i) v[i] = sc * (float)e[lane + 64 * i] + p[lane + 64 * i];
    NT_FOR_LANE_ELEMS(i) __builtin_nontemporal_store(v[i], o + lane + 64 * i);  // 134 MB per batch, read once later
  } else {
    for (int i = lane; i < d; i += 64) o[i] = sc * (float)e[i] + p[i];
  }
}

hipError_t launch_embed_src(const int32_t *src, const int32_t *len, int32_t *len_out, int B, int S, int d, int vocab,
                            int pad_id, const _Float16 *E, const float *pe, float *x, int32_t *flags, hipStream_t s) {
  long rows = (long)B * S;
  if (rows <= 0) return hipSuccess;
#define NT_CASE(NE_)                                                                                                  \
  case NE_:                                                                                                           \
    hipLaunchKernelGGL(embed_src_kernel<NE_>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, src, len, len_out, B, \
                       S, d, vocab, pad_id, E, pe, x, flags);                                                         \
    break;
  switch (ne_case(d)) { NT_CASE(4) NT_CASE(8) NT_CASE(16) NT_CASE(0) }
#undef NT_CASE
  return hipGetLastError();
}

template <int MODE, int NE>
__global__ __launch_bounds__(256) void layer_norm_kernel(const float *x, int M, int d, const float *gamma,
                                                         const float *beta, LnEps eps, void *out, long lo_offset,
                                                         float *lo_norm) {
  const int lane = threadIdx.x & 63;
  const long r = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= M) return;
  const int ne = d >> 6;
  float v[MAX_PER_LANE];
  const float *xr = x + r * d;
  NT_FOR_LANE_ELEMS(i) v[i] = xr[lane + 64 * i];
  row_layer_norm<NE>(v, ne, d, eps, lane, gamma, beta);
  float tail2 = 0.f;
  NT_FOR_LANE_ELEMS(i) {
      const long o = r * d + lane + 64 * i;
      if (MODE == OUT_F32) {
        ((float *)out)[o] = v[i];
      } else {
        const _Float16 hi = (_Float16)v[i];
        ((_Float16 *)out)[o] = hi;
        if (MODE == OUT_PLANES) {
          const _Float16 lo = (_Float16)(v[i] - (float)hi);
          ((_Float16 *)out)[o + lo_offset] = lo;
          tail2 += (float)lo * (float)lo;
        }
      }
    }
  if (MODE == OUT_PLANES && lo_norm) {
    tail2 = wave_sum(tail2);
    if (lane == 0) lo_norm[r] = sqrtf(tail2) * 1.0001f;  // rounded up: it is used as an upper bound
  }
}

hipError_t launch_layer_norm(const float *x, int M, int d, const float *gamma, const float *beta, LnEps eps,
                             void *out, int out_mode, long lo_offset, hipStream_t s, float *lo_norm) {
  if (M <= 0) return hipSuccess;
  dim3 grid((M + 3) / 4), block(256);
#define NT_CASE(NE_)                                                                                             \
  case NE_:                                                                                                      \
    if (out_mode == OUT_F32)                                                                                     \
      hipLaunchKernelGGL((layer_norm_kernel<OUT_F32, NE_>), grid, block, 0, s, x, M, d, gamma, beta, eps, out,     \
                         lo_offset, lo_norm);                                                                    \
    else if (out_mode == OUT_PLANES)                                                                             \
      hipLaunchKernelGGL((layer_norm_kernel<OUT_PLANES, NE_>), grid, block, 0, s, x, M, d, gamma, beta, eps, out,  \
                         lo_offset, lo_norm);                                                                    \
    else                                                                                                         \
      hipLaunchKernelGGL((layer_norm_kernel<OUT_F16, NE_>), grid, block, 0, s, x, M, d, gamma, beta, eps, out,     \
                         lo_offset, lo_norm);                                                                    \
    break;
  switch (ne_case(d)) { NT_CASE(4) NT_CASE(8) NT_CASE(16) NT_CASE(0) }
#undef NT_CASE
  return hipGetLastError();
}

__global__ void planes_to_float_kernel(const _Float16 *hi, const _Float16 *lo, float *out, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = (float)hi[i] + (float)lo[i];
}
hipError_t launch_planes_to_float(const _Float16 *hi, const _Float16 *lo, float *out, long n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(planes_to_float_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, hi, lo, out, n);
  return hipGetLastError();
}

__global__ void half_to_float_kernel(const _Float16 *in, float *out, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = (float)in[i];
}
hipError_t launch_half_to_float(const _Float16 *in, float *out, long n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(half_to_float_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, in, out, n);
  return hipGetLastError();
}

__global__ void fill_i32_kernel(int32_t *p, long n, int32_t v) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
hipError_t launch_fill_i32(int32_t *p, long n, int32_t v, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n, v);
  return hipGetLastError();
}

// Busy-waits for a given number of 100 MHz ticks (bounded by an iteration count, so it always ends).  Used at
// load time to find out which streams run concurrently.
__global__ void spin_kernel(long ticks, int *sink) {
  const long t0 = wall_clock64();
  int it = 0;
  while (wall_clock64() - t0 < ticks && it < 2000000) it++;
  if (it < 0) *sink = it;
}
hipError_t launch_spin(long ticks, int *sink, hipStream_t s) {
  hipLaunchKernelGGL(spin_kernel, dim3(1), dim3(64), 0, s, ticks, sink);
  return hipGetLastError();
}

// ---- probes of what the machine reaches: a loop of independent MFMAs, and a streaming read ----------------------
typedef _Float16 probe_half8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));
// RANDOM = false: every MFMA multiplies the same two constant operands, the most the pipes ever do (little switching
// in the multipliers, so the chip holds its clock).  RANDOM = true: eight A and eight B operands of random fp16 values
// in rotation, so that the operand bits change from one instruction to the next as they do on a model's weights and
// activations: the rate the power limit then allows, which is the ceiling of a real matrix product.
template <bool RANDOM>
__global__ __launch_bounds__(512) void probe_mfma_kernel(int iters, float *sink) {
  probe_half8 a[8], b[8];
  unsigned x = 12345u ^ (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int e = 0; e < 8; e++) {
      x = x * 1664525u + 1013904223u;
      a[i][e] = (_Float16)(RANDOM ? (float)(x >> 8) * (1.f / 8388608.f) - 1.f : 0.5f);
      x = x * 1664525u + 1013904223u;
      b[i][e] = (_Float16)(RANDOM ? ((float)(x >> 8) * (1.f / 8388608.f) - 1.f) * 0.05f : 0.01f);
    }
  probe_floatx16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int v = 0; v < 16; v++) acc[i][v] = 0.f;
  for (int it = 0; it < iters; it += 8) {
#pragma unroll
    for (int j = 0; j < 8; j++)
#pragma unroll
      for (int i = 0; i < 8; i++)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(i + 3 * j) & 7], b[(i + j) & 7], acc[i], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 8; i++) t += acc[i][0] + acc[i][7];
  if (t == 1.2345e33f) *sink = t;  // practically never: keeps the loop alive
}
__global__ __launch_bounds__(256) void probe_read_kernel(const float4 *src, long n4, float *sink) {
  float t = 0.f;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (long)gridDim.x * blockDim.x) {
    const float4 v = src[i];
    t += v.x + v.y + v.z + v.w;
  }
  if (t == 1.2345e33f) *sink = t;  // practically never: keeps the loads alive
}
// dst may be src itself: every thread writes back what it has read, so the buffer keeps its contents
__global__ __launch_bounds__(256) void probe_copy_kernel(const float4 *src, float4 *dst, long n4) {
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (long)gridDim.x * blockDim.x) dst[i] = src[i];
}
hipError_t launch_probe_mfma(int iters, int blocks, bool random_operands, float *sink, hipStream_t s) {
  if (random_operands) hipLaunchKernelGGL(probe_mfma_kernel<true>, dim3(blocks), dim3(512), 0, s, iters, sink);
  else hipLaunchKernelGGL(probe_mfma_kernel<false>, dim3(blocks), dim3(512), 0, s, iters, sink);
  return hipGetLastError();
}
hipError_t launch_probe_read(const void *src, long bytes, float *sink, hipStream_t s) {
  hipLaunchKernelGGL(probe_read_kernel, dim3(256 * 16), dim3(256), 0, s, (const float4 *)src, bytes / 16, sink);
  return hipGetLastError();
}
hipError_t launch_probe_copy(void *buf, long bytes, hipStream_t s) {
  hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 16), dim3(256), 0, s, (const float4 *)buf, (float4 *)buf, bytes / 16);
  return hipGetLastError();
}

template <int NE>
__global__ __launch_bounds__(256) void step_begin_kernel(StepBeginArgs a) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= a.rows_prev) return;
  int y = a.bos_id;
  if (a.cert_count && blockIdx.x == 0 && threadIdx.x == 0) *a.cert_count = 0;
  if (a.t > 0 && a.prev_cert) {
    const int sl = a.slot_of_row[r];
    y = (sl < 0) ? a.tok[r] : (int)(0xFFFFFFFFu - (unsigned int)a.final_key[sl]);
    if (y < 0 || y >= a.vocab) y = a.pad_id;  // cannot happen: every key holds a valid id
    if (lane == 0) a.out[(long)r * a.out_ld + a.t - 1] = y;
  } else if (a.t > 0 && a.pk) {
    unsigned long long k = 0ull;
    const unsigned long long *p = a.pk + (long)r * a.n_partials;
    for (int i = lane; i < a.n_partials; i += 64) {
      unsigned long long c = p[i];
      k = c > k ? c : k;
    }
    k = wave_max_u64(k);
    y = (int)(0xFFFFFFFFu - (unsigned int)k);
    if (y < 0 || y >= a.vocab) y = a.pad_id;  // cannot happen: every partial holds a valid id
    if (lane == 0) a.out[(long)r * a.out_ld + a.t - 1] = y;
  }
  if (r >= a.rows_now) return;
  if (a.forced) {
    y = a.forced[(long)r * a.forced_ld + a.t];
    if (y < 0 || y >= a.vocab) {
      if (lane == 0) a.flags[0] = 1;
      y = a.pad_id;
    }
  }
  const int d = a.d, ne = d >> 6;
  const float sc = sqrtf((float)d);
  const _Float16 *e = a.E + (long)y * d;
  const float *p = a.pe + (long)a.t * d;
  float v[MAX_PER_LANE];
  NT_FOR_LANE_ELEMS(i) v[i] = sc * (float)e[lane + 64 * i] + p[lane + 64 * i];
  NT_FOR_LANE_ELEMS(i) a.z[(long)r * d + lane + 64 * i] = v[i];
  if (!a.a) return;  // the consumer applies the LayerNorm itself
  row_layer_norm<NE>(v, ne, d, a.eps, lane, a.gamma, a.beta);
  NT_FOR_LANE_ELEMS(i) a.a[(long)r * d + lane + 64 * i] = v[i];
}

// ---- EOS-terminated decoding: the rows still decoding are a dense prefix ---------------------------------------
// token of step t-1 for every previous dense row; y[r] = the token if the row goes on, else -1
__global__ __launch_bounds__(256) void eos_collect_kernel(EosStepArgs a) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= a.rows_prev) return;
  const int b = a.origin_prev[r];
  if (b < 0) {
    if (lane == 0) a.y[r] = -1;
    return;
  }
  int y;
  if (a.prev_cert) {
    const int sl = a.slot_of_row[r];
    y = (sl < 0) ? a.tok[r] : (int)(0xFFFFFFFFu - (unsigned int)a.final_key[sl]);
  } else {
    unsigned long long k = 0ull;
    const unsigned long long *p = a.pk + (long)r * a.n_partials;
    for (int i = lane; i < a.n_partials; i += 64) {
      unsigned long long c = p[i];
      k = c > k ? c : k;
    }
    k = wave_max_u64(k);
    y = (int)(0xFFFFFFFFu - (unsigned int)k);
  }
  if (y < 0 || y >= a.vocab) y = a.pad_id;  // cannot happen: every key holds a valid id
  if (lane == 0) {
    a.out[(long)b * a.out_ld + a.t - 1] = y;
    const bool ends = (y == a.eos_id) || (a.t >= a.cap[b]);
    if (ends) a.out_len[b] = a.t;
    a.y[r] = ends ? -1 : y;
  }
}

// One workgroup: stable compaction of the rows with y >= 0.  At t == 0 every batch row with cap > 0 starts.
__global__ __launch_bounds__(1024) void eos_compact_kernel(EosStepArgs a) {
  __shared__ int wave_tot[16];
  __shared__ int base;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) base = 0;
  __syncthreads();
  for (int r0 = 0; r0 < a.rows_prev; r0 += 1024) {
    const int r = r0 + tid;
    int y = -1, b = -1;
    if (r < a.rows_prev) {
      if (a.t == 0) {
        b = r;
        y = (a.cap[r] > 0) ? a.bos_id : -1;
        if (y < 0) a.out_len[r] = 0;
      } else {
        y = a.y[r];
        b = a.origin_prev[r];
      }
    }
    const bool keep = y >= 0;
    const unsigned long long m = __ballot(keep);
    const int before = __popcll(m & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wave] = __popcll(m);
    __syncthreads();
    int off = base;
    for (int w = 0; w < wave; w++) off += wave_tot[w];
    if (keep) {
      a.origin[off + before] = b;
      a.tok_in[off + before] = y;
    }
    __syncthreads();
    if (tid == 0) {
      int tot = 0;
      for (int w = 0; w < 16; w++) tot += wave_tot[w];
      base += tot;
    }
    __syncthreads();
  }
  const int live = base;
  for (int r = live + tid; r < a.rows_prev; r += 1024) {
    a.origin[r] = -1;
    a.tok_in[r] = a.pad_id;
  }
  if (tid == 0) {
    *a.live = live;
    if (a.cert_count) *a.cert_count = 0;  // the certified arg-max of this step counts from zero
    if (a.progress)
      __hip_atomic_store(a.progress, a.progress_tag | ((unsigned long long)(unsigned int)a.t << 32) | (unsigned int)live,
                         __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

template <int NE>
__global__ __launch_bounds__(256) void eos_embed_kernel(EosStepArgs a) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= a.rows_now) return;
  // a dense row without a batch row (origin < 0) embeds pad_id: it computes like any other row (its attention
  // context is zero) and nothing it produces is stored
  const int y = a.tok_in[r];
  const int d = a.d, ne = d >> 6;
  const float sc = sqrtf((float)d);
  const _Float16 *e = a.E + (long)y * d;
  const float *p = a.pe + (long)a.t * d;
  float v[MAX_PER_LANE];
  NT_FOR_LANE_ELEMS(i) v[i] = sc * (float)e[lane + 64 * i] + p[lane + 64 * i];
  NT_FOR_LANE_ELEMS(i) a.z[(long)r * d + lane + 64 * i] = v[i];
}

hipError_t launch_eos_step_begin(const EosStepArgs &a, hipStream_t s) {
  if (a.rows_prev <= 0) return hipSuccess;
  if (a.rows_now > a.rows_prev) return hipErrorInvalidValue;
  if (a.t > 0) hipLaunchKernelGGL(eos_collect_kernel, dim3((a.rows_prev + 3) / 4), dim3(256), 0, s, a);
  hipLaunchKernelGGL(eos_compact_kernel, dim3(1), dim3(1024), 0, s, a);
#define NT_CASE(NE_)                                                                              \
  case NE_:                                                                                       \
    hipLaunchKernelGGL(eos_embed_kernel<NE_>, dim3((a.rows_now + 3) / 4), dim3(256), 0, s, a); \
    break;
  if (a.rows_now > 0 && !a.skip_embed) switch (ne_case(a.d)) { NT_CASE(4) NT_CASE(8) NT_CASE(16) NT_CASE(0) }
#undef NT_CASE
  return hipGetLastError();
}

hipError_t launch_step_begin(const StepBeginArgs &a, hipStream_t s) {
  if (a.rows_prev <= 0) return hipSuccess;
#define NT_CASE(NE_)                                                                                \
  case NE_:                                                                                         \
    hipLaunchKernelGGL(step_begin_kernel<NE_>, dim3((a.rows_prev + 3) / 4), dim3(256), 0, s, a); \
    break;
  switch (ne_case(a.d)) { NT_CASE(4) NT_CASE(8) NT_CASE(16) NT_CASE(0) }
#undef NT_CASE
  return hipGetLastError();
}

}  // namespace nt
