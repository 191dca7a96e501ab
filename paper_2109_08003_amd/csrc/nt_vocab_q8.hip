// 8-bit output layer fused with the row arg-max (gfx950): the GPU form of the paper's 8-bit matrix
// multiplication with packing (Sec. 3.2, Eq. 3-6).
//
// Weights: every vocabulary entry v (one column of the layer's matrix) has its own scale and zero point from the
// mean and standard deviation of its d weights (Eq. 3, 4); the signed 8-bit codes are computed once at load time
// and stored in MFMA fragment order ("packing").  Activations: every decoder state (one row) is quantised to
// unsigned 8-bit codes with its own scale and zero point from its minimum and maximum (Eq. 5, 6, per row instead
// of per matrix so that a sentence never depends on its batch mates).  With u the activation codes, q the weight
// codes, and a_zero, zero_v the zero points,
//     I[r][v] = sum_k (u[r][k] - a_zero[r]) (q[v][k] - zero_v)
//             = D[r][v] + c[r] * P[v] - zero_v * SA[r]
// where s = u - 128 are the codes as signed bytes, D = sum_k s q is what the i8 MFMA computes exactly,
// c[r] = 128 - a_zero[r], SA[r] = sum_k s[r][k], P[v] = sum_k q[v][k] - K * zero_v.  The logit is
// a_scale[r] * (b_scale[v] * float(I)); the arg-max of a row is taken on t = b_scale[v] * float(I) in fp32, the
// positive row factor left out.  Everything up to float(I) is exact integer arithmetic, so the result does not
// depend on tiling or on the order of the k-steps.
//
// The kernel has the shape of the fp16 streaming kernel (nt_vocab.hip): a workgroup keeps 128 rows of codes in the
// LDS (64.5 KiB), the weight fragments stream through a ring of registers, a wave owns a strip of 64 vocabulary
// entries at a time and all rows of the tile, a lane owns one row of each 32-row block and folds the strip's
// logits into its running best.  One 32x32x32 i8 MFMA covers twice the k-range of a 32x32x16 fp16 one in the same
// time, the bytes per weight halve, and there is no second pass: the integer result is final.
// The per-entry constants of a strip (scale, zero point, P: 768 B) are fetched at the start of the strip, parked
// in a per-wave LDS slot half-way through it, and read back when the strip is folded.
//
// Fragment order of the packed codes: [strip = v / 64][ks = k / 32][nb = (v % 64) / 32][lane][16 bytes] with
// lane = v % 32 + 32 * ((k % 32) / 16): lane l of the MFMA row operand holds q[v = l % 32][k = 16 * (l / 32) .. + 15].
// Constants: [strip][type: scale, -zero, P][nb][g = 0, 1][16] where entry e of (nb, g) is column
// nb * 32 + (e / 4) * 8 + g * 4 + e % 4 of the strip: the order in which a lane's accumulator registers run.
#include "nt_kernels.h"

#include <cmath>
#include <cstring>
#include <mutex>
#include <type_traits>
#include <vector>

namespace nt {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int q8_u32x4 __attribute__((ext_vector_type(4)));

constexpr int Q8_ROWS = 128;
constexpr int Q8_WAVES = 8;
constexpr int Q8_CONST_BYTES = 768;  // per strip: 3 types x 64 entries x 4 bytes

bool vocab_q8_supported(int K) { return K == 256 || K == 512; }

size_t vocab_q8_pack_bytes(int N, int K) { return (size_t)((N + 63) / 64) * 64 * K; }
size_t vocab_q8_const_bytes(int N) { return (size_t)((N + 63) / 64) * Q8_CONST_BYTES; }

// Eq. 3, 4 for one vocabulary entry, in double and in index order: codes, scale, zero point (itself kept inside
// the signed 8-bit range, which bounds every integer of the kernel: |I| < 2^26, every factor below 2^23).
static void q8_weight_row(const _Float16 *w, int K, int8_t *q, float *scale_out, int32_t *zero_out) {
#pragma clang fp contract(off)
  double mean = 0.0, var = 0.0;
  for (int k = 0; k < K; k++) mean += (double)(float)w[k];
  mean /= (double)K;
  for (int k = 0; k < K; k++) {
    const double c = (double)(float)w[k] - mean;
    var += c * c;
  }
  var /= (double)K;
  const double sd = std::sqrt(var);
  const double scale = sd > 0.0 ? 14.0 * sd / 255.0 : 1.0;
  double zero = std::rint(127.0 - (mean + 7.0 * sd) / scale);
  zero = zero < -128.0 ? -128.0 : (zero > 127.0 ? 127.0 : zero);
  for (int k = 0; k < K; k++) {
    double c = std::rint((double)(float)w[k] / scale + zero);
    c = c < -128.0 ? -128.0 : (c > 127.0 ? 127.0 : c);
    q[k] = (int8_t)c;
  }
  *scale_out = (float)scale;
  *zero_out = (int32_t)zero;
}

void vocab_q8_quantize_row(const _Float16 *w, int K, int8_t *q, float *scale, int32_t *zero) { q8_weight_row(w, K, q, scale, zero); }

// Wt: [N][K] fp16 (K contiguous).  codes: vocab_q8_pack_bytes(N, K); consts: vocab_q8_const_bytes(N).
// Entries beyond N get zero codes and zero constants (their logits are masked in the kernel).
void vocab_q8_pack(const _Float16 *Wt, int N, int K, int8_t *codes, void *consts) {
  const int NS = (N + 63) / 64, KS = K / 32;
  std::vector<int8_t> q((size_t)K);
  std::vector<int8_t> rowmajor((size_t)NS * 64 * K, 0);
  float *cf = (float *)consts;
  int32_t *ci = (int32_t *)consts;
  memset(consts, 0, vocab_q8_const_bytes(N));
  for (int v = 0; v < N; v++) {
    float sc;
    int32_t zero;
    q8_weight_row(Wt + (size_t)v * K, K, q.data(), &sc, &zero);
    int32_t sum = 0;
    for (int k = 0; k < K; k++) sum += q[(size_t)k];
    memcpy(rowmajor.data() + (size_t)v * K, q.data(), (size_t)K);
    const int strip = v / 64, col = v % 64, nb = col / 32, c32 = col % 32;
    const int g = (c32 >> 2) & 1, e = (c32 >> 3) * 4 + (c32 & 3);
    const size_t base = (size_t)strip * (Q8_CONST_BYTES / 4) + (size_t)nb * 32 + (size_t)g * 16 + (size_t)e;
    cf[base] = sc;
    ci[base + 64] = -zero;
    ci[base + 128] = sum - K * zero;
  }
  for (int strip = 0; strip < NS; strip++)
    for (int ks = 0; ks < KS; ks++)
      for (int nb = 0; nb < 2; nb++)
        for (int lane = 0; lane < 64; lane++) {
          const int v = strip * 64 + nb * 32 + (lane & 31), k = ks * 32 + (lane >> 5) * 16;
          memcpy(codes + ((((size_t)strip * KS + ks) * 2 + nb) * 64 + lane) * 16, rowmajor.data() + (size_t)v * K + k, 16);
        }
}

// ---- activations: [LayerNorm and] 8-bit codes per row ------------------------------------------------------------
__device__ __forceinline__ float q8_wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

// One wave per row; a lane owns NE = d / 64 consecutive elements.  codes: [M][d] signed bytes (u - 128);
// a_scale, c (= 128 - a_zero), sa (= sum of the signed codes) per row.  Eq. 5, 6 in fp32, one rounding per
// operation:  scale = (max - min) / 255,  zero = clamp(rint(255 - max / scale)),  u = clamp(rint(h / scale + zero)),
// both clamps to [0, 255].
template <int NE, bool LN>
__global__ __launch_bounds__(256) void q8_rows_kernel(const float *__restrict__ x, int M, const float *__restrict__ gamma,
                                                      const float *__restrict__ beta, LnEps eps,
                                                      int8_t *__restrict__ codes, float *__restrict__ a_scale,
                                                      int32_t *__restrict__ c_out, int32_t *__restrict__ sa_out) {
#pragma clang fp contract(off)
  constexpr int d = NE * 64;
  const int lane = threadIdx.x & 63;
  const long r = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= M) return;
  float v[NE];
#pragma unroll
  for (int j = 0; j < NE; j += 4) *(float4 *)&v[j] = *(const float4 *)(x + r * d + lane * NE + j);
  if (LN) {
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NE; j++) s += v[j];
    const float mean = q8_wave_sum(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < NE; j++) q += ln_term(v[j] - mean, eps.l1);
    const float rs = ln_rscale(q8_wave_sum(q) / (float)d, eps);
#pragma unroll
    for (int j = 0; j < NE; j++) v[j] = gamma[lane * NE + j] * ((v[j] - mean) * rs) + beta[lane * NE + j];
  }
  float mn = v[0], mx = v[0];
#pragma unroll
  for (int j = 1; j < NE; j++) {
    mn = fminf(mn, v[j]);
    mx = fmaxf(mx, v[j]);
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    mn = fminf(mn, __shfl_xor(mn, m, 64));
    mx = fmaxf(mx, __shfl_xor(mx, m, 64));
  }
  const float range = mx - mn;
  const float scale = range > 0.f ? range / 255.0f : 1.0f;
  const float ratio = mx / scale;
  const float zero = fminf(fmaxf(rintf(255.0f - ratio), 0.f), 255.f);  // the zero point is a code too
  int sum = 0;
  unsigned int packed[NE / 4];
#pragma unroll
  for (int j = 0; j < NE; j++) {
    float c = v[j] / scale;
    c = rintf(c + zero);
    c = fminf(fmaxf(c, 0.f), 255.f);
    const int sgn = (int)c - 128;
    sum += sgn;
    if ((j & 3) == 0) packed[j >> 2] = 0u;
    packed[j >> 2] |= (unsigned int)(sgn & 0xFF) << (8 * (j & 3));
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, 64);
  unsigned int *dst = (unsigned int *)(codes + r * d + lane * NE);
#pragma unroll
  for (int j = 0; j < NE / 4; j++) dst[j] = packed[j];
  if (lane == 0) {
    a_scale[r] = scale;
    c_out[r] = 128 - (int)zero;
    sa_out[r] = sum;
  }
}

hipError_t launch_q8_rows(const float *x, int M, int d, const float *gamma, const float *beta, LnEps eps, int8_t *codes,
                          float *a_scale, int32_t *c_out, int32_t *sa_out, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  const dim3 grid((M + 3) / 4), block(256);
  const bool ln = gamma != nullptr;
  if (d == 512 && ln) hipLaunchKernelGGL((q8_rows_kernel<8, true>), grid, block, 0, s, x, M, gamma, beta, eps, codes, a_scale, c_out, sa_out);
  else if (d == 512) hipLaunchKernelGGL((q8_rows_kernel<8, false>), grid, block, 0, s, x, M, gamma, beta, eps, codes, a_scale, c_out, sa_out);
  else if (d == 256 && ln) hipLaunchKernelGGL((q8_rows_kernel<4, true>), grid, block, 0, s, x, M, gamma, beta, eps, codes, a_scale, c_out, sa_out);
  else if (d == 256) hipLaunchKernelGGL((q8_rows_kernel<4, false>), grid, block, 0, s, x, M, gamma, beta, eps, codes, a_scale, c_out, sa_out);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// ---- the streaming arg-max kernel -----------------------------------------------------------------------------------
struct Q8Split {
  int m_tiles, G, per_xcd;
};
static Q8Split q8_split(int M) {
  Q8Split p;
  p.m_tiles = (M + Q8_ROWS - 1) / Q8_ROWS;
  if (p.m_tiles < 1) p.m_tiles = 1;
  p.G = 256 / p.m_tiles;
  if (p.G < 1) p.G = 1;
  if (p.G > 64) p.G = 64;
  p.per_xcd = (p.m_tiles * p.G + 7) / 8;
  return p;
}

int vocab_q8_partials(int M) { return q8_split(M).G; }

template <int K>
__global__ __launch_bounds__(Q8_WAVES * 64) void vocab_q8_kernel(const int8_t *__restrict__ codes,
                                                                const int32_t *__restrict__ c_row,
                                                                const int32_t *__restrict__ sa_row, int M,
                                                                const int8_t *__restrict__ Wq,
                                                                const void *__restrict__ consts, int N, int m_tiles,
                                                                int G, int per_xcd, int ns_div_g, int ns_mod_g,
                                                                unsigned int m_tiles_magic,
                                                                unsigned long long *__restrict__ pk) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int LD = K + 16;      // bytes per LDS row: the pad keeps the 16-byte fragment reads conflict-free
  constexpr int KS = K / 32;      // k-steps of one i8 MFMA
  constexpr int SL = 4;           // ring of W fragment slots per wave (lookahead SL - 1 k-steps)
  static_assert(KS % SL == 0, "the ring of W slots must divide the k-steps of a strip");
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int total = m_tiles * G;
  const int idx = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  {
    const int end = ((blockIdx.x & 7) + 1) * per_xcd;
    if (idx >= (end < total ? end : total)) return;  // uniform over the workgroup
  }
  // idx / m_tiles without a division (which would run on the vector unit and leave everything derived from it,
  // the offsets of the fragment loads included, in vector registers): multiply-high by ceil(2^32 / m_tiles) from
  // the host, exact for idx * m_tiles < 2^32
  const int gi = m_tiles_magic ? (int)__umulhi((unsigned int)idx, m_tiles_magic) : idx;  // (2^32 itself does not fit)
  const int mt = idx - gi * m_tiles;
  const int NS = (N + 63) >> 6;
  // range gi of G near-equal ranges of the NS strips (quotient and remainder come from the host)
  const int sb0 = gi * ns_div_g + (gi < ns_mod_g ? gi : ns_mod_g);
  const int sb1 = sb0 + ns_div_g + (gi < ns_mod_g ? 1 : 0);
  unsigned char *cslot = smem + Q8_ROWS * LD + wave * Q8_CONST_BYTES;  // this wave's copy of a strip's constants

  const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc((void *)Wq, 0, NS * 64 * K, 0x00020000);
  const int wlane = lane * 16;
  auto wload = [&](int soff, int nb) -> i32x4 {
    q8_u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(wrs, wlane + nb * 1024, soff, 0);
    return __builtin_bit_cast(i32x4, t);
  };

  for (int m0 = mt * Q8_ROWS; m0 < M; m0 += m_tiles * Q8_ROWS) {
    i32x4 wb[SL][2];
    int strip = sb0 + wave;
    const bool have = strip < sb1;
    {  // the tile of codes: global memory -> registers -> LDS.  Rows past M repeat row M - 1 (never stored)
      constexpr int CPR = K / 16, PER_T = Q8_ROWS * CPR / (Q8_WAVES * 64);
      q8_u32x4 fr[PER_T];
#pragma unroll
      for (int i = 0; i < PER_T; i++) {
        const int c = tid + Q8_WAVES * 64 * i, R = c / CPR, kc = c % CPR;
        int m = m0 + R;
        m = m < M ? m : M - 1;
        fr[i] = *(const q8_u32x4 *)(codes + (long)m * K + kc * 16);
      }
#pragma unroll
      for (int i = 0; i < PER_T; i++) {
        const int c = tid + Q8_WAVES * 64 * i, R = c / CPR, kc = c % CPR;
        *(q8_u32x4 *)(smem + R * LD + kc * 16) = fr[i];
      }
    }
    if (have) {
      const int sp = strip * (KS * 2048);
#pragma unroll
      for (int q = 0; q < SL - 1; q++) {
        wb[q][0] = wload(sp + q * 2048, 0);
        wb[q][1] = wload(sp + q * 2048, 1);
      }
    }
    __syncthreads();

    // this lane's rows: one per 32-row block
    int crow[4], sarow[4];
#pragma unroll
    for (int a = 0; a < 4; a++) {
      int m = m0 + a * 32 + li;
      m = m < M ? m : M - 1;
      crow[a] = c_row[m];
      sarow[a] = sa_row[m];
    }
    float rmax[4];
    int rcode[4];
#pragma unroll
    for (int a = 0; a < 4; a++) {
      rmax[a] = -INFINITY;
      rcode[a] = 0;
    }

    if (have) {
      i32x16 acc[4][2];
      const unsigned char *hrow = smem + li * LD + g * 16;
      int off2 = 64 * LD;  // second base register: the offsets of rows 64.. do not fit the 16-bit immediate
      asm volatile("" : "+v"(off2));
      const unsigned char *hrow2 = hrow + off2;
      i32x4 hf[4];
#pragma unroll
      for (int op = 0; op < 4; op++) hf[op] = *(const i32x4 *)((op < 2 ? hrow : hrow2) + (op & 1) * 32 * LD);
      for (; strip < sb1; strip += Q8_WAVES) {
        const bool more = strip + Q8_WAVES < sb1;
        const int pcur = strip * (KS * 2048);
        const int pnext = (more ? strip + Q8_WAVES : strip) * (KS * 2048);
        // the constants of this strip (768 B): 48 lanes fetch 16 bytes each now and put them into the wave's LDS
        // slot half-way through the k-loop, when they have arrived; the fold reads them back from there
        q8_u32x4 cfrag = {0u, 0u, 0u, 0u};
        if (lane < Q8_CONST_BYTES / 16)
          cfrag = *(const q8_u32x4 *)((const unsigned char *)consts + (long)strip * Q8_CONST_BYTES + lane * 16);
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
          const int tgt = ks + SL - 1;
          const int pf = tgt < KS ? pcur + tgt * 2048 : pnext + (tgt - KS) * 2048;
          const int ksn = (ks + 1) % KS;
#pragma unroll
          for (int op = 0; op < 4; op++) {
#pragma unroll
            for (int nb = 0; nb < 2; nb++) {
              if (ks == 0) {
                const i32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                acc[op][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wb[ks % SL][nb], hf[op], zero, 0, 0, 0);
              } else {
                acc[op][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wb[ks % SL][nb], hf[op], acc[op][nb], 0, 0, 0);
              }
            }
            hf[op] = *(const i32x4 *)((op < 2 ? hrow : hrow2) + (op & 1) * 32 * LD + ksn * 32);
            if (op == 0) {
              wb[tgt % SL][0] = wload(pf, 0);
              wb[tgt % SL][1] = wload(pf, 1);
            }
            if (ks == KS / 2 && op == 3 && lane < Q8_CONST_BYTES / 16) *(q8_u32x4 *)(cslot + lane * 16) = cfrag;
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // ---- strip done: logits t = scale[v] * float(D + c[r] P[v] - zero[v] SA[r]), folded into the running best ----
        // (the strip that runs past the end of the vocabulary takes the variant that masks those entries)
        auto fold = [&](auto masked_tag) {
          constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
          for (int nb = 0; nb < 2; nb++) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
              const float4 sc4 = *(const float4 *)(cslot + 0 + nb * 128 + g * 64 + j * 16);
              const int4 nz4 = *(const int4 *)(cslot + 256 + nb * 128 + g * 64 + j * 16);
              const int4 p4 = *(const int4 *)(cslot + 512 + nb * 128 + g * 64 + j * 16);
              const float sc[4] = {sc4.x, sc4.y, sc4.z, sc4.w};
              const int nz[4] = {nz4.x, nz4.y, nz4.z, nz4.w};
              const int pp[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
              for (int i = 0; i < 4; i++) {
                const int v = j * 4 + i;
#pragma unroll
                for (int a = 0; a < 4; a++) {
                  // I = D + c P - zero SA as two 24-bit multiply-adds (every factor is below 2^23 in magnitude).  The
                  // empty asm only keeps the compiler from merging the two additions into a three-operand add behind
                  // two multiplies; the accumulator itself is read by an instruction the compiler schedules (it knows
                  // the distance a matrix-core result needs).
                  int t1 = __mul24(crow[a], pp[i]) + acc[a][nb][v];
                  asm("" : "+v"(t1));
                  const int I = __mul24(nz[i], sarow[a]) + t1;
                  float val = sc[i] * (float)I;
                  if (MASKED) val = (strip * 64 + nb * 32 + j * 8 + g * 4 + i < N) ? val : -INFINITY;
                  const bool gt = val > rmax[a];  // codes ascend with the column: on equal logits the lower column stays
                  rmax[a] = gt ? val : rmax[a];
                  rcode[a] = gt ? (strip * 32 + nb * 16 + v) : rcode[a];
                }
              }
              __builtin_amdgcn_sched_barrier(0);  // one group of constants at a time: keeps the registers for the ring
            }
          }
        };
        if (strip * 64 + 64 <= N) fold(std::false_type{}); else fold(std::true_type{});
      }
    }
    __syncthreads();  // every wave is done with the tile: its LDS now carries the per-wave results
    unsigned long long *skey = (unsigned long long *)smem;  // [Q8_WAVES][Q8_ROWS]
#pragma unroll
    for (int a = 0; a < 4; a++) {
      const int c = rcode[a], v = c & 15;
      const int n = (c >> 5) * 64 + ((c >> 4) & 1) * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
      unsigned long long key = (rmax[a] == -INFINITY) ? 0ull : argmax_key(rmax[a], n);
      const unsigned long long okey = shfl_xor_u64(key, 32);  // the two lane groups hold interleaved columns of a row
      key = okey > key ? okey : key;
      if (g == 0) skey[wave * Q8_ROWS + a * 32 + li] = key;
    }
    __syncthreads();
    if (tid < Q8_ROWS) {
      unsigned long long best = 0ull;
#pragma unroll
      for (int w = 0; w < Q8_WAVES; w++) {
        const unsigned long long k = skey[w * Q8_ROWS + tid];
        best = k > best ? k : best;
      }
      const int m = m0 + tid;
      if (m < M) pk[(long)m * G + gi] = best;
    }
    __syncthreads();  // before the next tile overwrites the LDS
  }
}

hipError_t launch_vocab_q8_argmax(const int8_t *codes, const int32_t *c_row, const int32_t *sa_row, int M,
                                  const int8_t *Wq, const void *consts, int N, int K, unsigned long long *pk,
                                  hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (!vocab_q8_supported(K)) return hipErrorInvalidValue;
  const Q8Split p = q8_split(M);
  const size_t lds = (size_t)Q8_ROWS * (K + 16) + Q8_WAVES * Q8_CONST_BYTES;
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [&] {
    attr_err = hipFuncSetAttribute((const void *)vocab_q8_kernel<512>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr_err == hipSuccess)
      attr_err = hipFuncSetAttribute((const void *)vocab_q8_kernel<256>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  });
  if (attr_err != hipSuccess) return attr_err;
  const dim3 grid(8 * p.per_xcd), block(Q8_WAVES * 64);
  const int NS = (N + 63) / 64, qd = NS / p.G, qm = NS % p.G;
  const unsigned int magic = p.m_tiles == 1 ? 0u : (unsigned int)(((1ull << 32) + p.m_tiles - 1) / p.m_tiles);
  if (K == 512)
    hipLaunchKernelGGL((vocab_q8_kernel<512>), grid, block, lds, s, codes, c_row, sa_row, M, Wq, consts, N, p.m_tiles, p.G, p.per_xcd, qd, qm, magic, pk);
  else
    hipLaunchKernelGGL((vocab_q8_kernel<256>), grid, block, lds, s, codes, c_row, sa_row, M, Wq, consts, N, p.m_tiles, p.G, p.per_xcd, qd, qm, magic, pk);
  return hipGetLastError();
}

// ---- plain logits (debug / teacher-forced path): one thread per (row, vocabulary entry) -----------------------------
// logits[r * ld + v] = a_scale[r] * (b_scale[v] * float(I)), straight from the definition with the packed operands.
__global__ __launch_bounds__(256) void q8_logits_kernel(const int8_t *__restrict__ codes, const float *__restrict__ a_scale,
                                                        const int32_t *__restrict__ c_row, int M,
                                                        const int8_t *__restrict__ Wq, const void *__restrict__ consts,
                                                        int N, int K, float *__restrict__ logits, long ld) {
#pragma clang fp contract(off)
  const int v = blockIdx.x * 256 + threadIdx.x, r = blockIdx.y;
  if (v >= N || r >= M) return;
  const int KS = K / 32, strip = v >> 6, col = v & 63, nb = col >> 5, c32 = col & 31;
  const int g = (c32 >> 2) & 1, e = (c32 >> 3) * 4 + (c32 & 3);
  const long cb = (long)strip * (Q8_CONST_BYTES / 4) + nb * 32 + g * 16 + e;
  const float sc = ((const float *)consts)[cb];
  const int zero = -((const int32_t *)consts)[cb + 64];
  const int a_zero = 128 - c_row[r];
  int I = 0;
  for (int k = 0; k < K; k++) {
    const int ks = k >> 5, half = (k >> 4) & 1, b = k & 15;
    const int q = Wq[((((long)strip * KS + ks) * 2 + nb) * 64 + (c32 + 32 * half)) * 16 + b];
    const int u = (int)codes[(long)r * K + k] + 128;
    I += (u - a_zero) * (q - zero);
  }
  const float t = sc * (float)I;
  logits[(long)r * ld + v] = a_scale[r] * t;
}

hipError_t launch_q8_logits(const int8_t *codes, const float *a_scale, const int32_t *c_row, int M, const int8_t *Wq,
                            const void *consts, int N, int K, float *logits, long ld, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  hipLaunchKernelGGL(q8_logits_kernel, dim3((N + 255) / 256, M), dim3(256), 0, s, codes, a_scale, c_row, M, Wq, consts, N, K,
                     logits, ld);
  return hipGetLastError();
}

}  // namespace nt
