// Fused kernels of the decoder step (gfx950).
//
// A decoder row depends on no other row, and the decoder is the bottleneck of translation (Sec. 2.2 "Fast Student
// Models"); with a few hundred to a few thousand rows per step its projections are short, dependent launches whose
// time is latency, not arithmetic.  The paper's cure is graph optimisation (Sec. 3.3): fewer, larger nodes.  Here a
// workgroup owns a tile of 32 rows and carries it through a chain of operations without leaving the chip:
//
//   dec_qkv_kernel    token of the previous step (arg-max result) -> embedding * sqrt(d) + position -> LayerNorm ->
//                     Q|K|V projection (q scaled; k, v written straight into the cache slot of this step)
//   dec_chain_kernel  attention context -> output projection + bias + residual -> LayerNorm -> either the next
//                     projection (cross-attention query, first FFN matrix) or, after the last sub-layer, the final
//                     hidden state as a head/tail pair of fp16 planes plus the norm of its tail
//
// Both are built on the streaming form of nt_gemm_stream.hip: the 32-row tile of activations (head and tail fp16
// planes, about 22 significant bits) stays in the LDS, the weights come in MFMA fragment order through a ring of
// registers that runs seven k-steps ahead, both planes are multiplied with the same weight fragment into one fp32
// accumulator.  Between the two projections of a chain the tile lives in the LDS as fp32: the eight waves each own
// 64 output columns of the first projection, so a row's LayerNorm statistics need all of them; the row is then
// normalised by one wave (butterfly reductions), split into planes and becomes the A tile of the second projection.
//
// Fragment order of the weights: [strip = n / 64][ks = k / 16][nb = (n % 64) / 32][lane][8 halfs] with
// lane = n % 32 + 32 * ((k % 16) / 8)  (vocab_pack).
#include "nt_kernels.h"

#include <mutex>

namespace nt {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int DC_WAVES = 8;
constexpr int DC_TM = 32;  // rows of a tile
constexpr int DC_SL = 8;   // register slots of W fragments per wave; the lookahead is DC_SL - 1 k-steps (16 slots: slower)

template <int K>
struct DcShape {
  static constexpr int LD = K + 8;   // halfs per LDS row of the plane tile: the 16 B pad keeps fragment reads conflict-free
  static constexpr int ZLD = K + 4;  // floats per LDS row of the fp32 tile
  static constexpr int KS = K / 16;
  static constexpr int NE = K / 64;  // consecutive elements of a row held by a lane in the row-wise phases
  static constexpr size_t plane_bytes = (size_t)2 * DC_TM * LD * 2;
  static constexpr size_t z_bytes = (size_t)DC_TM * ZLD * 4;
};

bool dec_fused_supported(int K) { return K == 256 || K == 512; }

// weight fragments through a buffer resource: scalar offset per fragment, constant lane offset; a read past the end
// returns zeros instead of faulting
struct DcWeights {
  __amdgpu_buffer_rsrc_t rs;
  int wlane;
  __device__ __forceinline__ DcWeights(const _Float16 *Wp, int n_strips, int K, int lane)
      : rs(__builtin_amdgcn_make_buffer_rsrc((void *)Wp, 0, n_strips * 64 * K * 2, 0x00020000)), wlane(lane * 16) {}
  __device__ __forceinline__ half8 load(int soff, int nb) const {
    u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rs, wlane + nb * 1024, soff, 0);
    return __builtin_bit_cast(half8, t);
  }
};

// the first DC_SL - 1 k-steps of a strip into the ring
template <int K>
__device__ __forceinline__ void dc_preload(const DcWeights &w, int strip, half8 (&wb)[DC_SL][2]) {
  const int sp = strip * (DcShape<K>::KS * 2048);
#pragma unroll
  for (int q = 0; q < DC_SL - 1; q++) {
    wb[q][0] = w.load(sp + q * 2048, 0);
    wb[q][1] = w.load(sp + q * 2048, 1);
  }
}

// One strip of 64 output columns for the 32 rows of the tile: acc[nb][v] becomes
// C[(v / 4) * 8 + g * 4 + v % 4][strip * 64 + nb * 32 + li].  hrow: this lane's fragment address in the head plane
// (the tail plane follows 32 LDS rows later); hf: the two fragments of k-step 0, reloaded for the next strip on the
// way out; the ring holds k-steps 0 .. DC_SL - 2 of this strip on entry and of strip `next` on exit.
template <int K>
__device__ __forceinline__ void dc_strip(const DcWeights &w, const _Float16 *hrow, half8 (&hf)[2], half8 (&wb)[DC_SL][2],
                                         int strip, int next, floatx16 (&acc)[2]) {
  constexpr int KS = DcShape<K>::KS, LD = DcShape<K>::LD;
  static_assert(KS % DC_SL == 0, "the ring of W slots must divide the k-steps of a strip");
  const int pcur = strip * (KS * 2048), pnext = next * (KS * 2048);
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    const int tgt = ks + DC_SL - 1;
    const int pf = tgt < KS ? pcur + tgt * 2048 : pnext + (tgt - KS) * 2048;
    const int ksn = (ks + 1) % KS;
#pragma unroll
    for (int op = 0; op < 2; op++) {
#pragma unroll
      for (int nb = 0; nb < 2; nb++) {
        if (ks == 0 && op == 0) {
          const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(hf[op], wb[ks % DC_SL][nb], zero, 0, 0, 0);
        } else {
          acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(hf[op], wb[ks % DC_SL][nb], acc[nb], 0, 0, 0);
        }
      }
      // refill what was just consumed; the scheduling barrier keeps the loads this far ahead of their use
      hf[op] = *(const half8 *)(hrow + op * DC_TM * LD + ksn * 16);
      if (op == 0) {
        wb[tgt % DC_SL][0] = w.load(pf, 0);
        wb[tgt % DC_SL][1] = w.load(pf, 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// Epilogue of a projection that follows a LayerNorm (no residual): v = (acc + bias) * scale on the first scale_cols
// columns, ReLU, fp32 or fp16 (optionally head + tail) into one of two destinations.  Tiles inside the matrix take
// straight-line stores (a guard around every store makes each wait for the acknowledgement of the one before it).
template <bool C_F32>
__device__ __forceinline__ void dc_store_strip(const floatx16 (&acc)[2], const GemmEpilogue &e, int strip, int m0, int M,
                                               int li, int g) {
  constexpr int CE = C_F32 ? 4 : 2;
  const bool full = m0 + DC_TM <= M;
#pragma unroll
  for (int nb = 0; nb < 2; nb++) {
    const int nbase = strip * 64 + nb * 32;  // uniform; n_split is a multiple of 32
    const int n = nbase + li;
    const float bias = e.bias ? e.bias[n] : 0.f;
    const float scl = (n < e.scale_cols) ? e.scale : 1.f;
    const bool first = nbase < e.n_split;
    char *dst = (char *)(first ? e.dst0 : e.dst1);
    const long ld = first ? e.ld0 : e.ld1;
    const int ncb = first ? nbase : nbase - e.n_split;
    char *dblock = dst + ((long)m0 * ld + ncb) * CE;
    const unsigned dlane = (unsigned)((g * 4 * ld + li) * CE);
    auto put = [&](int v) {
      const int r = (v >> 2) * 8 + (v & 3);
      float val = (acc[nb][v] + bias) * scl;
      if (e.relu) val = fmaxf(val, 0.f);
      char *at_ = dblock + (dlane + (unsigned)(r * ld * CE));
      if (C_F32) {
        *(float *)at_ = val;
      } else {
        const _Float16 hi = (_Float16)val;
        *(_Float16 *)at_ = hi;
        if (e.dst_lo_offset) *((_Float16 *)at_ + e.dst_lo_offset) = (_Float16)(val - (float)hi);
      }
    };
    if (full) {
#pragma unroll
      for (int v = 0; v < 16; v++) put(v);
    } else {
#pragma unroll
      for (int v = 0; v < 16; v++)
        if (m0 + (v >> 2) * 8 + (v & 3) + g * 4 < M) put(v);
    }
  }
}

// LayerNorm of the rows a wave owns (rows wave, wave + 8, ... of the tile; xv[i][j] is element lane * NE + j of the
// i-th of them), fp32 statistics: mean first, then the biased variance (or mean absolute deviation) of the centred
// values.  The butterflies of all rows advance together, one exchange step at a time.  Output: y in place.
template <int K>
__device__ __forceinline__ void dc_layer_norm(float (&xv)[DC_TM / DC_WAVES][DcShape<K>::NE], const float *gamma,
                                              const float *beta, LnEps eps, int lane) {
  constexpr int NE = DcShape<K>::NE, RPW = DC_TM / DC_WAVES;
  float gam[NE], bet[NE];
#pragma unroll
  for (int j = 0; j < NE; j += 4) {
    *(float4 *)&gam[j] = *(const float4 *)(gamma + lane * NE + j);
    *(float4 *)&bet[j] = *(const float4 *)(beta + lane * NE + j);
  }
  float mean[RPW], rstd[RPW];
#pragma unroll
  for (int i = 0; i < RPW; i++) {
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < NE; j++) sum += xv[i][j];
    mean[i] = sum;
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    float o[RPW];
#pragma unroll
    for (int i = 0; i < RPW; i++) o[i] = __shfl_xor(mean[i], m, 64);
#pragma unroll
    for (int i = 0; i < RPW; i++) mean[i] += o[i];
  }
#pragma unroll
  for (int i = 0; i < RPW; i++) {
    mean[i] = mean[i] / (float)K;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < NE; j++) q += ln_term(xv[i][j] - mean[i], eps.l1);
    rstd[i] = q;
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    float o[RPW];
#pragma unroll
    for (int i = 0; i < RPW; i++) o[i] = __shfl_xor(rstd[i], m, 64);
#pragma unroll
    for (int i = 0; i < RPW; i++) rstd[i] += o[i];
  }
#pragma unroll
  for (int i = 0; i < RPW; i++) {
    rstd[i] = ln_rscale(rstd[i] / (float)K, eps);
#pragma unroll
    for (int j = 0; j < NE; j++) xv[i][j] = gam[j] * ((xv[i][j] - mean[i]) * rstd[i]) + bet[j];
  }
}

// y (the rows of one wave) -> head / tail planes of the A tile in the LDS
template <int K>
__device__ __forceinline__ void dc_planes_to_lds(const float (&y)[DC_TM / DC_WAVES][DcShape<K>::NE], _Float16 *sh, int wave,
                                                 int lane) {
  constexpr int NE = DcShape<K>::NE, LD = DcShape<K>::LD, RPW = DC_TM / DC_WAVES;
  typedef _Float16 halfNE __attribute__((ext_vector_type(NE)));
#pragma unroll
  for (int i = 0; i < RPW; i++) {
    halfNE hi, lo;
#pragma unroll
    for (int j = 0; j < NE; j++) {
      hi[j] = (_Float16)y[i][j];
      lo[j] = (_Float16)(y[i][j] - (float)hi[j]);
    }
    const int R = wave + DC_WAVES * i;
    *(halfNE *)(sh + R * LD + lane * NE) = hi;
    *(halfNE *)(sh + (R + DC_TM) * LD + lane * NE) = lo;
  }
}

__device__ __forceinline__ unsigned long long dc_wave_max_u64(unsigned long long x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const unsigned long long o = shfl_xor_u64(x, m);
    x = o > x ? o : x;
  }
  return x;
}

// -----------------------------------------------------------------------------------------------------------------
// Start of a decoder step fused into the self-attention projection.
// Grid: row tiles of rows_prev x col_groups.  Every workgroup of a row tile gathers and normalises the tile (cheap);
// the first of them also collects the tokens of the previous step and writes the residual stream z.  Row tiles
// beyond rows_now exist only to collect tokens of rows that have just finished.
// -----------------------------------------------------------------------------------------------------------------
template <int K>
__global__ __launch_bounds__(DC_WAVES * 64) void dec_qkv_kernel(DecQkvArgs a, int col_groups) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  _Float16 *sh = (_Float16 *)smem;
  typedef DcShape<K> S;
  constexpr int NE = S::NE, RPW = DC_TM / DC_WAVES, LD = S::LD;
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mt = blockIdx.x / col_groups, cg = blockIdx.x % col_groups;
  const int m0 = mt * DC_TM;
  const StepBeginArgs &sb = a.sb;
  const int M = sb.rows_now;
  if (m0 >= M && cg != 0) return;  // a tile kept only for the collection of tokens: one workgroup is enough
  if (sb.cert_count && blockIdx.x == 0 && tid == 0) *sb.cert_count = 0;

  // ---- the tokens: result of the previous step's arg-max (collected into out), or given ----
  int y[RPW];
#pragma unroll
  for (int i = 0; i < RPW; i++) {
    const int r = m0 + wave + DC_WAVES * i;
    int tokn = sb.bos_id;
    if (a.tok_in) {
      tokn = r < M ? a.tok_in[r] : sb.pad_id;
    } else if (sb.t > 0 && r < sb.rows_prev && (sb.prev_cert || sb.pk)) {
      if (sb.prev_cert) {
        const int sl = sb.slot_of_row[r];
        tokn = (sl < 0) ? sb.tok[r] : (int)(0xFFFFFFFFu - (unsigned int)sb.final_key[sl]);
      } else {
        unsigned long long k = 0ull;
        const unsigned long long *p = sb.pk + (long)r * sb.n_partials;
        for (int q = lane; q < sb.n_partials; q += 64) {
          const unsigned long long c = p[q];
          k = c > k ? c : k;
        }
        k = dc_wave_max_u64(k);
        tokn = (int)(0xFFFFFFFFu - (unsigned int)k);
      }
      if (tokn < 0 || tokn >= sb.vocab) tokn = sb.pad_id;  // cannot happen: every key holds a valid id
      if (cg == 0 && lane == 0) sb.out[(long)r * sb.out_ld + sb.t - 1] = tokn;
    }
    if (sb.forced && r < M) {
      tokn = sb.forced[(long)r * sb.forced_ld + sb.t];
      if (tokn < 0 || tokn >= sb.vocab) {
        if (lane == 0) sb.flags[0] = 1;
        tokn = sb.pad_id;
      }
    }
    if (r >= M) tokn = sb.pad_id;  // rows past the active ones compute on the padding token and store nothing
    y[i] = __builtin_amdgcn_readfirstlane(tokn);
  }
  if (m0 >= M) return;  // uniform over the workgroup

  // ---- z = sqrt(d) * E[y] + PE[t]; the residual stream is written once per row tile ----
  float xv[RPW][NE];
  {
    const float sc = sqrtf((float)K);
    typedef _Float16 halfNE __attribute__((ext_vector_type(NE)));
    float pv[NE];
#pragma unroll
    for (int j = 0; j < NE; j += 4) *(float4 *)&pv[j] = *(const float4 *)(sb.pe + (long)sb.t * K + lane * NE + j);
#pragma unroll
    for (int i = 0; i < RPW; i++) {
      const halfNE ev = *(const halfNE *)(sb.E + (long)y[i] * K + lane * NE);
#pragma unroll
      for (int j = 0; j < NE; j++) xv[i][j] = sc * (float)ev[j] + pv[j];
    }
    if (cg == 0) {
#pragma unroll
      for (int i = 0; i < RPW; i++) {
        const int r = m0 + wave + DC_WAVES * i;
        if (r < M) {
#pragma unroll
          for (int j = 0; j < NE; j += 4)
            *(float4 *)(sb.z + (long)r * K + lane * NE + j) = make_float4(xv[i][j], xv[i][j + 1], xv[i][j + 2], xv[i][j + 3]);
        }
      }
    }
  }
  dc_layer_norm<K>(xv, sb.gamma, sb.beta, sb.eps, lane);
  dc_planes_to_lds<K>(xv, sh, wave, lane);

  // ---- Q|K|V projection of the tile: strips sb0 .. sb1 of this column group, wave by wave ----
  const int NS = a.N >> 6;
  const int sb0 = (int)((long)cg * NS / col_groups), sb1 = (int)((long)(cg + 1) * NS / col_groups);
  const DcWeights w(a.Wp, NS, K, lane);
  half8 wb[DC_SL][2];
  int strip = sb0 + wave;
  const bool have = strip < sb1;
  if (have) dc_preload<K>(w, strip, wb);
  __syncthreads();
  if (!have) return;
  const _Float16 *hrow = sh + li * LD + g * 8;
  half8 hf[2];
  hf[0] = *(const half8 *)hrow;
  hf[1] = *(const half8 *)(hrow + DC_TM * LD);
  for (; strip < sb1; strip += DC_WAVES) {
    floatx16 acc[2];
    dc_strip<K>(w, hrow, hf, wb, strip, strip + DC_WAVES < sb1 ? strip + DC_WAVES : strip, acc);
    dc_store_strip<true>(acc, a.e, strip, m0, M, li, g);
  }
}

// -----------------------------------------------------------------------------------------------------------------
// attention context -> projection + bias + residual -> LayerNorm -> [next projection | final planes]
// One workgroup per row tile; wave w owns output columns 64 w .. 64 w + 63 of the first projection (N1 = K).
// -----------------------------------------------------------------------------------------------------------------
template <int K, bool SECOND, bool C2_F32>
__global__ __launch_bounds__(DC_WAVES * 64) void dec_chain_kernel(DecChainArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  typedef DcShape<K> S;
  _Float16 *sh = (_Float16 *)smem;
  float *zt = (float *)(smem + S::plane_bytes);
  constexpr int NE = S::NE, RPW = DC_TM / DC_WAVES, LD = S::LD, ZLD = S::ZLD, NS1 = K / 64;
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m0 = blockIdx.x * DC_TM, M = a.M;
  const bool full = m0 + DC_TM <= M;

  // ---- the A tile (head rows, then tail rows): global memory -> LDS.  Rows past M repeat row M - 1 ----
  if (K == 512) {
#pragma unroll
    for (int i = 0; i < 2 * DC_TM / DC_WAVES; i++) {
      const int R = wave + DC_WAVES * i;
      const _Float16 *src = R >= DC_TM ? a.A_lo : a.A_hi;
      int m = m0 + (R % DC_TM);
      m = m < M ? m : M - 1;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + (long)m * a.lda + lane * 8),
                                       (__attribute__((address_space(3))) void *)(sh + R * LD), 16, 0, 0);
    }
  } else {
    constexpr int CPR = K / 8, PER_T = 2 * DC_TM * CPR / (DC_WAVES * 64);
    u32x4 fr[PER_T];
#pragma unroll
    for (int i = 0; i < PER_T; i++) {
      const int c = tid + DC_WAVES * 64 * i, R = c / CPR, kc = c % CPR;
      const _Float16 *src = R >= DC_TM ? a.A_lo : a.A_hi;
      int m = m0 + (R % DC_TM);
      m = m < M ? m : M - 1;
      fr[i] = *(const u32x4 *)(src + (long)m * a.lda + kc * 8);
    }
#pragma unroll
    for (int i = 0; i < PER_T; i++) {
      const int c = tid + DC_WAVES * 64 * i, R = c / CPR, kc = c % CPR;
      *(u32x4 *)(sh + R * LD + kc * 8) = fr[i];
    }
  }
  const bool have1 = wave < NS1;
  half8 wb[DC_SL][2];
  const DcWeights w1(a.W1p, NS1, K, lane);
  if (have1) dc_preload<K>(w1, wave, wb);
  // bias and residual of this wave's columns, requested now so that the epilogue finds them there (rows past M
  // read row M - 1: always valid memory)
  float res[2][16], b1[2];
  if (have1) {
#pragma unroll
    for (int nb = 0; nb < 2; nb++) {
      const int n = wave * 64 + nb * 32 + li;
      b1[nb] = a.b1 ? a.b1[n] : 0.f;
#pragma unroll
      for (int v = 0; v < 16; v++) {
        int m = m0 + (v >> 2) * 8 + g * 4 + (v & 3);
        m = m < M ? m : M - 1;
        res[nb][v] = a.z[(long)m * a.ldz + n];
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's rows have landed in the LDS before the barrier
  __syncthreads();

  const _Float16 *hrow = sh + li * LD + g * 8;
  half8 hf[2];
  if (have1) {
    hf[0] = *(const half8 *)hrow;
    hf[1] = *(const half8 *)(hrow + DC_TM * LD);
    floatx16 acc[2];
    dc_strip<K>(w1, hrow, hf, wb, wave, wave, acc);
    // z' = acc + bias + z: into the fp32 tile, and back to the residual stream where a later sub-layer needs it
#pragma unroll
    for (int nb = 0; nb < 2; nb++) {
      const int n = wave * 64 + nb * 32 + li;
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int r = (v >> 2) * 8 + g * 4 + (v & 3);
        const float val = acc[nb][v] + b1[nb] + res[nb][v];
        res[nb][v] = val;
        zt[r * ZLD + n] = val;
      }
    }
    if (a.write_z) {
      if (full) {
#pragma unroll
        for (int nb = 0; nb < 2; nb++)
#pragma unroll
          for (int v = 0; v < 16; v++)
            a.z[(long)(m0 + (v >> 2) * 8 + g * 4 + (v & 3)) * a.ldz + wave * 64 + nb * 32 + li] = res[nb][v];
      } else {
#pragma unroll
        for (int nb = 0; nb < 2; nb++)
#pragma unroll
          for (int v = 0; v < 16; v++) {
            const int m = m0 + (v >> 2) * 8 + g * 4 + (v & 3);
            if (m < M) a.z[(long)m * a.ldz + wave * 64 + nb * 32 + li] = res[nb][v];
          }
      }
    }
  }
  // the second projection's first fragments travel while the tile is normalised
  const int NS2 = SECOND ? (a.N2 >> 6) : 0;
  const DcWeights w2(SECOND ? a.W2p : a.W1p, SECOND ? NS2 : NS1, K, lane);
  int strip = wave;
  const bool have2 = SECOND && strip < NS2;
  if (have2) dc_preload<K>(w2, strip, wb);
  __syncthreads();  // the fp32 tile is complete, and every wave is done with the old planes

  // ---- LayerNorm of the tile, rows wave, wave + 8, ... ----
  float xv[RPW][NE];
#pragma unroll
  for (int i = 0; i < RPW; i++) {
    const float *zr = zt + (wave + DC_WAVES * i) * ZLD + lane * NE;
#pragma unroll
    for (int j = 0; j < NE; j += 4) {
      const f32x4 t = *(const f32x4 *)(zr + j);
      xv[i][j] = t[0], xv[i][j + 1] = t[1], xv[i][j + 2] = t[2], xv[i][j + 3] = t[3];
    }
  }
  dc_layer_norm<K>(xv, a.gamma, a.beta, a.eps, lane);
  if (!SECOND) {
    // final hidden state: head / tail planes and the Euclidean norm of the tail (rounded up: it is used as a bound)
    typedef _Float16 halfNE __attribute__((ext_vector_type(NE)));
#pragma unroll
    for (int i = 0; i < RPW; i++) {
      const int m = m0 + wave + DC_WAVES * i;
      halfNE hi, lo;
      float tail2 = 0.f;
#pragma unroll
      for (int j = 0; j < NE; j++) {
        hi[j] = (_Float16)xv[i][j];
        lo[j] = (_Float16)(xv[i][j] - (float)hi[j]);
        tail2 += (float)lo[j] * (float)lo[j];
      }
#pragma unroll
      for (int s = 32; s >= 1; s >>= 1) tail2 += __shfl_xor(tail2, s, 64);
      if (m < M) {
        *(halfNE *)(a.h_hi + (long)m * K + lane * NE) = hi;
        *(halfNE *)(a.h_hi + a.h_lo_offset + (long)m * K + lane * NE) = lo;
        if (a.lo_norm && lane == 0) a.lo_norm[m] = sqrtf(tail2) * 1.0001f;
      }
    }
    return;
  }
  dc_planes_to_lds<K>(xv, sh, wave, lane);
  __syncthreads();
  if (!have2) return;
  hf[0] = *(const half8 *)hrow;
  hf[1] = *(const half8 *)(hrow + DC_TM * LD);
  for (; strip < NS2; strip += DC_WAVES) {
    floatx16 acc[2];
    dc_strip<K>(w2, hrow, hf, wb, strip, strip + DC_WAVES < NS2 ? strip + DC_WAVES : strip, acc);
    dc_store_strip<C2_F32>(acc, a.e2, strip, m0, M, li, g);
  }
}

template <typename KernT>
static hipError_t dc_raise_lds(KernT kern, size_t lds, std::once_flag &once, hipError_t &err) {
  // raising the dynamic LDS limit is per kernel, once per process (several host threads may get here at once)
  std::call_once(once, [&] { err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); });
  return err;
}

template <int K>
static hipError_t dq_launch(const DecQkvArgs &a, hipStream_t s) {
  auto kern = dec_qkv_kernel<K>;
  const size_t lds = DcShape<K>::plane_bytes;
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  if (dc_raise_lds(kern, lds, once, attr_err) != hipSuccess) return attr_err;
  const int rows = a.sb.rows_prev > a.sb.rows_now ? a.sb.rows_prev : a.sb.rows_now;
  const int row_tiles = (rows + DC_TM - 1) / DC_TM, NS = a.N / 64;
  int col_groups = 1;
  // Column groups: as many workgroups share the weight stream of a row tile.  With thousands of rows a strip per wave
  // (three groups for Q|K|V) is best; up to 512 rows - a handful of row tiles, the launch is the latency of one
  // workgroup's stream - two strips per workgroup are: +3 to 4 % on a 4,096-token budget (more groups at 1,900 rows:
  // 21.3 / 25.4 us with four / two busy waves against 20.8).
  const int busy = rows <= 512 ? 2 : DC_WAVES;
  for (int cg = NS / busy; cg > 1; cg--)
    if (NS % cg == 0 && (long)row_tiles * cg <= 1024) {
      col_groups = cg;
      break;
    }
  hipLaunchKernelGGL(kern, dim3(row_tiles * col_groups), dim3(DC_WAVES * 64), lds, s, a, col_groups);
  return hipGetLastError();
}

hipError_t launch_dec_qkv(const DecQkvArgs &a, hipStream_t s) {
  const int K = a.sb.d;
  if (a.sb.rows_prev <= 0 && a.sb.rows_now <= 0) return hipSuccess;
  if (!dec_fused_supported(K) || a.N % 64 != 0 || a.e.n_split % 32 != 0 || a.sb.rows_now > a.sb.rows_prev) return hipErrorInvalidValue;
  return K == 512 ? dq_launch<512>(a, s) : dq_launch<256>(a, s);
}

template <int K, bool SECOND, bool C2_F32>
static hipError_t dch_launch(const DecChainArgs &a, hipStream_t s) {
  auto kern = dec_chain_kernel<K, SECOND, C2_F32>;
  const size_t lds = DcShape<K>::plane_bytes + DcShape<K>::z_bytes;
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  if (dc_raise_lds(kern, lds, once, attr_err) != hipSuccess) return attr_err;
  hipLaunchKernelGGL(kern, dim3((a.M + DC_TM - 1) / DC_TM), dim3(DC_WAVES * 64), lds, s, a);
  return hipGetLastError();
}

hipError_t launch_dec_chain(const DecChainArgs &a, int K, bool c2_f32, hipStream_t s) {
  if (a.M <= 0) return hipSuccess;
  const bool second = a.W2p != nullptr;
  if (!dec_fused_supported(K) || (second && (a.N2 % 64 != 0 || a.e2.n_split % 32 != 0))) return hipErrorInvalidValue;
#define NT_DC_CASE(K_, S_, C_) \
  if (K == K_ && second == S_ && (!S_ || c2_f32 == C_)) return dch_launch<K_, S_, C_>(a, s);
  NT_DC_CASE(512, false, true) NT_DC_CASE(512, true, true) NT_DC_CASE(512, true, false)
  NT_DC_CASE(256, false, true) NT_DC_CASE(256, true, true) NT_DC_CASE(256, true, false)
#undef NT_DC_CASE
  return hipErrorInvalidValue;
}

}  // namespace nt
