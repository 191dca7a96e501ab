// Streaming projection GEMM for K = 256 / 512 (gfx950): C[M,N] = A[M,K] * Wt[N,K]^T with A given
// as a head/tail pair of fp16 planes.
//
// Same division of labour as the streaming output projection: a workgroup keeps its tile of A
// (32 or 64 rows, both planes) in the LDS for its whole life, filled once straight from global
// memory, and the weights - stored at load time in MFMA fragment order - stream through
// registers, one fully coalesced 1 KiB load per fragment, running a few k-steps ahead of their
// use.  The main loop has no LDS writes, no barriers and no address arithmetic; against the tiled
// kernel (both operand tiles written to and read from the LDS for every 64 MFMAs) the LDS
// traffic per MFMA drops to a quarter.  Both planes are multiplied with the same weight
// fragment into one fp32 accumulator.
//
// A wave owns strips of 64 output columns (wave, wave + 8, ... of the workgroup's range) and all
// rows of the tile; the epilogue does what the tiled kernel's does (bias, scale, ReLU, residual, two
// destinations, optional tail plane).  Here the A fragment is the row operand of the MFMA, so a
// lane owns an output column and a store instruction covers 128 contiguous bytes per row.  Tiles
// inside the matrix take an epilogue without branches, so that the stores of a strip are issued
// back to back; encoder-sized launches mark their whole-line streams non-temporal.
//
// Fragment order of Wp: [strip = n / 64][ks = k / 16][nb = (n % 64) / 32][lane][8 halfs] with
// lane = n % 32 + 32 * ((k % 16) / 8).
#include "nt_kernels.h"

#include <mutex>
#include <type_traits>

namespace nt {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int GS_WAVES = 8;

bool gemm_stream_supported(int N, int K) { return (K == 256 || K == 512) && N % 64 == 0; }

// RB = 32-row blocks per tile (1: decoder-sized M; 2: encoder-sized M).
// LN = true: A_hi points to fp32 rows X[M][lda] instead; the tile is LayerNorm-ed (fp32 statistics: mean first, then
// the biased variance of the centred values) and split into head/tail planes while it is written to the LDS, which
// saves the separate LayerNorm kernel and the round trip of its output through memory.
// TAIL = false: only the head plane of A is multiplied (11 significant bits: half the MFMA work and half the tile).
// NC > 1: the contraction runs over NC * K columns of A in NC passes over the K-wide tile (K = 512, planes from memory):
// between passes the tile is refilled behind a barrier while the weight ring keeps streaming, and every wave keeps the
// accumulators of its one strip (N is 512 per column group) - the second matrix of an FFN, whose K is the FFN width.
template <int RB, int K, bool C_F32, bool LN, bool TAIL, int NC>
__global__ __launch_bounds__(GS_WAVES * 64) void gemm_stream_kernel(const _Float16 *__restrict__ A_hi,
                                                                   const _Float16 *__restrict__ A_lo, long lda, int M,
                                                                   const _Float16 *__restrict__ Wp, int N, int col_groups,
                                                                   GemmEpilogue e, GemmLayerNorm ln) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  _Float16 *sh = (_Float16 *)smem;
  constexpr int TM = 32 * RB, ROWS = (TAIL ? 2 : 1) * TM;  // LDS fragment rows: head rows, then tail rows
  constexpr int LD = K + 8;                   // halfs per LDS row: the 16 B pad keeps the fragment reads conflict-free
  constexpr int KS = K / 16;
  // register slots of W fragments per wave; the lookahead is SL - 1 k-steps.  (A deeper ring did not shorten the
  // decoder-sized launches, and fewer registers leave room for other kernels' waves on the same CU.)
  constexpr int SL = 8;
  constexpr int NOPS = (TAIL ? 2 : 1) * RB;
  static_assert(KS % SL == 0, "the ring of W slots must divide the k-steps of a strip");
  static_assert(NC == 1 || (K == 512 && !LN), "several passes: 512-wide tiles of planes only");
  constexpr int KST = NC * KS;  // k-steps of a whole strip
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mt = blockIdx.x / col_groups, cg = blockIdx.x % col_groups;
  const int m0 = mt * TM;
  const int NS = N >> 6;
  const int sb0 = (int)((long)cg * NS / col_groups), sb1 = (int)((long)(cg + 1) * NS / col_groups);

  const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc((void *)Wp, 0, NS * 64 * (NC * K) * 2, 0x00020000);
  const int wlane = lane * 16;
  auto wload = [&](int soff, int nb) -> half8 {
    u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(wrs, wlane + nb * 1024, soff, 0);
    return __builtin_bit_cast(half8, t);
  };

  // ---- the A tile: global memory -> LDS.  Rows past M repeat row M - 1 (their results are never stored) ----
  // planes, K = 512: one wave instruction moves one row of one plane (1 KiB) without passing through registers;
  // pass c of NC takes columns c * K .. c * K + K - 1 of A
  auto fill_planes = [&](int c) {
#pragma unroll
    for (int i = 0; i < ROWS / GS_WAVES; i++) {
      const int R = wave + GS_WAVES * i;
      const _Float16 *src = R >= TM ? A_lo : A_hi;
      int m = m0 + (R % TM);
      m = m < M ? m : M - 1;
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void *)(src + (long)m * lda + c * K + lane * 8),
          (__attribute__((address_space(3))) void *)(sh + R * LD), 16, 0, RB == 2 ? 2 : 0);
    }
  };
  if constexpr (LN) {
    // a wave takes rows wave, wave + 8, ...; a lane holds NE consecutive elements of the row
    constexpr int NE = K / 64, RPW = TM / GS_WAVES;
    const float *X = (const float *)A_hi;
    float xv[RPW][NE];
#pragma unroll
    for (int i = 0; i < RPW; i++) {
      int m = m0 + wave + GS_WAVES * i;
      m = m < M ? m : M - 1;
      const float *xr = X + (long)m * lda + lane * NE;
#pragma unroll
      for (int j = 0; j < NE; j += 4) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        // encoder-sized launches stream their rows, residuals and fp32 outputs past the L2 (non-temporal), so that
        // the weight fragments, which every workgroup reads, stay in it.  Only whole-line accesses are marked:
        // where a line is consumed or produced in pieces (the q/k/v reads and half-line context stores of the encoder
        // attention), the pieces rely on the cache and the hint cost 7 % of the whole job
        const f32x4 t = RB == 2 ? __builtin_nontemporal_load((const f32x4 *)(xr + j)) : *(const f32x4 *)(xr + j);
        xv[i][j] = t[0], xv[i][j + 1] = t[1], xv[i][j + 2] = t[2], xv[i][j + 3] = t[3];
      }
    }
    float gam[NE], bet[NE];
#pragma unroll
    for (int j = 0; j < NE; j += 4) {
      *(float4 *)&gam[j] = *(const float4 *)(ln.gamma + lane * NE + j);
      *(float4 *)&bet[j] = *(const float4 *)(ln.beta + lane * NE + j);
    }
    // The butterflies of all rows advance together, one exchange step at a time: a step of one row waits for the
    // cross-lane exchange before it (about 150 clocks), and row after row these waits were most of the fill.
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
      for (int j = 0; j < NE; j++) {
        const float c = xv[i][j] - mean[i];
        q += ln_term(c, ln.eps.l1);
      }
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
      rstd[i] = ln_rscale(rstd[i] / (float)K, ln.eps);
      typedef _Float16 halfNE __attribute__((ext_vector_type(NE)));
      halfNE hi, lo;
#pragma unroll
      for (int j = 0; j < NE; j++) {
        const float y = gam[j] * ((xv[i][j] - mean[i]) * rstd[i]) + bet[j];
        hi[j] = (_Float16)y;
        lo[j] = (_Float16)(y - (float)hi[j]);
      }
      const int R = wave + GS_WAVES * i;
      *(halfNE *)(sh + R * LD + lane * NE) = hi;
      if (TAIL) *(halfNE *)(sh + (R + TM) * LD + lane * NE) = lo;
    }
  } else if (K == 512) {
    fill_planes(0);
  } else {
    constexpr int CPR = K / 8, PER_T = ROWS * CPR / (GS_WAVES * 64);
    u32x4 fr[PER_T];
#pragma unroll
    for (int i = 0; i < PER_T; i++) {
      const int c = tid + GS_WAVES * 64 * i, R = c / CPR, kc = c % CPR;
      const _Float16 *src = R >= TM ? A_lo : A_hi;
      int m = m0 + (R % TM);
      m = m < M ? m : M - 1;
      fr[i] = *(const u32x4 *)(src + (long)m * lda + kc * 8);
    }
#pragma unroll
    for (int i = 0; i < PER_T; i++) {
      const int c = tid + GS_WAVES * 64 * i, R = c / CPR, kc = c % CPR;
      *(u32x4 *)(sh + R * LD + kc * 8) = fr[i];
    }
  }
  half8 wb[SL][2];
  int strip = sb0 + wave;
  const bool have = strip < sb1;
  if (have) {
    const int sp = strip * (KST * 2048);
#pragma unroll
    for (int q = 0; q < SL - 1; q++) {
      wb[q][0] = wload(sp + q * 2048, 0);
      wb[q][1] = wload(sp + q * 2048, 1);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's rows have landed in the LDS before the barrier
  __syncthreads();
  if (!have) return;
  // Two waves share a SIMD.  With equal priority they take turns at the matrix pipe, finish their strips together
  // and then both sit in the store phase of the epilogue (the long one when the output is fp32) while the pipe
  // idles.  Giving one of them priority makes the phases alternate instead.
  if (wave < GS_WAVES / 2) __builtin_amdgcn_s_setprio(2);

  floatx16 acc[RB][2];
  // fragment row of operand op: head rows of block op % RB, then the tail rows; two base registers, because the
  // byte offsets of the upper half do not fit the 16-bit offset field
  const _Float16 *hrow = sh + li * LD + g * 8;
  constexpr int HALF = ROWS > 32 ? ROWS / 2 : ROWS;  // LDS rows reached from the first base register
  int off2 = HALF * LD;
  asm volatile("" : "+v"(off2));
  const _Float16 *hrow2 = hrow + off2;
  auto frag = [&](int op, int ks) -> half8 {
    const int R0 = op * 32;  // ops 0 .. RB-1: head planes, RB .. 2RB-1: tail planes
    return *(const half8 *)((R0 < HALF ? hrow : hrow2) + (R0 % HALF) * LD + ks * 16);
  };
  half8 hf[NOPS];
#pragma unroll
  for (int op = 0; op < NOPS; op++) hf[op] = frag(op, 0);

  if (NC > 1) {
#pragma unroll
    for (int rb = 0; rb < RB; rb++)
#pragma unroll
      for (int nb = 0; nb < 2; nb++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc[rb][nb][v] = 0.f;
  }
  for (; strip < sb1; strip += GS_WAVES) {
    const bool more = strip + GS_WAVES < sb1;
    int pcur = strip * (KST * 2048);
    const int pnext = (more ? strip + GS_WAVES : strip) * (KST * 2048);
    // bias and scale of the strip's columns, requested here so that the epilogue does not wait for them behind the
    // weight fragments in flight
    float bias[2] = {0.f, 0.f}, scl[2];
#pragma unroll
    for (int nb = 0; nb < 2; nb++) {
      const int n = strip * 64 + nb * 32 + li;
      if (e.bias) bias[nb] = e.bias[n];
      scl[nb] = (n < e.scale_cols) ? e.scale : 1.f;
    }
    // The k-loop of a strip, over the head plane's row blocks alone (NO = RB) or over both planes' (NO = NOPS): the
    // epilogue's tail_col0 .. tail_col1 name the output columns whose strips take the tail plane as well.
    auto k_loop = [&](auto nops_tag, const float (&bias_)[2], const float (&scl_)[2]) {
      constexpr int NO = decltype(nops_tag)::value;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        const int tgt = ks + SL - 1;
        // several passes: the ring simply runs on into the next pass's fragments of the same strip (past the last
        // pass it reads the next strip, or zeros beyond the matrix: unused either way)
        const int pf = (NC > 1 || tgt < KS) ? pcur + tgt * 2048 : pnext + (tgt - KS) * 2048;
        const int ksn = (ks + 1) % KS;
#pragma unroll
        for (int op = 0; op < NO; op++) {
#pragma unroll
          for (int nb = 0; nb < 2; nb++) {
            if (NC == 1 && ks == 0 && op < RB) {
              const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
              acc[op % RB][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(hf[op], wb[ks % SL][nb], zero, 0, 0, 0);
            } else {
              acc[op % RB][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(hf[op], wb[ks % SL][nb], acc[op % RB][nb], 0, 0, 0);
            }
          }
          // refill what was just consumed; the scheduling barrier keeps the loads this far ahead of their use
          hf[op] = frag(op, ksn);
          if (op == 0) {
            wb[tgt % SL][0] = wload(pf, 0);
            wb[tgt % SL][1] = wload(pf, 1);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        // the wait for bias and scale is taken here, where it counts only the fragments requested since; left to the
        // epilogue it becomes a wait for everything in flight
        if (ks == SL) asm volatile("" ::"v"(bias_[0]), "v"(bias_[1]), "v"(scl_[0]), "v"(scl_[1]));
      }
    };
    const bool with_tail = TAIL && strip * 64 >= e.tail_col0 && strip * 64 < e.tail_col1;
#pragma unroll 1
    for (int c = 0; c < NC; c++) {
      if (NC > 1 && c > 0) {
        // next pass: every wave is done with the tile, it is refilled, and the first fragments are read again
        __syncthreads();
        fill_planes(c);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
#pragma unroll
        for (int op = 0; op < NOPS; op++) hf[op] = frag(op, 0);
        pcur += KS * 2048;
      }
      // (the choice by output columns is for the single-pass form; a second instance of the loop here costs registers)
      if (NC > 1 || with_tail) k_loop(std::integral_constant<int, NOPS>{}, bias, scl);
      else k_loop(std::integral_constant<int, RB>{}, bias, scl);
    }
    // ---- epilogue of the strip: acc[rb][nb][v] is C[m0 + rb*32 + (v/4)*8 + g*4 + v%4][strip*64 + nb*32 + li] ----
    // Addresses are a uniform 64-bit base per 32 x 32 block plus a 32-bit lane offset (n_split is a multiple of 32,
    // so a block never straddles the two destinations).
    //
    // The stores of a strip must go out back to back.  Loads and stores of a wave complete in order on one counter;
    // with a per-row guard around every store the compiler can no longer count what is outstanding and waits for
    // the counter to reach zero before each store, i.e. for the acknowledgement of the previous one (150 ns each,
    // 10 us per strip).  So the guards are hoisted: a tile that lies within M (all but the last) and the
    // presence of a residual are decided once, uniformly, and the path taken is straight-line code.  The residual
    // may be the destination itself (in-place update); a block's residual values are requested before the
    // stores of the block before it, so that waiting for them does not wait for those stores.
    constexpr int CE = C_F32 ? 4 : 2;
    constexpr int NBLK = 2 * RB;  // 32 x 32 blocks of the strip: block = nb * RB + rb
    // ce: bytes per element of the block's destination (fp32 kernels may write their first destination as plain
    // fp16: GemmEpilogue::first_f16; the choice is uniform over a block)
    auto block_at = [&](int blk, char *&dblock, const char *&rblock, unsigned &dlane, unsigned &rlane, long &ld,
                        int &mb, int &ce) {
      const int nb = blk / RB, rb = blk % RB;
      const int nbase = strip * 64 + nb * 32;  // uniform
      const bool first = nbase < e.n_split;
      char *dst = (char *)(first ? e.dst0 : e.dst1);
      ld = first ? e.ld0 : e.ld1;
      const int ncb = first ? nbase : nbase - e.n_split;
      mb = m0 + rb * 32;  // uniform
      ce = (C_F32 && e.first_f16 && first) ? 2 : CE;
      dblock = dst + ((long)mb * ld + ncb) * ce;
      rblock = (const char *)e.resid + ((long)mb * e.ldr + nbase) * 4;
      dlane = (unsigned)((g * 4 * ld + li) * ce);
      rlane = (unsigned)((g * 4 * e.ldr + li) * 4);
      // the per-row offsets derived from these do not depend on the strip; computed once and kept, they would hold
      // dozens of registers through the main loop
      asm volatile("" : "+v"(dlane), "+v"(rlane));
    };
    auto finish = [&](int blk, int v, float r) -> float {
      float val = (acc[blk % RB][blk / RB][v] + bias[blk / RB]) * scl[blk / RB];
      if (e.relu) val = fmaxf(val, 0.f);
      return val + r;
    };
    auto put = [&](char *at_, float val, int ce) {
      if (C_F32 && ce == 2) {
        *(_Float16 *)at_ = (_Float16)val;
      } else if (C_F32) {
        if (RB == 2) __builtin_nontemporal_store(val, (float *)at_);
        else *(float *)at_ = val;
      } else {
        const _Float16 hi = (_Float16)val;
        *(_Float16 *)at_ = hi;  // 64 bytes per row and instruction: the other half of the line follows, keep it cached
        if (e.dst_lo_offset) *((_Float16 *)at_ + e.dst_lo_offset) = (_Float16)(val - (float)hi);
      }
    };
    // The projections that follow a LayerNorm add no residual, and the others all do: the straight-line path is
    // compiled for that case only; anything else takes the guarded path below.
    constexpr bool RESID = !LN;
    if (__builtin_expect(m0 + TM <= M && RESID == (e.resid != nullptr), 1)) {
      float res[RESID ? 2 : 1][16];
      auto request = [&](int blk) {
        char *dblock; const char *rblock; unsigned dlane, rlane; long ld; int mb, ce;
        block_at(blk, dblock, rblock, dlane, rlane, ld, mb, ce);
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const int r = (v >> 2) * 8 + (v & 3);
          const float *rp = (const float *)(rblock + (rlane + (unsigned)(r * e.ldr * 4)));
          res[blk & 1][v] = RB == 2 ? __builtin_nontemporal_load(rp) : *rp;
        }
      };
      if (RESID) request(0);
#pragma unroll
      for (int blk = 0; blk < NBLK; blk++) {
        __builtin_amdgcn_sched_barrier(0);  // one block at a time: bounds the loads and addresses in flight
        if (RESID && blk + 1 < NBLK) request(blk + 1);
        __builtin_amdgcn_sched_barrier(0);
        char *dblock; const char *rblock; unsigned dlane, rlane; long ld; int mb, ce;
        block_at(blk, dblock, rblock, dlane, rlane, ld, mb, ce);
        if (C_F32 && ce == 2) {  // uniform: the stores of a block stay straight-line code of one kind
#pragma unroll
          for (int v = 0; v < 16; v++) {
            const int r = (v >> 2) * 8 + (v & 3);
            put(dblock + (dlane + (unsigned)(r * ld * 2)), finish(blk, v, RESID ? res[blk & 1][v] : 0.f), 2);
          }
        } else {
#pragma unroll
          for (int v = 0; v < 16; v++) {
            const int r = (v >> 2) * 8 + (v & 3);
            put(dblock + (dlane + (unsigned)(r * ld * CE)), finish(blk, v, RESID ? res[blk & 1][v] : 0.f), CE);
          }
        }
      }
    } else {
      // the last row tile (or the unusual residual case): every row is checked against M
#pragma unroll
      for (int blk = 0; blk < NBLK; blk++) {
        __builtin_amdgcn_sched_barrier(0);
        char *dblock; const char *rblock; unsigned dlane, rlane; long ld; int mb, ce;
        block_at(blk, dblock, rblock, dlane, rlane, ld, mb, ce);
        // read the 16 residual values of the block first, then compute and store
        float res[16];
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const int r = (v >> 2) * 8 + (v & 3);
          res[v] = (e.resid && mb + r + g * 4 < M) ? *(const float *)(rblock + (rlane + (unsigned)(r * e.ldr * 4))) : 0.f;
        }
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const int r = (v >> 2) * 8 + (v & 3);
          if (mb + r + g * 4 >= M) continue;
          put(dblock + (dlane + (unsigned)(r * ld * ce)), finish(blk, v, res[v]), ce);
        }
      }
      // Nothing of this path may be left in flight at the end of the iteration: what is pending here (loads into
      // registers that the other path reuses) is also assumed pending there, and costs it a full wait per strip.
      __builtin_amdgcn_s_waitcnt(0x0F70);
    }
  }
}

template <int RB, int K, bool C_F32, bool LN, bool TAIL, int NC = 1>
static hipError_t gs_launch(const _Float16 *A, const _Float16 *A_lo, long lda, int M, const _Float16 *Wp, int N,
                            const GemmEpilogue &e, const GemmLayerNorm &ln, hipStream_t s) {
  auto kern = gemm_stream_kernel<RB, K, C_F32, LN, TAIL, NC>;
  const size_t lds = (size_t)(TAIL ? 64 : 32) * RB * (K + 8) * 2;
  // raising the dynamic LDS limit is per kernel, once per process (several host threads may get here at once)
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [&] {
    attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  });
  if (attr_err != hipSuccess) return attr_err;
  const int row_tiles = (M + 32 * RB - 1) / (32 * RB), NS = N / 64;
  // enough workgroups for the chip: split the strips of a row tile over several workgroups as long as every wave
  // of a workgroup still gets a strip and the grid stays within a few rounds
  int col_groups = 1;
  for (int cg = NS / GS_WAVES; cg > 1; cg--)
    if (NS % cg == 0 && (long)row_tiles * cg <= 1024) {
      col_groups = cg;
      break;
    }
  if (NC > 1) col_groups = NS / GS_WAVES;  // several passes: exactly one strip per wave
  hipLaunchKernelGGL(kern, dim3(row_tiles * col_groups), dim3(GS_WAVES * 64), lds, s, A, A_lo, lda, M, Wp, N, col_groups, e,
                     ln);
  return hipGetLastError();
}

template <bool LN>
static hipError_t gs_dispatch(bool c_f32, const _Float16 *A, const _Float16 *A_lo, long lda, const _Float16 *Wp, int M,
                              int N, int K, const GemmEpilogue &e, const GemmLayerNorm &ln, bool tail, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (!gemm_stream_supported(N, K) || e.n_split % 32 != 0) return hipErrorInvalidValue;
  const bool small = M <= 8192;  // 32-row tiles: twice the workgroups
#define NT_GS_CASE(RB_, K_, CF_)                                                                                       \
  if (small == (RB_ == 1) && K == K_ && c_f32 == CF_)                                                                  \
    return tail ? gs_launch<RB_, K_, CF_, LN, true>(A, A_lo, lda, M, Wp, N, e, ln, s)                                  \
                : gs_launch<RB_, K_, CF_, LN, false>(A, A_lo, lda, M, Wp, N, e, ln, s);
  NT_GS_CASE(1, 512, true) NT_GS_CASE(1, 512, false) NT_GS_CASE(2, 512, true) NT_GS_CASE(2, 512, false)
  NT_GS_CASE(1, 256, true) NT_GS_CASE(1, 256, false) NT_GS_CASE(2, 256, true) NT_GS_CASE(2, 256, false)
#undef NT_GS_CASE
  return hipErrorInvalidValue;
}

// K = 1024 / 2048 in passes over a 512-wide tile; N a multiple of 512 (one strip per wave and column group)
bool gemm_stream_k_supported(int N, int K) { return (K == 1024 || K == 2048) && N >= 512 && N % 512 == 0; }

hipError_t launch_gemm_stream_k(bool c_f32, const _Float16 *A, const _Float16 *A_lo, long lda, const _Float16 *Wp, int M,
                                int N, int K, const GemmEpilogue &e, hipStream_t s, bool tail) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (!gemm_stream_k_supported(N, K) || e.n_split % 32 != 0) return hipErrorInvalidValue;
  tail = tail && A_lo != nullptr;
  const GemmLayerNorm ln{};
#define NT_GSK_CASE(NC_, CF_, TL_)                        \
  if (K == 512 * NC_ && c_f32 == CF_ && tail == TL_)      \
    return M <= 8192 ? gs_launch<1, 512, CF_, false, TL_, NC_>(A, A_lo, lda, M, Wp, N, e, ln, s) \
                     : gs_launch<2, 512, CF_, false, TL_, NC_>(A, A_lo, lda, M, Wp, N, e, ln, s);
  NT_GSK_CASE(2, true, true) NT_GSK_CASE(2, true, false) NT_GSK_CASE(4, true, true) NT_GSK_CASE(4, true, false)
#undef NT_GSK_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_gemm_stream(bool c_f32, const _Float16 *A, const _Float16 *A_lo, long lda, const _Float16 *Wp, int M,
                              int N, int K, const GemmEpilogue &e, hipStream_t s, bool tail) {
  return gs_dispatch<false>(c_f32, A, A_lo, lda, Wp, M, N, K, e, GemmLayerNorm{}, tail && A_lo != nullptr, s);
}

hipError_t launch_gemm_stream_ln(bool c_f32, const float *X, long ldx, const GemmLayerNorm &ln, const _Float16 *Wp, int M,
                                 int N, int K, const GemmEpilogue &e, hipStream_t s, bool tail) {
  return gs_dispatch<true>(c_f32, (const _Float16 *)X, nullptr, ldx, Wp, M, N, K, e, ln, tail, s);
}

}  // namespace nt
