// Output projection fused with the row arg-max, streaming form (gfx950).
//
// The log-softmax of the output layer is not needed for greedy search (Sec. 3.3 "Graph
// Optimization"); here the logits never reach memory at all: every lane keeps the running
// largest logit of its rows while the vocabulary streams past.
//
// Shape of the problem: a few hundred to a few thousand rows of h (the decoder states of one
// step) against a 32,000 x 512 matrix that never changes.  A tiled GEMM stages both operands
// through the LDS and is bound by LDS traffic there (two operand tiles written and read for every
// 64 MFMAs).  Here the roles are fixed instead:
//   * a workgroup keeps its tile of h (128 rows, or 64 rows as head + tail planes) in the LDS for
//     its whole life: 130 KiB, filled once, straight from global memory (global_load ... lds);
//   * the output matrix is stored at load time in MFMA fragment order, so a wave fetches a
//     fragment with one fully coalesced 1 KiB load directly into the registers the MFMA reads:
//     no LDS write, no barrier and no address arithmetic in the main loop (buffer loads with a
//     scalar offset; a read past the end returns zeros instead of faulting);
//   * a wave owns a strip of 64 vocabulary entries at a time and all rows of the tile: 8 MFMAs per
//     16-wide k-step against 4 LDS fragment reads and 2 global fragment loads; the W fragments
//     run SL - 1 k-steps ahead of their use in a ring of registers;
//   * the MFMA operands are swapped (W is the row operand), so a lane owns one row of h and its
//     accumulator registers run along the vocabulary: the arg-max fold is in-lane.
// Workgroups that share a vocabulary range are placed on the same XCD (ids are dealt round-robin
// to the 8 XCDs), so the range is pulled into one L2 only and re-read from there.
//
// Fragment order of Wp: [strip = v / 64][ks = k / 16][nb = (v % 64) / 32][lane][8 halfs] with
// lane = v % 32 + 32 * ((k % 16) / 8): lane l of the MFMA row operand holds W[v = l % 32][k = 8 * (l / 32) .. + 7].
#include "nt_kernels.h"

#include <mutex>
#include <type_traits>

namespace nt {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int VS_ROWS = 128;  // LDS fragment rows per tile (exact variant: 64 matrix rows x 2 planes)
constexpr int VS_WAVES = 8;
constexpr int VS_CUS_PER_XCD = 32;
// Ranges of the vocabulary for the head+tail kernel that serves steps of fewer than 512 rows.  64 ranges are 7.8 strips
// each, one per wave; more ranges only spread the same strips over more CUs with idle waves (up to 256 workgroups of
// two busy waves), as fast for a launch alone but in the way of the other pipeline lanes' kernels: 64 instead of 256
// gave +8 % on a 4,096-token budget with four lanes and the same with one (32: +9 % and -7 %).
constexpr int VS_EXACT_MAX_RANGES = 64;

bool vocab_stream_supported(int K) { return K == 256 || K == 512; }

size_t vocab_pack_bytes(int N, int K) { return (size_t)((N + 63) / 64) * 64 * K * 2; }

void vocab_pack(const _Float16 *Wt, int N, int K, _Float16 *dst) {
  const int NS = (N + 63) / 64, KS = K / 16;
  for (int strip = 0; strip < NS; strip++)
    for (int ks = 0; ks < KS; ks++)
      for (int nb = 0; nb < 2; nb++)
        for (int lane = 0; lane < 64; lane++) {
          const int v = strip * 64 + nb * 32 + (lane & 31), k = ks * 16 + (lane >> 5) * 8;
          _Float16 *o = dst + ((((size_t)strip * KS + ks) * 2 + nb) * 64 + lane) * 8;
          for (int e = 0; e < 8; e++) o[e] = v < N ? Wt[(size_t)v * K + k + e] : (_Float16)0.f;
        }
}

// Work split: tiles of rows x G ranges of the vocabulary, one workgroup each, G chosen so that one
// round of workgroups fills the chip.  The list of (range, tile) pairs, range-major, is cut into
// 8 equal pieces, one per XCD: the tiles of one range then sit on one XCD (two at a piece boundary).
struct VsSplit {
  int m_tiles, G, per_xcd;
};
static VsSplit vs_split(int M, int tile_m, int max_ranges) {
  VsSplit p;
  p.m_tiles = (M + tile_m - 1) / tile_m;
  if (p.m_tiles < 1) p.m_tiles = 1;
  p.G = (8 * VS_CUS_PER_XCD) / p.m_tiles;
  if (p.G < 1) p.G = 1;
  if (p.G > max_ranges) p.G = max_ranges;
  p.per_xcd = (p.m_tiles * p.G + 7) / 8;
  return p;
}

// EXACT = false ("single pass"): 128 rows per tile, logits from the head plane only; besides the partial keys the
//   runner-up logit of every range goes to ps, so that the caller can certify the arg-max.
// EXACT = true: 64 rows per tile (32 for gathered rows, which are few), logits from the head/tail plane pair (both
//   multiplied with the same W fragment into one accumulator).  Either every row m < M is processed and partial keys go to
//   pk[m * G + range], or (row_map != nullptr) the rows row_map[0 .. *count) are gathered, every workgroup walks
//   all their tiles, and each result is folded into final_key[slot] with a 64-bit atomic max
//   (order-independent, hence still deterministic).
template <bool EXACT, int K, bool GATHER>
__global__ __launch_bounds__(VS_WAVES * 64) void vocab_stream_kernel(const _Float16 *__restrict__ h_hi,
                                                                    const _Float16 *__restrict__ h_lo, long ldh,
                                                                    const int *__restrict__ row_map,
                                                                    const int *__restrict__ count, int M,
                                                                    const _Float16 *__restrict__ Wp, int N, int m_tiles,
                                                                    int G, int per_xcd, unsigned long long *__restrict__ pk,
                                                                    float *__restrict__ ps,
                                                                    unsigned long long *__restrict__ final_key,
                                                                    const unsigned long long *__restrict__ need_mask,
                                                                    int mask_ranges) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  _Float16 *sh = (_Float16 *)smem;
  constexpr int NACC = EXACT ? (GATHER ? 1 : 2) : 4;  // 32-row blocks of h per tile
  constexpr int NW = VS_WAVES;
  constexpr int TILE_M = 32 * NACC;
  constexpr int FR = EXACT ? 2 * TILE_M : TILE_M;  // fragment rows in the LDS: head rows, then tail rows
  constexpr int NOP = FR / 32;
  constexpr int LD = K + 8;                 // halfs per LDS row: the 16 B pad keeps the fragment reads conflict-free
  constexpr int KS = K / 16;
  // register slots of W fragments per wave; the lookahead is SL - 1 k-steps (the single-pass variant has 128
  // accumulator registers and no room for more than four slots)
  constexpr int SL = EXACT ? 8 : 4;
  static_assert(KS % SL == 0, "the ring of W slots must divide the k-steps of a strip");
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int total = m_tiles * G;
  const int idx = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  {
    const int end = ((blockIdx.x & 7) + 1) * per_xcd;
    if (idx >= (end < total ? end : total)) return;  // uniform over the workgroup
  }
  const int gi = idx / m_tiles, mt = idx % m_tiles;
  const int NS = (N + 63) >> 6;
  const int sb0 = gi * NS / G, sb1 = (gi + 1) * NS / G;  // G <= 256 and NS < 2^22: no overflow
  if (GATHER) M = *count;  // number of gathered rows, decided on the device
  // gathered rows of the current tile and their result slots (beyond the h tile and the per-wave results)
  int *sel_row = (int *)(smem + FR * LD * 2), *sel_slot = sel_row + 64, *wtot = sel_slot + 64;

  // W fragments come through a buffer resource: scalar offset per fragment, constant lane offset
  const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc((void *)Wp, 0, NS * 64 * K * 2, 0x00020000);
  const int wlane = lane * 16;
  auto wload = [&](int soff, int nb) -> half8 {
    u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(wrs, wlane + nb * 1024, soff, 0);
    return __builtin_bit_cast(half8, t);
  };

  // One tile: rows m0 .. m0 + TILE_M - 1 below Mlim (gathered: positions in sel_row / sel_slot).
  auto tile = [&](const int m0, const int Mlim) {
    half8 wb[SL][2];
    int strip = sb0 + wave;
    const bool have = strip < sb1;
    // ---- the h tile: global memory -> LDS.  Rows past M repeat row M - 1 (their results are never stored) ----
    if (K == 512) {
      // one wave instruction moves one row (1 KiB) without passing through registers
#pragma unroll
      for (int i = 0; i < FR / NW; i++) {
        const int R = wave + NW * i;
        const int rr = EXACT ? (R & (TILE_M - 1)) : R;
        const _Float16 *src = (EXACT && R >= TILE_M) ? h_lo : h_hi;
        int m = m0 + rr;
        m = m < Mlim ? m : Mlim - 1;
        const long gm = GATHER ? __builtin_amdgcn_readfirstlane(sel_row[m]) : m;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + gm * ldh + lane * 8),
                                         (__attribute__((address_space(3))) void *)(sh + R * LD), 16, 0, 0);
      }
    } else {
      constexpr int CPR = K / 8, PER_T = FR * CPR / (NW * 64);
      u32x4 fr[PER_T];
#pragma unroll
      for (int i = 0; i < PER_T; i++) {
        const int c = tid + NW * 64 * i, R = c / CPR, kc = c % CPR;
        const int rr = EXACT ? (R & (TILE_M - 1)) : R;
        const _Float16 *src = (EXACT && R >= TILE_M) ? h_lo : h_hi;
        int m = m0 + rr;
        m = m < Mlim ? m : Mlim - 1;
        const long gm = GATHER ? sel_row[m] : m;
        fr[i] = *(const u32x4 *)(src + gm * ldh + kc * 8);
      }
#pragma unroll
      for (int i = 0; i < PER_T; i++) {
        const int c = tid + NW * 64 * i, R = c / CPR, kc = c % CPR;
        *(u32x4 *)(sh + R * LD + kc * 8) = fr[i];
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
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's rows have landed in the LDS before the barrier
    __syncthreads();

    // running state per 32-row block: largest logit, runner-up, and where the largest sits: strip * 32 + position
    // code (inside the fold of a strip the code is written without the strip, which is added when the strip is done)
    float rmax[NACC], rsec[NACC];
    int rcode[NACC];
#pragma unroll
    for (int a = 0; a < NACC; a++) {
      rmax[a] = -INFINITY;
      rsec[a] = -INFINITY;
      rcode[a] = 0;
    }

    if (have) {
      floatx16 acc[NACC][2];
      const _Float16 *hrow = sh + li * LD + g * 8;
      int off2 = 64 * LD;  // second base register: the byte offsets of fragment rows 64.. do not fit 16 bits
      asm volatile("" : "+v"(off2));
      const _Float16 *hrow2 = hrow + off2;
      half8 hf[NOP];
#pragma unroll
      for (int op = 0; op < NOP; op++) hf[op] = *(const half8 *)((op < 2 ? hrow : hrow2) + (op & 1) * 32 * LD);
      for (; strip < sb1; strip += NW) {
        const bool more = strip + NW < sb1;
        const int pcur = strip * (KS * 2048);
        const int pnext = (more ? strip + NW : strip) * (KS * 2048);
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
          // the lookahead runs into the next strip of this wave at the end of a strip (at the very end it
          // re-reads this strip: valid memory, unused data)
          const int tgt = ks + SL - 1;
          const int pf = tgt < KS ? pcur + tgt * 2048 : pnext + (tgt - KS) * 2048;
          const int ksn = (ks + 1) % KS;
#pragma unroll
          for (int op = 0; op < NOP; op++) {
#pragma unroll
            for (int nb = 0; nb < 2; nb++) {
              if (ks == 0 && op < NACC) {
                const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                acc[op % NACC][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wb[ks % SL][nb], hf[op], zero, 0, 0, 0);
              } else {
                acc[op % NACC][nb] =
                    __builtin_amdgcn_mfma_f32_32x32x16_f16(wb[ks % SL][nb], hf[op], acc[op % NACC][nb], 0, 0, 0);
              }
            }
            // refill what was just consumed: the h fragment of the next k-step and, once per k-step, the W
            // slot that the previous k-step used.  The scheduling barrier keeps this order: the compiler
            // would otherwise sink the loads next to their uses and lose the lookahead.
            hf[op] = *(const half8 *)((op < 2 ? hrow : hrow2) + (op & 1) * 32 * LD + ksn * 16);
            if (op == 0) {
              wb[tgt % SL][0] = wload(pf, 0);
              wb[tgt % SL][1] = wload(pf, 1);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // ---- strip done: fold its 64 logits per row into the running state ----
        auto fold = [&](auto masked_tag) {
          constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
          for (int a = 0; a < NACC; a++) {
            const float before = rmax[a];
#pragma unroll
            for (int nb = 0; nb < 2; nb++)
#pragma unroll
              for (int v = 0; v < 16; v++) {  // codes ascend with the column: on equal logits the lower column stays
                float val = acc[a][nb][v];
                if (MASKED) {
                  const int n = strip * 64 + nb * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
                  val = n < N ? val : -INFINITY;
                }
                if (!EXACT) rsec[a] = __builtin_amdgcn_fmed3f(rmax[a], rsec[a], val);
                const bool gt = val > rmax[a];
                rmax[a] = gt ? val : rmax[a];
                rcode[a] = gt ? (nb * 16 + v) : rcode[a];
              }
            rcode[a] = rmax[a] > before ? strip * 32 + rcode[a] : rcode[a];
          }
        };
        if (strip * 64 + 64 <= N) fold(std::false_type{}); else fold(std::true_type{});
      }
    }
    __syncthreads();  // every wave is done with the h tile: its LDS now carries the per-wave results
    unsigned long long *skey = (unsigned long long *)smem;  // [NW][TILE_M]
    float *ssec = (float *)(smem + NW * TILE_M * 8);  // [NW][TILE_M]
#pragma unroll
    for (int a = 0; a < NACC; a++) {
      const int c = rcode[a], v = c & 15;
      const int n = (c >> 5) * 64 + ((c >> 4) & 1) * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
      unsigned long long key = (rmax[a] == -INFINITY) ? 0ull : argmax_key(rmax[a], n);
      float second = rsec[a];
      // the two lane groups hold interleaved columns of the same row: merge them
      const unsigned long long okey = shfl_xor_u64(key, 32);
      const float osec = __shfl_xor(second, 32, 64);
      const bool take = okey > key;
      const unsigned long long loser = take ? key : okey;
      if (!EXACT) second = fmaxf(fmaxf(second, osec), loser ? key_value(loser) : -INFINITY);
      key = take ? okey : key;
      if (g == 0) {
        skey[wave * TILE_M + a * 32 + li] = key;
        ssec[wave * TILE_M + a * 32 + li] = second;
      }
    }
    __syncthreads();
    if (tid < TILE_M) {
      unsigned long long best = 0ull;
      float second = -INFINITY;
#pragma unroll
      for (int w = 0; w < NW; w++) {
        const unsigned long long k = skey[w * TILE_M + tid];
        const float s2 = ssec[w * TILE_M + tid];
        const bool take = k > best;
        const unsigned long long loser = take ? best : k;
        second = fmaxf(fmaxf(second, s2), loser ? key_value(loser) : -INFINITY);
        best = take ? k : best;
      }
      const int m = m0 + tid;
      if (m < Mlim) {
        if (GATHER) {
          atomicMax(final_key + sel_slot[m], best);
        } else {
          pk[(long)m * G + gi] = best;
          if (!EXACT) ps[(long)m * G + gi] = second;
        }
      }
    }
    __syncthreads();  // before the next tile overwrites the LDS
  };

  if (!GATHER) {
    for (int m0 = mt * TILE_M; m0 < M; m0 += m_tiles * TILE_M) tile(m0, M);
    return;
  }
  // Gathered rows: the caller has marked, per row, which of mask_ranges equal ranges of the vocabulary can hold its
  // arg-max at all; this workgroup takes the rows whose marks meet its own strips.  The list is walked 512 entries
  // at a time; the wanted entries are ranked with a workgroup prefix sum and processed 32 rows per tile.
  // range r of the caller covers strips [r * NS / mask_ranges, (r + 1) * NS / mask_ranges): strip s lies in range
  // ((s + 1) * mask_ranges - 1) / NS
  unsigned long long mine = 0ull;
  if (sb1 > sb0) {
    const int r_lo = ((sb0 + 1) * mask_ranges - 1) / NS, r_hi = (sb1 * mask_ranges - 1) / NS;
    mine = (r_hi >= 63 ? ~0ull : (1ull << (r_hi + 1)) - 1ull) & ~((1ull << r_lo) - 1ull);
  }
  for (int c0 = 0; c0 < M; c0 += NW * 64) {
    const int i = c0 + tid;
    const bool need = i < M && (need_mask[i] & mine) != 0ull;
    const unsigned long long bal = __ballot(need);
    if (lane == 0) wtot[wave] = __popcll(bal);
    __syncthreads();
    int rank = __popcll(bal & ((1ull << lane) - 1ull)), total = 0;
#pragma unroll
    for (int w = 0; w < NW; w++) {
      const int c = wtot[w];
      rank += w < wave ? c : 0;
      total += c;
    }
    for (int t0 = 0; t0 < total; t0 += TILE_M) {  // total is uniform over the workgroup
      if (need && rank >= t0 && rank < t0 + TILE_M) {
        sel_row[rank - t0] = row_map[i];
        sel_slot[rank - t0] = i;
      }
      __syncthreads();
      tile(0, total - t0 < TILE_M ? total - t0 : TILE_M);
    }
    __syncthreads();  // wtot is rewritten by the next chunk
  }
}

static size_t vs_lds_bytes(int K, int frag_rows) { return (size_t)frag_rows * (K + 8) * 2 + 1024; }

template <bool EXACT, int K, bool GATHER>
static hipError_t vs_launch(const _Float16 *h, const _Float16 *h_lo, long ldh, const int *row_map, const int *count, int M,
                            const _Float16 *Wp, int N, const VsSplit &p, unsigned long long *pk, float *ps,
                            unsigned long long *final_key, const unsigned long long *need_mask, int mask_ranges,
                            hipStream_t s) {
  auto kern = vocab_stream_kernel<EXACT, K, GATHER>;
  constexpr int FR = (EXACT && GATHER) ? 64 : VS_ROWS;  // as in the kernel
  // raising the dynamic LDS limit is per kernel, once per process (several host threads may get here at once)
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [&] {
    attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)vs_lds_bytes(K, FR));
  });
  if (attr_err != hipSuccess) return attr_err;
  hipLaunchKernelGGL(kern, dim3(8 * p.per_xcd), dim3(VS_WAVES * 64), vs_lds_bytes(K, FR), s, h, h_lo, ldh, row_map, count, M, Wp,
                     N, p.m_tiles, p.G, p.per_xcd, pk, ps, final_key, need_mask, mask_ranges);
  return hipGetLastError();
}

template <bool EXACT, bool GATHER>
static hipError_t vs_launch_k(const _Float16 *h, const _Float16 *h_lo, long ldh, const int *row_map, const int *count,
                              int M, const VocabWeights &w, const VsSplit &p, unsigned long long *pk, float *ps,
                              unsigned long long *final_key, const unsigned long long *need_mask, int mask_ranges,
                              hipStream_t s) {
  if (w.K == 512)
    return vs_launch<EXACT, 512, GATHER>(h, h_lo, ldh, row_map, count, M, w.Wp, w.N, p, pk, ps, final_key, need_mask,
                                         mask_ranges, s);
  if (w.K == 256)
    return vs_launch<EXACT, 256, GATHER>(h, h_lo, ldh, row_map, count, M, w.Wp, w.N, p, pk, ps, final_key, need_mask,
                                         mask_ranges, s);
  return hipErrorInvalidValue;
}

static bool use_stream(const VocabWeights &w) { return !w.force_tiled && w.Wp && vocab_stream_supported(w.K); }

int vocab_argmax_partials(const VocabWeights &w, int M, bool certified) {
  if (!use_stream(w)) return vocab_argmax_partials_tiled(M, w.N);
  return certified ? vs_split(M, 128, 64).G : vs_split(M, 64, VS_EXACT_MAX_RANGES).G;
}

hipError_t launch_vocab_argmax(const _Float16 *h, const _Float16 *h_lo, long ldh, const VocabWeights &w, int M,
                               unsigned long long *pk, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (!use_stream(w)) return launch_vocab_argmax_tiled(h, h_lo, ldh, w.Wt, M, w.N, w.K, pk, s);
  return vs_launch_k<true, false>(h, h_lo, ldh, nullptr, nullptr, M, w, vs_split(M, 64, VS_EXACT_MAX_RANGES), pk, nullptr, nullptr, nullptr, 0, s);
}

// Certified single-pass arg-max.  With h = hi + lo, the head-only logit l'(v) = hi . w_v differs
// from the head+tail logit by at most |lo . w_v| <= ||lo|| * max_v ||w_v||.  If the head-only
// winner leads the runner-up by more than twice that bound (plus a little slack for the fp32
// accumulation order) it is also the winner of the head+tail logits, and the second MFMA pass is
// not needed.  The few rows that fail the test (about 2 % with flat random logits) are collected
// and recomputed with both planes by the gathered variant.
hipError_t launch_vocab_argmax_certified(const _Float16 *h, const _Float16 *h_lo, long ldh, const VocabWeights &w, int M,
                                         const float *lo_norm, float w_norm_max, unsigned long long *pk, float *ps,
                                         int32_t *tok, int32_t *slot_of_row, int32_t *list, int32_t *count,
                                         unsigned long long *final_key, unsigned long long *need_mask, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (!use_stream(w))
    return launch_vocab_argmax_certified_tiled(h, h_lo, ldh, w.Wt, M, w.N, w.K, lo_norm, w_norm_max, pk, ps, tok,
                                               slot_of_row, list, count, final_key, need_mask, s);
  const VsSplit p = vs_split(M, 128, 64);  // at most 64 ranges: one bit each in the masks of the recompute
  hipError_t e = vs_launch_k<false, false>(h, h_lo, ldh, nullptr, nullptr, M, w, p, pk, ps, nullptr, nullptr, 0, s);
  if (e != hipSuccess) return e;
  e = launch_argmax_select(pk, ps, p.G, M, lo_norm, w_norm_max, tok, slot_of_row, list, count, final_key, need_mask, s);
  if (e != hipSuccess) return e;
  // recompute of the uncertified rows: their number is known on the device only, so each of 128 workgroups takes
  // a range of the vocabulary and those gathered rows that still have a candidate there (often none).  It is
  // little work, bound by the latency of one strip per wave: half the chip gives the shortest launch, and the
  // whole job runs as fast with it as with a quarter (measured among 32 ... 256 workgroups).
  VsSplit q;
  q.m_tiles = 1;
  q.G = 4 * VS_CUS_PER_XCD;
  q.per_xcd = VS_CUS_PER_XCD / 2;
  return vs_launch_k<true, true>(h, h_lo, ldh, list, count, M, w, q, nullptr, nullptr, final_key, need_mask, p.G, s);
}

}  // namespace nt
