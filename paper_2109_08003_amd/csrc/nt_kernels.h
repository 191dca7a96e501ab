// Internal launch interface between the host side of libnt and its gfx950 kernels.
// Every launcher validates nothing: the host code checks shapes before calling.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nt {

// ---- GEMM: C[M,N] = A[M,K] * Wt[N,K]^T, fp16 MFMA with fp32 accumulation -------------
// Epilogue, applied to acc (fp32):  v = acc + bias[n];  if (n < scale_cols) v *= scale;
// if (relu) v = max(v,0);  if (resid) v += resid[m*ldr+n];  then columns [0,n_split) go to
// dst0[m*ld0+n] and columns [n_split,N) to dst1[m*ld1+(n-n_split)].
// Flavour of a layer normalisation y = gamma * (x - mean) * r + beta.  Vanilla: r = 1 / sqrt(var + eps) with the
// biased variance.  L1-norm (Sec. 3.1 "FP16 Inference"): r = 1 / (sqrt(pi/2) * mean|x - mean| + eps), the scaled
// mean absolute deviation, which equals the standard deviation for normally distributed activations.
struct LnEps {
  float eps = 0.f;
  int l1 = 0;
};
#ifdef __HIPCC__
// what a row sums over its centred elements, and how the mean of those terms becomes the scale r
__device__ __forceinline__ float ln_term(float c, int l1) { return l1 ? fabsf(c) : c * c; }
__device__ __forceinline__ float ln_rscale(float mean_term, LnEps e) {
  return e.l1 ? 1.0f / (1.2533141373f * mean_term + e.eps) : 1.0f / sqrtf(mean_term + e.eps);
}
#endif

struct GemmEpilogue {
  const float *bias = nullptr;
  float scale = 1.f;
  int scale_cols = 0;
  int relu = 0;
  const float *resid = nullptr;
  long ldr = 0;
  void *dst0 = nullptr;
  long ld0 = 0;
  int n_split = 0;  // set to N when there is a single destination
  void *dst1 = nullptr;
  long ld1 = 0;
  // streaming kernels with a head/tail A operand: only the strips of 64 output columns that start in
  // [tail_col0, tail_col1) multiply the tail plane too (the others see fp16 activations: half the MFMA work)
  int tail_col0 = 0, tail_col1 = 1 << 30;
  int first_f16 = 0;       // streaming kernels with fp32 destinations: the first destination is plain fp16 instead
  long dst_lo_offset = 0;  // fp16 destinations only: if != 0 the tail fp16(v - fp16(v)) is also stored, this many
                           // elements after the head (the result becomes a head/tail plane pair)
};

// How the A operand is given (see nt_gemm.hip): one fp16 plane, a head/tail pair of fp16 planes
// (~22 significant bits, two MFMA passes), or fp32 that the kernel splits while staging.
enum AMode { A_F16 = 0, A_PLANES = 1, A_F32 = 2 };

// a_mode: AMode; A_lo is the tail plane for A_PLANES (ignored otherwise).  c_f32: destinations are
// fp32, else fp16.  K must be a multiple of 64; lda in elements.
// Wp (optional): the same weights in MFMA fragment order (vocab_pack layout); with A_PLANES and a supported
// shape the streaming kernel is used, and tail = false then leaves the tail plane out of the product.
hipError_t launch_gemm(int a_mode, bool c_f32, const void *A, const void *A_lo, long lda, const _Float16 *Wt, int M,
                       int N, int K, const GemmEpilogue &e, hipStream_t s, const _Float16 *Wp = nullptr, bool tail = true);

// Streaming form for K = 256 / 512 and N % 64 == 0 (nt_gemm_stream.hip): the A tile (head/tail planes) stays in
// the LDS, the weights stream through registers in fragment order.
struct GemmLayerNorm {
  const float *gamma = nullptr, *beta = nullptr;
  LnEps eps;
};
bool gemm_stream_supported(int N, int K);
// C = LayerNorm(X) * Wt^T: X [M][ldx] fp32 is normalised and split into planes while the tile is loaded
// The same with K = 1024 / 2048 (an FFN's second matrix), fp32 results: NC passes over a 512-wide tile of the planes,
// Wp = vocab_pack of Wt [N][K]; N a multiple of 512.
bool gemm_stream_k_supported(int N, int K);
hipError_t launch_gemm_stream_k(bool c_f32, const _Float16 *A, const _Float16 *A_lo, long lda, const _Float16 *Wp, int M,
                                int N, int K, const GemmEpilogue &e, hipStream_t s, bool tail = true);
// tail = false: only the head plane of A enters the product (fp16 activations: half the matrix-core work)
hipError_t launch_gemm_stream_ln(bool c_f32, const float *X, long ldx, const GemmLayerNorm &ln, const _Float16 *Wp, int M,
                                 int N, int K, const GemmEpilogue &e, hipStream_t s, bool tail = true);
hipError_t launch_gemm_stream(bool c_f32, const _Float16 *A, const _Float16 *A_lo, long lda, const _Float16 *Wp, int M,
                              int N, int K, const GemmEpilogue &e, hipStream_t s, bool tail = true);

// Decoder-step variant for small M (fp32 A and C): 32 x 32 tiles, whole-K operand panels loaded
// in one round trip.  If ln_g != nullptr the rows of A are LayerNorm-ed first (requires K to be
// the row width, 256 or 512).  K must be a multiple of 256.
bool skinny_gemm_supported(int K, bool with_ln);
hipError_t launch_skinny_gemm(const float *A, long lda, const _Float16 *Wt, int M, int N, int K, const float *ln_g,
                              const float *ln_b, LnEps ln_eps, const GemmEpilogue &e, hipStream_t s);

// ---- output projection fused with row arg-max ------------------------------------------
// For every row m < M: the largest of h[m,:] . W_out[v,:] over v < N, lowest v on ties, as packed
// keys.  Each workgroup reduces a range of the vocabulary; partial keys go to pk[m * n_partials + p].
//
// Key = (order-preserving bits of the fp32 logit) << 32 | (0xFFFFFFFF - v): the maximum key is the
// largest logit and, among equal logits, the lowest id.  Max over keys is associative and
// commutative, so the result does not depend on the tiling: deterministic without float atomics.
__device__ __forceinline__ unsigned long long argmax_key(float val, int v) {
  unsigned int b = __float_as_uint(val);
  b = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
  return ((unsigned long long)b << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned int)v);
}
__device__ __forceinline__ float key_value(unsigned long long key) {
  unsigned int b = (unsigned int)(key >> 32);
  b = (b & 0x80000000u) ? (b & 0x7FFFFFFFu) : ~b;
  return __uint_as_float(b);
}
__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long x, int mask) {
  unsigned int lo = (unsigned int)x, hi = (unsigned int)(x >> 32);
  lo = __shfl_xor(lo, mask, 64);
  hi = __shfl_xor(hi, mask, 64);
  return ((unsigned long long)hi << 32) | lo;
}

// The output matrix in two layouts: Wt [N][K] row-major, and Wp in MFMA fragment order (see
// vocab_pack_bytes / vocab_pack; built once at load time).  The streaming kernels need K = 256 or
// 512 (vocab_stream_supported); other widths, or force_tiled, take the tiled kernels on Wt.
struct VocabWeights {
  const _Float16 *Wt = nullptr;
  const _Float16 *Wp = nullptr;
  int N = 0, K = 0;
  bool force_tiled = false;
};
bool vocab_stream_supported(int K);
size_t vocab_pack_bytes(int N, int K);
// host: dst[vocab_pack_bytes] <- fragment order of Wt [N][K]
void vocab_pack(const _Float16 *Wt, int N, int K, _Float16 *dst);

// n_partials of the launch configuration used with M rows (exact: head + tail planes; certified:
// head plane first).  Never more than max(32768, M) / M per row.
int vocab_argmax_partials(const VocabWeights &w, int M, bool certified);
// h is a head/tail pair of fp16 planes.
hipError_t launch_vocab_argmax(const _Float16 *h, const _Float16 *h_lo, long ldh, const VocabWeights &w, int M,
                               unsigned long long *pk, hipStream_t s);

// Same result as launch_vocab_argmax, usually at half the MFMA work: a head-only pass whose winner is
// certified against a rigorous bound on the contribution of the tail (lo_norm[m] = ||tail of row m||,
// w_norm_max = max_v ||W_out[v,:]||); rows that cannot be certified are recomputed with both planes.
// Results: tok[m] when slot_of_row[m] < 0, else the key in final_key[slot_of_row[m]].
// *count must be 0 when the call starts (the step-begin kernel clears it).  need_mask [M]: scratch, per recompute
// slot the ranges of the vocabulary that can still hold the arg-max (the recompute skips the others).
hipError_t launch_vocab_argmax_certified(const _Float16 *h, const _Float16 *h_lo, long ldh, const VocabWeights &w, int M,
                                         const float *lo_norm, float w_norm_max, unsigned long long *pk, float *ps,
                                         int32_t *tok, int32_t *slot_of_row, int32_t *list, int32_t *count,
                                         unsigned long long *final_key, unsigned long long *need_mask, hipStream_t s);

// the tiled implementations (nt_gemm.hip) and the certification kernel shared by both
int vocab_argmax_partials_tiled(int M, int N);
hipError_t launch_vocab_argmax_tiled(const _Float16 *h, const _Float16 *h_lo, long ldh, const _Float16 *Wt, int M, int N,
                                     int K, unsigned long long *pk, hipStream_t s);
hipError_t launch_vocab_argmax_certified_tiled(const _Float16 *h, const _Float16 *h_lo, long ldh, const _Float16 *Wt, int M,
                                               int N, int K, const float *lo_norm, float w_norm_max,
                                               unsigned long long *pk, float *ps, int32_t *tok, int32_t *slot_of_row,
                                               int32_t *list, int32_t *count, unsigned long long *final_key,
                                               unsigned long long *need_mask, hipStream_t s);
hipError_t launch_argmax_select(const unsigned long long *pk, const float *ps, int n_partials, int M, const float *lo_norm,
                                float w_norm_max, int32_t *tok, int32_t *slot_of_row, int32_t *list, int32_t *count,
                                unsigned long long *final_key, unsigned long long *need_mask, hipStream_t s);

// ---- 8-bit output layer fused with the row arg-max (nt_vocab_q8.hip; Sec. 3.2, Eq. 3-6) ----------------------------
bool vocab_q8_supported(int K);
size_t vocab_q8_pack_bytes(int N, int K);
size_t vocab_q8_const_bytes(int N);
// Host: quantise Wt [N][K] per vocabulary entry and lay the codes out in MFMA fragment order, the per-entry
// constants (scale, zero point, sum of codes - K * zero point) in accumulator order.
void vocab_q8_pack(const _Float16 *Wt, int N, int K, int8_t *codes, void *consts);
// Host: Eq. 3, 4 for one vocabulary entry (what vocab_q8_pack applies to every row)
void vocab_q8_quantize_row(const _Float16 *w, int K, int8_t *q, float *scale, int32_t *zero);
// x [M][d] fp32 -> [LayerNorm if gamma != nullptr ->] unsigned 8-bit codes per row, stored as signed bytes
// (code - 128) in codes [M][d]; a_scale [M]; c [M] = 128 - zero point; sa [M] = sum of the signed bytes.  d = 256 / 512.
hipError_t launch_q8_rows(const float *x, int M, int d, const float *gamma, const float *beta, LnEps eps, int8_t *codes,
                          float *a_scale, int32_t *c_out, int32_t *sa_out, hipStream_t s);
// partial keys per row that launch_vocab_q8_argmax writes for M rows
int vocab_q8_partials(int M);
// pk[m * vocab_q8_partials(M) + p]: largest b_scale[v] * float(I[m][v]) of a range of the vocabulary, as packed keys
hipError_t launch_vocab_q8_argmax(const int8_t *codes, const int32_t *c_row, const int32_t *sa_row, int M,
                                  const int8_t *Wq, const void *consts, int N, int K, unsigned long long *pk,
                                  hipStream_t s);
// logits[m * ld + v] = a_scale[m] * (b_scale[v] * float(I[m][v])) by the definition (debug / teacher-forced path)
hipError_t launch_q8_logits(const int8_t *codes, const float *a_scale, const int32_t *c_row, int M, const int8_t *Wq,
                            const void *consts, int N, int K, float *logits, long ld, hipStream_t s);

// ---- row kernels --------------------------------------------------------------------
// x[r,:] = sqrt(d) * E[id] + PE[pos]; rows r = b*S + s, pos = s.  Out-of-range ids are
// replaced by pad_id and flags[0] is set.  Also clamps len into [1,S] -> len_out.
hipError_t launch_embed_src(const int32_t *src, const int32_t *len, int32_t *len_out, int B, int S, int d, int vocab,
                            int pad_id, const _Float16 *E, const float *pe, float *x, int32_t *flags, hipStream_t s);

// out = gamma * (x - mean) * r + beta per row of d, r as LnEps says.
enum OutMode { OUT_F16 = 0, OUT_F32 = 1, OUT_PLANES = 2 };  // OUT_PLANES: fp16 head at out, tail at out + lo_offset
// lo_norm (OUT_PLANES only, optional): receives the Euclidean norm of every row's tail plane.
hipError_t launch_layer_norm(const float *x, int M, int d, const float *gamma, const float *beta, LnEps eps,
                             void *out, int out_mode, long lo_offset, hipStream_t s, float *lo_norm = nullptr);

// out[i] = hi[i] + lo[i] (debug readback of a head/tail plane pair)
hipError_t launch_planes_to_float(const _Float16 *hi, const _Float16 *lo, float *out, long n, hipStream_t s);

// fp16 -> fp32 copy (debug readback)
hipError_t launch_half_to_float(const _Float16 *in, float *out, long n, hipStream_t s);
hipError_t launch_fill_i32(int32_t *p, long n, int32_t v, hipStream_t s);
// one wave that busy-waits for `ticks` periods of the 100 MHz wall clock (bounded); sink is never written
hipError_t launch_spin(long ticks, int *sink, hipStream_t s);

// Probes: `blocks` workgroups of four waves, each wave `iters` x 4 independent 32x32x16 fp16 MFMAs (2 * 32 * 32 * 16
// flops each); a grid-stride read of `bytes` bytes (a multiple of 16).  sink is never written.
// workgroups of eight waves, iters (a multiple of 8) rounds of eight independent 32x32x16 fp16 MFMAs per wave
hipError_t launch_probe_mfma(int iters, int blocks, bool random_operands, float *sink, hipStream_t s);
hipError_t launch_probe_read(const void *src, long bytes, float *sink, hipStream_t s);
// reads bytes of buf and writes them back in place (the contents do not change)
hipError_t launch_probe_copy(void *buf, long bytes, hipStream_t s);

// Start of decoder step t for rows [0, rows_prev): (1) if t > 0, reduce the arg-max partials of
// step t-1 and store the token in out[r*out_ld + t-1]; (2) for rows < rows_now: take the input
// token (BOS at t = 0, forced[r*forced_ld + t] if forced, else the token just reduced),
// z = sqrt(d) * E[y] + PE[t], and a = LayerNorm(z) unless a == nullptr.
struct StepBeginArgs {
  int t, rows_prev, rows_now, d, vocab, bos_id, pad_id;
  const unsigned long long *pk;
  int n_partials;
  int32_t *out;
  long out_ld;
  const int32_t *forced;
  long forced_ld;
  const _Float16 *E;
  const float *pe;
  const float *gamma, *beta;
  LnEps eps;
  float *z, *a;
  int32_t *flags;
  // certified arg-max of the previous step (prev_cert != 0): token = tok[r], or the key in
  // final_key[slot_of_row[r]] when the row had to be recomputed; cert_count is cleared for this step
  int prev_cert;
  const int32_t *tok, *slot_of_row;
  const unsigned long long *final_key;
  int32_t *cert_count;
};
hipError_t launch_step_begin(const StepBeginArgs &a, hipStream_t s);

// ---- fused decoder-step kernels (nt_decoder.hip), model widths 256 / 512 ----------------------------------------
bool dec_fused_supported(int K);
// Step start fused into the first layer's self-attention projection: tokens as launch_step_begin takes them (or
// tok_in[r] directly when tok_in != nullptr: the EOS mode's dense rows), z = sqrt(d) * E[y] + PE[t] written to sb.z,
// LayerNorm (sb.gamma, sb.beta), then [q|k|v] = a * Wp^T with epilogue e (N columns; Wp in MFMA fragment order).
// sb.a is ignored.  Rows in [rows_now, rows_prev) only have their token collected.
struct DecQkvArgs {
  StepBeginArgs sb;
  const int32_t *tok_in;
  const _Float16 *Wp;
  int N;
  GemmEpilogue e;
};
hipError_t launch_dec_qkv(const DecQkvArgs &a, hipStream_t s);
// One launch for: z' = A * W1^T + b1 + z (A: head/tail planes [M][lda], W1 [K][K] in fragment order; z' is written
// back to z if write_z), y = LayerNorm(z'), then either (W2p == nullptr) y as head/tail planes at h_hi /
// h_hi + h_lo_offset with row stride K, plus lo_norm[m] = ||tail|| (optional), or C = y * W2^T with epilogue e2
// (N2 columns, fp32 or fp16 destinations).
struct DecChainArgs {
  const _Float16 *A_hi, *A_lo;
  long lda;
  const _Float16 *W1p;
  const float *b1;
  float *z;
  long ldz;
  int write_z;
  int M;
  const float *gamma, *beta;
  LnEps eps;
  _Float16 *h_hi;
  long h_lo_offset;
  float *lo_norm;
  const _Float16 *W2p;
  int N2;
  GemmEpilogue e2;
};
hipError_t launch_dec_chain(const DecChainArgs &a, int K, bool c2_f32, hipStream_t s);

// Start of decoder step t when sentences end at EOS (Sec. 3.3 "Greedy Search"): the rows still decoding are kept
// as a dense prefix.  Dense row r of a step belongs to batch row origin[r] (-1: no row; such rows compute on the
// padding token and store nothing).  Three launches:
//   collect  (t > 0) token of step t-1 for every previous dense row -> out[b][t-1]; a row ends when the token is
//            eos_id or when it has cap[b] tokens, and then gets out_len[b] = t
//   compact  stable compaction of the rows that go on -> origin / tok_in of step t, their count -> *live and, if
//            progress != nullptr, progress_tag | t << 32 | count into that host-visible word.  At t == 0 the rows
//            with cap > 0 start with bos_id.
//   embed    z[r] = sqrt(d) * E[tok_in[r]] + PE[t] for r < rows_now (tok_in is pad_id where origin[r] < 0)
// rows_prev: dense rows of step t-1 (B at t == 0); rows_now <= rows_prev: dense rows step t will run on, an upper
// bound of the count the compaction finds.
struct EosStepArgs {
  int t, rows_prev, rows_now, d, vocab, bos_id, pad_id, eos_id;
  // arg-max result of step t-1, as in StepBeginArgs
  const unsigned long long *pk;
  int n_partials, prev_cert;
  const int32_t *tok, *slot_of_row;
  const unsigned long long *final_key;
  int32_t *cert_count;
  int32_t *out;
  long out_ld;
  int32_t *out_len;
  const int32_t *cap;          // [B] most tokens of each batch row
  const int32_t *origin_prev;  // [rows_prev] of step t-1 (unused at t == 0)
  int32_t *origin;             // [rows_prev] of step t
  int32_t *y;                  // [rows_prev] scratch: token of a previous dense row that goes on, else -1
  int32_t *tok_in;             // [rows_prev] input token of each dense row of step t
  int32_t *live;
  unsigned long long *progress;
  unsigned long long progress_tag;
  const _Float16 *E;
  const float *pe;
  float *z;
  int skip_embed;              // != 0: no embedding launch (the first projection of the step embeds tok_in itself)
};
hipError_t launch_eos_step_begin(const EosStepArgs &a, hipStream_t s);

// ---- attention ------------------------------------------------------------------------
// Encoder self-attention on a padded batch.  qkv [B*S, 3d] (q already scaled | k | v), len [B];
// ctx [B*S, d].  f32: qkv is fp32 (split-precision MFMA inside) and ctx is written as a head/tail
// pair of fp16 planes (tail ctx_lo_offset elements after the head); else both are fp16.  Keys >=
// len get weight exactly 0; query rows >= len get 0.  rk: optional relative keys [2*clip+1, dh].
hipError_t launch_enc_attention(const void *qkv, bool f32, const int32_t *len, void *ctx, long ctx_lo_offset, int B,
                                int S, int d, int heads, const float *rk, int clip, hipStream_t s);
// The register-resident form with the scaled query and the key as plain fp16 (qk [B*S, 2d]: q | k) and the value as
// fp32 (v [B*S, d]); sentences of at most 128 tokens, no relative keys (enc_attention_qk16_supported).  Scores then
// take one MFMA per product instead of three; probabilities, values and the context keep head + tail.
bool enc_attention_qk16_supported(int S, int d, int heads, const float *rk);
hipError_t launch_enc_attention_qk16(const _Float16 *qk, const float *v, const int32_t *len, void *ctx, long ctx_lo_offset,
                                     int B, int S, int d, int heads, hipStream_t s);

// Single-query attention against a cache, one query per (row, head).
//   q [rows, d] fp32 (scaled); ctx [rows, d] fp32.
//   cache row r: kv + r*row_stride elements, position j at + j*2d: k[d] then v[d].
//   n_keys: fixed count (self-attention: t+1) when len == nullptr, else len[r] (cross).
//   kv_f32 selects fp32 or fp16 cache elements.
//   rk (self only): relative keys; the query sits at position qpos, key j at position j.
//   ctx_lo_offset != 0: ctx is written as a head/tail pair of fp16 planes instead (head at ctx, tail that many
//   elements later).
//   origin (optional): query row r uses cache row (and len entry) origin[r]; origin[r] < 0 gives a zero context.
//   kv_new (optional, fp32 caches with a fixed key count only): [rows, 2d], the key and value of position
//   n_keys-1 of every query row; they are used from there and stored into the cache by this kernel.
hipError_t launch_attn_decode(const float *q, const void *kv, bool kv_f32, long row_stride, const int32_t *len,
                              int n_keys, int rows, int d, int heads, const float *rk, int clip, int qpos,
                              float *ctx, hipStream_t s, long ctx_lo_offset = 0, const int32_t *origin = nullptr,
                              const float *kv_new = nullptr);

// ---- single-query attention against 16-bit integer caches (nt_attn16.hip): one head, d = 256 / 512, no relative keys
bool attn_i16_supported(int d, int heads, int clip);
// Cache row c, position p: key codes at kv + ((c * row_positions + p) * 2) * d, value codes d elements later; their
// scales at sc[(c * row_positions + p) * 2] and [... + 1] (value = code * scale).
struct AttnI16Args {
  const float *q;        // [rows, d] fp32, already scaled
  short *kv;
  float *sc;
  long row_positions;    // positions a cache row holds (self: steps of the decode, cross: padded source length)
  const int32_t *len;    // cross-attention: keys of each cache row; nullptr for self-attention
  int n_keys;            // self-attention: t + 1; the last key/value pair is kv_new's, appended to the cache by the kernel
  int rows, d;
  int shape_rows;        // row count that selects the kernel form (0: rows).  The forms differ in the last bit, so a
                         // caller whose row count depends on timing passes one that does not
  const float *kv_new;   // self-attention: [rows, 2 d] fp32 (key | value of this step); nullptr for cross-attention
  const int32_t *origin; // optional: query row r uses cache row origin[r] (< 0: zero context)
  float *ctx;            // [rows, d] fp32, or (ctx_lo_offset != 0) head/tail fp16 planes
  long ctx_lo_offset;
};
hipError_t launch_attn_decode_i16(const AttnI16Args &a, hipStream_t s);
// x [M][2 d] fp32 (key | value of M positions) -> codes [M][2][d] and scales [M][2]
hipError_t launch_quantize_kv_i16(const float *x, long M, int d, short *cache, float *sc, hipStream_t s);

// max dynamic LDS the encoder attention needs for (S, dh); used to validate shapes at load.
size_t enc_attention_lds_bytes(int S, int dh, bool f32);

}  // namespace nt
