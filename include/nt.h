/*
 * libnt - batched inference of the lightweight student Transformer on one AMD MI355X.
 *
 * C ABI.  The boundary is cut at token ids: sentences in, translations out, a whole input
 * set translated as fast as possible (paper, abstract and Sec. 3.3 "Parallel Execution";
 * tokenisation and BPE are outside).  Every step of the path runs in hand-written gfx950
 * kernels; the library uses HIP only and never falls back to the CPU.
 *
 * Conventions
 *   - every function returns NT_OK (0) or a negative nt_status; nothing throws, aborts or
 *     prints.  nt_last_error() gives a thread-local message for the last failure.
 *   - "d_" arguments are device pointers, "h_" arguments are host pointers.  The caller owns
 *     every buffer it passes.  The library owns the weights, the activation arena and the
 *     key/value caches; it allocates only inside nt_load_weights and frees only in nt_free.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  nt_encode
 *     and nt_decode_greedy only enqueue work; nt_decode_greedy_eos enqueues a few steps ahead
 *     of the device and returns when the device is that close to the end; the two
 *     nt_translate_batch calls synchronise before they return host results.
 *   - one nt_model must not be used from two threads at once; nt_plan_batches is pure.
 *   - ids: 0 = PAD, 1 = BOS, 2 = EOS, 3 = UNK by convention; the library uses bos_id and
 *     pad_id of the configuration and the eos_id argument of the EOS-terminated calls.  The
 *     decoder may emit any id in [0, vocab).
 */
#ifndef NT_H
#define NT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  NT_OK = 0,
  NT_EINVAL = -1, /* null pointer, bad struct size, bad argument                         */
  NT_ESHAPE = -2, /* configuration or batch shape the kernels do not support             */
  NT_EBLOB = -3,  /* weight blob size does not match the configuration                   */
  NT_ENOMEM = -4, /* device or host allocation failed / batch does not fit the arena     */
  NT_EHIP = -5,   /* a HIP call or kernel launch failed                                  */
  NT_ERANGE = -6, /* token id outside [0,vocab), length outside [0,max_len], bad offsets */
  NT_ESTATE = -7  /* call order: decode without a preceding encode of the same batch     */
} nt_status;

typedef struct nt_model nt_model; /* opaque */

/*
 * Model and arena description.  Architecture fields follow the paper's student family
 * (Sec. 2.2 "Fast Student Models", Table 2) and the vanilla / teacher shapes it is compared
 * with (Sec. 2.1, Table 1, Table 3):
 *   n_enc, n_dec   encoder / decoder layers (student: 6 / 1)
 *   d_model        model width; must be a multiple of 64 and at most 1024
 *   n_heads        attention heads in every attention (student: 1); head width
 *                  d_model / n_heads must be 64, 128, 256 or 512
 *   d_ffn          FFN width in every layer, 0 = the FFN sub-layers are removed (student);
 *                  a multiple of 64 otherwise
 *   dec_n_heads, dec_d_ffn
 *                  the decoder's own shape where it differs from the encoder's (Table 2 and
 *                  Sec. 5: the submitted students put a base encoder, 8 heads and FFN 2,048, in
 *                  front of a one-head decoder layer whose FFN is 512 wide or absent).
 *                  dec_n_heads 0 = n_heads; dec_d_ffn 0 = d_ffn, -1 = no decoder FFN, otherwise
 *                  the width (a multiple of 64).  n_heads and d_ffn then describe the encoder.
 *   vocab          shared source/target vocabulary
 *   max_len        longest source sentence and longest target prefix (positions), <= 512
 *   rpr_clip       clipping distance of the relative position keys in self-attention
 *                  (Sec. 2.1: 8 for the teachers), 0 = none
 *   tie_output     1: the output projection is the embedding matrix (Sec. 2.3); 0: the blob
 *                  holds a separate W_out
 *   ln_eps         LayerNorm epsilon (pre-LN blocks, biased variance)
 *   ln_l1          1: every layer normalisation is the L1-norm variant the paper's GPU systems use
 *                  (Sec. 3.1 "FP16 Inference"): y = g (x - mean) / (sqrt(pi/2) mean|x - mean| + ln_eps) + b,
 *                  the mean absolute deviation scaled so that it equals the standard deviation for
 *                  normal activations; 0: the vanilla form
 *   q8_output      1: the output layer is an 8-bit matrix multiplication (Sec. 3.2 "8-bit Matrix
 *                  Multiplication with Packing", the paper's CPU optimisation, here on the int8 matrix
 *                  cores).  Every vocabulary entry's d weights are quantised at load time with their own
 *                  scale 14 sd / 255 and zero point (Eq. 3, 4) and packed in matrix-core order; every
 *                  decoder state is quantised per row with scale (max - min) / 255 and its zero point
 *                  (Eq. 5, 6; per row, not per matrix, so that a sentence never depends on its batch
 *                  mates).  Zero points are integers inside the 8-bit range; Eq. 4 and 6 are read as
 *                  127 - (mean + 7 sd) / scale and 255 - max / scale.  The logit is
 *                  a_scale * (b_scale[v] * float(I)) with I = sum_k (u_k - a_zero)(q_vk - zero_v) exact.
 *                  Needs d_model 256 or 512.  0: fp16 matrix cores with ~22-bit activations.
 *   max_batch_tokens, max_batch_rows
 *                  largest padded batch (rows x longest row) and most rows per batch the
 *                  arena must hold; the peak footprint is fixed at load time, in the spirit
 *                  of the paper's memory optimisation (Sec. 3.3).  max_batch_rows = 0 means
 *                  max_batch_tokens rows.
 */
typedef struct {
  uint32_t struct_size; /* sizeof(nt_config), checked */
  int32_t n_enc, n_dec, d_model, n_heads, d_ffn, vocab, max_len;
  int32_t rpr_clip, tie_output, bos_id, pad_id;
  float ln_eps;
  int32_t max_batch_rows;
  int64_t max_batch_tokens;
  int32_t pipeline_lanes; /* batches kept in flight by nt_translate_batch, each with its own arena and
                             internal stream; 0 = default (4, one per hardware queue), 1 = no overlap */
  int32_t dec_n_heads, dec_d_ffn;
  int32_t ln_l1;
  int32_t q8_output;
} nt_config;

/* Number of fp16 elements the weight blob of this configuration must hold (0 if invalid). */
int64_t nt_param_count(const nt_config *cfg);

/*
 * Number of greedy steps run for a source of `len` tokens: ceil(1.2 * len) + 2, evaluated
 * in integers (the benchmark's fixed-length decoding rule; EOS is an ordinary token).
 */
int32_t nt_n_steps(int32_t len);

/*
 * Load a model.  h_blob_fp16: host pointer to the flat little-endian fp16 blob, tensors in
 * the documented order, every matrix as W[in][out].  The matrices are copied to the device
 * and re-laid-out once into the K-contiguous form the MFMA kernels read (the paper hoists
 * its transposes to the start of decoding, Sec. 3.3 "Graph Optimization"); the sinusoid
 * table is built; the arena and caches are allocated.  Synchronises hip_stream.
 * Errors: NT_EINVAL, NT_ESHAPE, NT_EBLOB (blob_bytes != 2 * nt_param_count), NT_ENOMEM, NT_EHIP.
 */
int nt_load_weights(const nt_config *cfg, const void *h_blob_fp16, size_t blob_bytes, void *hip_stream,
                    nt_model **out);

void nt_free(nt_model *m);

/*
 * Encoder over one padded batch (Sec. 2.2; Sec. 3.1 "FP16 Inference").
 *   d_src [B, S] int32 row-major, row b holds d_len[b] ids then padding (any value);
 *   d_len [B] int32, each in [1, S].
 * Leaves, inside the model: the encoder output and the cross-attention keys/values of every
 * decoder layer.  Pad positions never influence real ones.  Ids outside [0,vocab) and
 * lengths outside [1,S] cannot be rejected without reading device memory: they are clamped
 * in the kernels (id -> pad_id, len -> [1,S]) and a sticky device flag is raised that
 * nt_check_device_flags reports.
 * Errors: NT_EINVAL, NT_ESHAPE (S > max_len), NT_ENOMEM (B*S or B beyond the arena), NT_EHIP.
 */
int nt_encode(nt_model *m, const int32_t *d_src, const int32_t *d_len, int32_t B, int32_t S, void *hip_stream);

/*
 * Greedy decoding of the batch left by the last nt_encode (Sec. 3.3 "Greedy Search"; the
 * output layer's log-softmax is dropped, Sec. 3.3 "Graph Optimization").  Runs exactly
 * n_steps incremental steps from BOS with key/value caches; the next token of a row is the
 * arg-max of its logits, lowest id on ties; it stays on the device and feeds the next step.
 *   d_out [B, n_steps] int32, device.  Row b, step t.
 *   h_row_steps: optional host array [B], non-increasing, each in [0, n_steps]: row b is only
 *   advanced for its first h_row_steps[b] steps (rows sorted by length finish in order, so
 *   the active rows are always a prefix); entries of d_out beyond that are set to pad_id.
 *   NULL = every row runs n_steps steps.  A row's arithmetic never reads another row.  The number of
 *   active rows does select between kernel forms whose fp32 summation order differs (how many waves
 *   share a row's keys in the attention kernels; for model widths other than 256 / 512 a
 *   one-round-trip projection kernel below 128 rows), so the same sentence decoded in batches of very
 *   different size can differ in the last bit of a logit, and therefore in a token where two logits
 *   tie to within that bit; the EOS-terminated call below fixes the choice by the caps alone.
 * Errors: NT_EINVAL, NT_ESTATE (B differs from the encoded batch), NT_ERANGE (n_steps >
 * max_len, h_row_steps not non-increasing), NT_ENOMEM (B * n_steps beyond the self cache), NT_EHIP.
 */
int nt_decode_greedy(nt_model *m, int32_t B, int32_t n_steps, const int32_t *h_row_steps, int32_t *d_out,
                     void *hip_stream);

/*
 * The 8-bit output layer alone (models loaded with q8_output = 1), for checking it against its
 * definition on given inputs: d_h [R, d_model] fp32 rows (used as they are: no LayerNorm) are
 * quantised per row and multiplied with the packed 8-bit output matrix.
 *   d_argmax [R] int32 (optional): arg-max over the vocabulary of b_scale[v] * float(I), lowest id on
 *   ties, from the fused kernel that greedy decoding uses;
 *   d_logits [R, vocab] fp32 (optional): a_scale * (b_scale[v] * float(I)).
 * R must not exceed max_batch_rows.  Errors: NT_ESTATE if the model has no 8-bit output layer.
 */
int nt_debug_q8_output_layer(nt_model *m, const float *d_h, int32_t R, int32_t *d_argmax, float *d_logits,
                             void *hip_stream);

/*
 * nt_debug_q8_output_layer for callers that cannot allocate device memory or let a library do so (code under
 * HIP graph capture, tight serving loops, harnesses that forbid it): same arguments and results, but
 * the layer's scratch (activation codes, per-row constants, arg-max partial keys) is a fixed array inside
 * the library's code object, NT_STATIC_MAX_ROWS rows of at most 512 columns (0.8 MiB per GPU, held until
 * the process ends), instead of the model's arena.  The call uses no memory of the model's arena besides
 * the weights, allocates nothing and only enqueues kernels on hip_stream.  Every call on a GPU shares
 * that GPU's array: calls that overlap on one GPU (two streams, two threads, two models) race; calls in
 * stream order do not.  Errors: NT_ERANGE if R is outside [1, NT_STATIC_MAX_ROWS]; otherwise as
 * nt_debug_q8_output_layer.
 */
#define NT_STATIC_MAX_ROWS 1024
int nt_q8_output_layer_static(nt_model *m, const float *d_h, int32_t R, int32_t *d_argmax, float *d_logits,
                              void *hip_stream);

/*
 * The weight side of the 8-bit output layer for one vocabulary entry, as nt_load_weights applies it to every row
 * of the output matrix (Eq. 3, 4): h_w_fp16 [K] fp16 host -> h_codes [K] signed 8-bit, *h_scale, *h_zero.  Runs on
 * the host; needs no model and no GPU.
 */
int nt_debug_q8_quantize_row(const void *h_w_fp16, int32_t K, int8_t *h_codes, float *h_scale, int32_t *h_zero);

/*
 * Greedy decoding that ends a sentence at its end symbol (Sec. 3.3 "Greedy Search": the paper's
 * systems decode with beam size 1 until EOS, where the benchmark's rule above runs a fixed number
 * of steps).  Row b ends with the first eos_id it emits, which is stored, or after
 * h_row_steps[b] tokens (n_steps if h_row_steps is NULL), whichever comes first.
 *   d_out [B, n_steps] int32, device: the tokens of row b, then pad_id.
 *   d_out_len [B] int32, device: number of tokens of row b (EOS included).
 * Rows that have ended leave the computation: the rows still decoding are kept as a dense prefix
 * on the device (their caches stay where they are and are reached through a row map), and the
 * device publishes their count after every step in pinned host memory.  The count only falls, so
 * whatever the host last read is a valid upper bound: it sizes every later launch with it and
 * stops launching once it reads zero.  The host never waits for the stream to drain, but it
 * enqueues at most a few steps ahead of the device, so the call returns when the device is
 * within those few steps of the end; the outputs are complete once hip_stream has been
 * synchronised.  Tokens are those nt_decode_greedy produces, cut after the first EOS.
 * Errors: as nt_decode_greedy; NT_ERANGE for eos_id outside the vocabulary; NT_EHIP if the device
 * publishes no progress for 30 seconds.
 */
int nt_decode_greedy_eos(nt_model *m, int32_t B, int32_t n_steps, const int32_t *h_row_steps, int32_t eos_id,
                         int32_t *d_out, int32_t *d_out_len, void *hip_stream);

/*
 * Translate N sentences end to end (dynamic batching: Sec. 3.1 "Dynamic Batching"; sorting by
 * descending length and sbatch/wbatch caps: Sec. 3.3 "Graph Optimization", "Better Decoding
 * Configurations").
 *   h_tokens: all source ids concatenated; h_offsets [N+1]: sentence i is
 *   h_tokens[h_offsets[i] .. h_offsets[i+1]).
 *   token_budget: cap on rows x longest-row per batch (wbatch); max_rows: cap on rows per
 *   batch (sbatch), 0 = none.  Both are also limited by the arena given at load time.
 *   h_out: output ids, sentence i at h_out[h_out_offsets[i] .. h_out_offsets[i+1]) with
 *   nt_n_steps(len_i) ids (0 for an empty sentence); h_out_offsets [N+1] is written by the
 *   call; h_out must hold sum_i nt_n_steps(len_i) ids.
 * N = 0 succeeds and writes only h_out_offsets[0] = 0.  The input is validated on the host
 * before anything is launched: an id outside [0,vocab), a sentence longer than max_len or
 * non-monotone offsets give NT_ERANGE and no output.
 */
int nt_translate_batch(nt_model *m, const int32_t *h_tokens, const int64_t *h_offsets, int64_t N,
                       int64_t token_budget, int32_t max_rows, int32_t *h_out, int64_t *h_out_offsets,
                       void *hip_stream);

/*
 * The same with EOS-terminated greedy decoding (nt_decode_greedy_eos; cap nt_n_steps(len_i) per
 * sentence).  Sentence i keeps its nt_n_steps(len_i) slots in h_out: h_out_len[i] tokens, the last
 * one eos_id unless the cap cut the sentence, then pad_id.  h_out_len [N] is written by the call
 * (0 for an empty sentence).  The pipeline lanes advance their batches step by step in turn, each
 * sized by the latest count of rows still decoding that its device side has published.
 */
int nt_translate_batch_eos(nt_model *m, const int32_t *h_tokens, const int64_t *h_offsets, int64_t N,
                           int64_t token_budget, int32_t max_rows, int32_t eos_id, int32_t *h_out,
                           int64_t *h_out_offsets, int32_t *h_out_len, void *hip_stream);

/*
 * Number of output ids the two nt_translate_batch calls write for these sentences: the sum of
 * nt_n_steps(len_i) over the non-empty sentences (the size h_out must have).  Host only.
 * Errors: NT_EINVAL (null argument, negative N), NT_ERANGE (offsets decrease).
 */
int nt_output_slots(const int64_t *h_offsets, int64_t N, int64_t *total);

/*
 * Host-only batch planner used by nt_translate_batch: the paper's dynamic batching (Sec. 3.1
 * "Dynamic Batching": as many sentences per batch as a cap on its tokens allows), over sentences
 * sorted by descending length (Sec. 3.3 "Graph Optimization", memory optimisation) under the two
 * caps of Sec. 3.3 "Better Decoding Configurations" (sbatch = max_rows sentences, wbatch = budget
 * tokens, counted padded).  Stable sort by
 * descending length (ties by index); batches are maximal prefixes of the sorted list with
 * rows * longest <= budget and rows <= max_rows (0 = no cap); a sentence longer than the
 * budget forms a batch of its own; empty sentences are placed last and belong to no batch.
 *   order [N]: sentence indices in sorted order; batch_starts [N+1 entries available]:
 *   batch k is order[batch_starts[k] .. batch_starts[k+1]); *n_batches is written.
 * Errors: NT_EINVAL (null, budget < 1, negative length).
 */
int nt_plan_batches(const int32_t *h_lengths, int64_t N, int64_t budget, int32_t max_rows, int64_t *order,
                    int64_t *batch_starts, int64_t *n_batches);

/* ---- not on the hot path: needed to check parity -------------------------------------- */

/*
 * Copy the encoder output of the last nt_encode - the final LayerNorm of the encoder stack (Sec. 2.2
 * "Fast Student Models": the deep encoder whose output every decoder step attends to) - as fp32
 * [B, S, d_model] (pad rows included).
 */
int nt_debug_encoder_out(nt_model *m, float *d_out, void *hip_stream);

/*
 * Teacher-forced decoder logits for the batch left by the last nt_encode (the decoder layer of
 * Sec. 2.2 and the output layer without its log-softmax, Sec. 3.3 "Graph Optimization", evaluated
 * on given target prefixes instead of the greedy search of Sec. 3.3 "Greedy Search"): the decoder is fed
 * d_tgt_in [B, T] (column 0 is normally BOS) instead of its own arg-max and the fp32 logits of
 * every step are written to d_logits [B, T, vocab].  Same kernels as nt_decode_greedy except
 * that the output projection stores its tile instead of reducing it.
 */
int nt_debug_teacher_forced_logits(nt_model *m, const int32_t *d_tgt_in, int32_t B, int32_t T, float *d_logits,
                                   void *hip_stream);

/*
 * Testing aids that select numerical paths of the output projection (both default to 0; they act on
 * every pipeline lane of the model and on the calls that follow):
 *   nt_debug_set_vocab_tiled(m, 1)    take the LDS-tiled arg-max kernels that other model widths use,
 *                                     instead of the streaming kernels;
 *   nt_debug_set_cert_distrust(m, 1)  certify no row in the single-pass arg-max, so that every row
 *                                     takes the head+tail recompute pass.
 *   nt_debug_set_encoder_tails(m, mask)  which encoder projections multiply the tail plane of their activations
 *                                     (about 22 significant bits) and which the head plane only (fp16, half the
 *                                     matrix-core work): bit 0 LayerNorm -> Q|K|V, bit 1 attention context -> output
 *                                     projection, bit 2 final LayerNorm -> cross-attention K|V, bit 3 first FFN
 *                                     matrix; with bit 0 clear, bits 4 / 5 / 6 select the q / k / v columns of
 *                                     Q|K|V alone (a contiguous group); bit 7: the scaled query and the key are
 *                                     stored as plain fp16 (sentences of at most 128 tokens, one head, width
 *                                     512).  The library's default is the plan its precision study adopted: the
 *                                     v columns, the output projection and bit 7 for the one-head student
 *                                     without FFN, every tail for other encoders.
 * Errors: NT_EINVAL (null model, value other than 0 / 1, mask beyond 8 bits).
 */
int nt_debug_set_vocab_tiled(nt_model *m, int on);
int nt_debug_set_cert_distrust(nt_model *m, int on);
int nt_debug_set_encoder_tails(nt_model *m, uint32_t mask);

/*
 * Read and clear the sticky device flags (synchronises the stream).  Returns NT_OK, or
 * NT_ERANGE if a kernel has clamped an out-of-range id or length since the last call.
 */
int nt_check_device_flags(nt_model *m, void *hip_stream);

/*
 * Per-launch kernel timing for measurement (off by default; it adds two event records per
 * timed launch).  kernel_mask has one bit per kernel family, ids 0 .. nt_debug_timing_count()-1,
 * names from nt_debug_timing_name().  Enabling (or re-enabling) clears what was recorded.
 * nt_debug_timing_read synchronises the stream and returns, for one family, the summed
 * event-to-event time of its launches, their number, and the summed algorithmic bytes and
 * flops of those launches (the minimum traffic / arithmetic the operation needs at its shape:
 * operands read once, results written once).  Cross-attention bytes are exact when the batch
 * came through nt_translate_batch (host lengths known) and use the padded length otherwise.
 */
int nt_debug_timing_enable(nt_model *m, uint64_t kernel_mask);
int nt_debug_timing_count(void);
const char *nt_debug_timing_name(int kernel);
int nt_debug_timing_read(nt_model *m, int kernel, double *total_ms, int64_t *launches, double *bytes, double *flops,
                         void *hip_stream);

/*
 * What this GPU reaches on plain probes, for rooflines against measured rather than datasheet peaks:
 *   mfma_tflops                     a loop of independent 32x32x16 fp16 MFMAs on every SIMD whose operands are random
 *                                   values that change from one instruction to the next, as a model's weights and
 *                                   activations do (TFLOP/s): what the power limit lets the matrix pipes sustain on
 *                                   real data;
 *   mfma_tflops_constant_operands   the same loop on two constant operands: little switching in the multipliers, the
 *                                   chip holds its clock, close to the datasheet figure;
 *   hbm_read_gbs                    a streaming read of up to 1 GiB of the model's arena (GB/s);
 *   hbm_copy_gbs                    the same bytes read and written back in place, bytes read + bytes written per
 *                                   second (GB/s): what kernels that write as much as they read can reach.
 * Best of three runs each; synchronises hip_stream; the arena keeps its contents (no other stream may use this
 * model meanwhile).  Measurement aid, a few tens of milliseconds.
 * Errors: NT_EINVAL (null argument), NT_EHIP.
 */
int nt_debug_probe_peaks(nt_model *m, double *mfma_tflops, double *mfma_tflops_constant_operands, double *hbm_read_gbs,
                         double *hbm_copy_gbs, void *hip_stream);

/*
 * Pipeline lanes.  A model holds pipeline_lanes lanes that share the weights; each lane has its own
 * arena, caches and state.  nt_pipeline_lane(m, i) returns lane i (lane 0 is m itself) as a model
 * handle that nt_encode / nt_decode_greedy / nt_debug_* accept, so that a caller who keeps its batches
 * on the device can run independent batches on different streams at the same time.  Lane handles are
 * owned by m: never pass them to nt_free.  nt_translate_batch uses all lanes by itself.
 * nt_lane_stream returns the HIP stream (hipStream_t) that the library created for a lane and that
 * nt_translate_batch launches the lane's work on; it is owned by the model.  A caller that drives the
 * lanes itself may launch on these streams: nt_load_weights has checked with a short probe kernel that
 * they run concurrently (streams that land on the same hardware queue do not overlap; there are four
 * queues per process unless the runtime is told otherwise).  Returns NULL for a null model.
 */
int nt_pipeline_lanes(const nt_model *m);
nt_model *nt_pipeline_lane(nt_model *m, int i);
void *nt_lane_stream(nt_model *m);

/* Bytes of device memory held by the model (weights, arena, caches). */
int64_t nt_device_bytes(const nt_model *m);

/* Message for the last error on this thread (valid until the next failing call). */
const char *nt_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* NT_H */
