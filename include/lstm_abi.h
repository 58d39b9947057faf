/*
 * C ABI of the MI355X (gfx950) masked LSTM / BLSTM layer library.
 *
 * The operation is the recurrent layer the paper names in Listing 1 ("class": "rec",
 * "unit": "nativelstm2", "direction": +1 / -1; two such layers on the same input, concatenated,
 * form one bidirectional layer) and the stepped decoder cell ("rnn_cell" / "LSTMBlock"), with
 * the input projection taken out of the recurrent loop (Sec. 3, Sec. 7).  The paper prints no
 * cell equations; the library implements the peephole-free LSTM
 *
 *     z = x_t W_x + h W_h + b          (4n columns, gate blocks i | f | g | o)
 *     i,f,o = sigmoid(z_i,z_f,z_o)     g = tanh(z_g)
 *     c' = f*c + i*g                   h' = o*tanh(c')
 *
 * over end-padded, variable-length batches.  Frame t of row b is valid iff t < seq_lens[b].
 * At a padded frame the state is carried unchanged, y is 0, the stored cell state is the carried
 * one, and the frame contributes no gradient; values stored in x / dy at padded frames never
 * reach a result.  direction -1 walks t = T-1 .. 0 over the same tensors.
 *
 * Beside the layer (lstm_query, lstm_fwd, lstm_bwd, blstm_fwd, blstm_bwd) the library holds what the paper's encoders
 * and decoder put around it, each documented at its declaration below: the hoisted product by itself (lstm_gemm),
 * max-pooling in time between encoder layers (lstm_time_pool_fwd / _bwd), one step of the attention decoder
 * (lstm_attention_step, lstm_readout), one step of batched beam search (lstm_beam_step, lstm_beam_gather, lstm_beam_gather_many, lstm_embed),
 * and diagnostics (lstm_sync_status, lstm_profile_*, lstm_strerror).
 *
 * Conventions common to every entry point
 *   - All data pointers are DEVICE pointers owned by the caller, 16-byte aligned (unless an entry
 *     point states a weaker requirement), row-major,
 *     time-major.  The library allocates and frees nothing; scratch comes from `workspace`,
 *     state saved for the backward pass goes to `reserve`; sizes come from lstm_query().
 *   - `stream` is a hipStream_t cast to void* (NULL = the default stream).  Calls only enqueue
 *     work; they never synchronise.  Buffers must stay alive until the stream has passed the call.
 *   - dtype LSTM_F32: every tensor is float.  dtype LSTM_BF16_F32STATE: x, W_x, W_h, y, dy, dx
 *     are bfloat16; b, c, h0, c0, hT, cT, dhT, dcT, dh0, dc0, dW_x, dW_h, db are float.  All
 *     accumulation, the cell state and the gate activations are float in both modes.
 *   - Optional pointers (may be NULL): b (zero bias), h0, c0 (zero state), seq_lens (all rows
 *     have length T), hT, cT, dhT, dcT (zero), dx, dh0, dc0 (not produced); c only with LSTM_FLAG_INFERENCE
 *     (the backward call reads it).
 *   - seq_lens is int32[B] in device memory, any order; values are clamped to [0, T] in the kernels.
 *   - Return value: 0 on success, a negative lstm_status otherwise.  Arguments are validated on
 *     the host before the first HIP call, so every argument error is reported without a GPU.
 *     Nothing throws or aborts across this boundary.  LSTM_OK says that the work was enqueued; it does not cover
 *     a bounded wait inside a single-launch recurrent kernel that expires later on the device (see lstm_sync_status).
 */
#ifndef MI355X_LSTM_ABI_H
#define MI355X_LSTM_ABI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { LSTM_F32 = 0, LSTM_BF16_F32STATE = 1 } lstm_dtype;

typedef enum {
  LSTM_OK = 0,
  LSTM_ERR_NULL = -1,       /* required pointer (or the descriptor) is NULL                     */
  LSTM_ERR_DIM = -2,        /* negative T or B, or n / n_in < 1, or a size that overflows int32  */
  LSTM_ERR_DIRECTION = -3,  /* direction is neither +1 nor -1 (lstm_* only)                      */
  LSTM_ERR_UNSUPPORTED = -4,/* unknown dtype or flag bit                                         */
  LSTM_ERR_ALIGN = -5,      /* a pointer is not 16-byte aligned                                  */
  LSTM_ERR_SIZE = -6,       /* reserve_bytes / workspace_bytes smaller than lstm_query() demands */
  LSTM_ERR_HIP = -7         /* HIP runtime error while enqueueing, or the device is not gfx950   */
} lstm_status;

enum {
  LSTM_FLAG_ACCUMULATE = 1, /* *_bwd: add into dW_x, dW_h, db instead of overwriting them        */
  LSTM_FLAG_PER_STEP = 2,   /* force one kernel launch per time step (no single-launch loop; the default is
                              * one launch for the whole time loop where a kernel for it exists: bfloat16
                              * storage with n <= 1024; float storage with n a multiple of 8 and
                              * n <= 1024, backward with B <= 256) */
  LSTM_FLAG_INFERENCE = 4,  /* *_fwd: nothing is saved for backward; reserve may be NULL         */
  LSTM_FLAG_WEIGHTS_PACKED = 8,/* *_fwd with T == 1 and LSTM_FLAG_INFERENCE: the caller states that the
                              * previous *_fwd call on this workspace had the same T, B, n_in, n, dtype,
                              * bidirectionality and the same W_x, W_h contents, so the packed copy of the
                              * weights that the workspace still holds is used again instead of being
                              * rebuilt (a false statement gives wrong results, not an error).  Ignored
                              * by every other call. */
  LSTM_FLAG_PLAIN_LAUNCH = 16 /* the single-launch recurrent kernels, whose work-groups wait for each other
                              * and therefore must all be resident at once, are started with an ordinary
                              * launch instead of a cooperative one (which costs tens of microseconds of
                              * idle device per launch).  The caller states that nothing else occupies the
                              * device while the call's work runs (no other stream, no other process).
                              * If that is false the work-groups' bounded waits expire: the call's outputs
                              * are invalid and lstm_sync_status() says so; nothing hangs. */
};

typedef struct {
  int32_t T, B, n_in, n;    /* padded length, batch rows, input width, units per direction       */
  int32_t direction;        /* +1 or -1; read by lstm_fwd / lstm_bwd only                        */
  int32_t dtype;            /* lstm_dtype                                                        */
  int32_t flags;            /* LSTM_FLAG_* bits                                                  */
  int32_t reserved;         /* must be 0                                                         */
  uint64_t reserve_bytes;   /* bytes the caller allocated behind `reserve`                       */
  uint64_t workspace_bytes; /* bytes the caller allocated behind `workspace`                     */
} lstm_desc;

/* Sizes of `reserve` and `workspace` for this problem (bidirectional != 0 for blstm_*).
 * The workspace size covers both the forward and the backward call.  T == 0 or B == 0 is legal
 * (the calls are then no-ops) and yields small non-zero sizes.  Only T, B, n_in, n, dtype and
 * flags of the descriptor are read. */
int lstm_query(const lstm_desc* desc, int bidirectional, size_t* reserve_bytes, size_t* workspace_bytes);

/* Forward pass of one direction (Listing 1, "rec"/"nativelstm2" with "direction").
 *   x[T,B,n_in]  W_x[n_in,4n]  W_h[n,4n]  b[4n]  h0,c0[B,n]  seq_lens[B]
 *   -> y[T,B,n] (0 at padded frames), c[T,B,n] (cell state after each frame, carried at padded
 *      frames; may be NULL with LSTM_FLAG_INFERENCE only), hT,cT[B,n] (state after each row's last processed valid frame),
 *      reserve (opaque: gate activations and the hidden state entering each frame).
 * With T == 1 and LSTM_FLAG_INFERENCE this is the stepped decoder cell (Sec. 7, Listing 1: the decoder's
 * recurrent unit, stepped once per output word for all beam entries): feed hT,cT back as h0,c0.  For
 * bfloat16 storage that step runs as one product [x_t | h] [W_x ; W_h] + b over all rows followed by the
 * cell update; pass LSTM_FLAG_WEIGHTS_PACKED from the second step on to keep the packed weights. */
int lstm_fwd(const lstm_desc* desc, const void* x, const void* W_x, const void* W_h, const void* b,
             const void* h0, const void* c0, const int32_t* seq_lens,
             void* y, void* c, void* hT, void* cT, void* reserve, void* workspace, void* stream);

/* Backward pass (back-propagation through time) of one direction: the exact gradient of
 * sum(dy*y) + sum(dhT*hT) + sum(dcT*cT).  y, c and reserve must be the forward call's, untouched.
 *   dy[T,B,n]  dhT,dcT[B,n]
 *   -> dx[T,B,n_in] (0 at padded frames), dW_x[n_in,4n], dW_h[n,4n], db[4n], dh0,dc0[B,n]. */
int lstm_bwd(const lstm_desc* desc, const void* x, const void* W_x, const void* W_h,
             const void* h0, const void* c0, const int32_t* seq_lens,
             const void* y, const void* c, const void* reserve,
             const void* dy, const void* dhT, const void* dcT,
             void* dx, void* dW_x, void* dW_h, void* db, void* dh0, void* dc0,
             void* workspace, void* stream);

/* Bidirectional layer (Listing 1: enc*_fw + enc*_bw + "copy"): both directions run concurrently.
 * W_x[2,n_in,4n], W_h[2,n,4n], b[2,4n], h0,c0,hT,cT[2,B,n], c[2,T,B,n]; index 0 = direction +1,
 * 1 = direction -1.  y[T,B,2n]: direction +1 in columns 0..n-1, direction -1 in n..2n-1. */
int blstm_fwd(const lstm_desc* desc, const void* x, const void* W_x, const void* W_h, const void* b,
              const void* h0, const void* c0, const int32_t* seq_lens,
              void* y, void* c, void* hT, void* cT, void* reserve, void* workspace, void* stream);

/* Backward of the bidirectional layer.  dy[T,B,2n]; dx[T,B,n_in] is the SUM of both directions;
 * dW_x[2,n_in,4n], dW_h[2,n,4n], db[2,4n], dhT,dcT,dh0,dc0[2,B,n]. */
int blstm_bwd(const lstm_desc* desc, const void* x, const void* W_x, const void* W_h,
              const void* h0, const void* c0, const int32_t* seq_lens,
              const void* y, const void* c, const void* reserve,
              const void* dy, const void* dhT, const void* dcT,
              void* dx, void* dW_x, void* dW_h, void* db, void* dh0, void* dc0,
              void* workspace, void* stream);

/* The hoisted matrix product the layer uses for Zx = X W_x + b, dX = DZ W_x^T, dW_x = X^T DZ and
 * dW_h = Hprev^T DZ (Sec. 3: work moved out of the recurrent loop), exposed so that each shape can be
 * tested and timed by itself.  C[M,N] (+)= A B + bias, float accumulation.
 *   in_bf16 / out_bf16: operand and result storage (bfloat16 or float; out_bf16 requires in_bf16).
 *   a_kcontig != 0: A is [M][lda] (k contiguous), else [K][lda] (m contiguous);
 *   b_kcontig != 0: B is [N][ldb] (k contiguous), else [K][ldb] (n contiguous).
 *   Supported pairs: (1,0), (1,1), (0,0).  bias[N] may be NULL.  accumulate != 0 adds into a float C.
 *   lens != NULL (only with a_kcontig == 0): row k of the K axis is frame (t = k / Bt, b = k % Bt) of a
 *   batch of Bt rows and T frames and is read as zero unless t < lens[b].
 * Leading dimensions are in elements; rows must be aligned to the element size only. */
int lstm_gemm(int in_bf16, int out_bf16, int a_kcontig, int b_kcontig, int M, int N, int K,
              const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, const float* bias,
              int accumulate, const int32_t* lens, int Bt, int T, void* stream);

/* Max-pooling in time between encoder layers.  The paper's attention-based speech encoder (Sec. 4, the
 * attention model on Switchboard: six bidirectional layers, a maximum taken over time between them, the
 * input shortened by a factor of 8 in total) pools the layer outputs over time; window, stride and padding
 * are not given.  This library's reading: non-overlapping windows of
 * `pool` frames (stride = window; pool = 2 after each of three layers gives the factor 8), taken inside every
 * sequence separately:
 *     T' = ceil(T / pool),  lens_out[b] = ceil(seq_lens[b] / pool),
 *     out[t', b, :] = max over the valid frames t in [pool t', pool t' + pool), t < seq_lens[b], of y[t, b, :]
 * for t' < lens_out[b], and 0 at padded output frames (the last window of a sequence may be short; values stored
 * at padded input frames are never read).  The backward call sends the gradient of an output element to the
 * frame that supplied the maximum - the earliest one if several are equal - and writes 0 everywhere else,
 * padded frames included: dy is written completely and need not be cleared.
 *   dtype: LSTM_F32 (float tensors) or LSTM_BF16_F32STATE (bfloat16 tensors); the maximum is exact in both.
 *   y [T][B][ldy >= F], out [T'][B][ldo >= F], dout like out, dy like y: device pointers, element-aligned
 *   (16-byte aligned rows are faster); leading dimensions in elements.  1 <= pool <= 255.
 *   arg: device, T' * B * F bytes, written by the forward call at valid output frames (offset of the chosen frame inside its window)
 *   and read by the backward call; may be NULL in the forward call if no backward call follows.
 *   seq_lens: device int32[B] or NULL (all rows have length T); lens_out: device int32[B] or NULL.
 * Errors: LSTM_ERR_NULL, LSTM_ERR_DIM (negative sizes, F < 1, pool out of range, ld < F), LSTM_ERR_UNSUPPORTED
 * (dtype), LSTM_ERR_ALIGN, LSTM_ERR_HIP.  The calls only enqueue work on `stream`. */
int lstm_time_pool_fwd(int dtype, int T, int B, int F, int pool, const void* y, int64_t ldy, const int32_t* seq_lens,
                       void* out, int64_t ldo, uint8_t* arg, int32_t* lens_out, void* stream);
int lstm_time_pool_bwd(int dtype, int T, int B, int F, int pool, const void* dout, int64_t ldo, const uint8_t* arg,
                       const int32_t* seq_lens, void* dy, int64_t ldy, void* stream);

/* One step of the attention decoder, from the cell output s to the attention context (Listing 1, sub-network of
 * layer "output": "s_tr", "weight_feedback", "e_in", "e_tanh", "e", "a", "accum_a", "att"; "enc_ctx" is the
 * loop-invariant projection of the encoder states and is computed by the caller once per sentence, e.g. with
 * lstm_gemm, as Sec. 7 describes for work that does not depend on the loop).  With j a source position, r a row
 * of the decoder batch and q(r) = r / beam its sentence (the `beam` hypotheses of a sentence are neighbours):
 *     s_tr[r]   = s[r] W_s + b_s
 *     e[r, j]   = v . tanh(enc_ctx[j, q(r)] + accum_in[r, j] * w_fb + b_fb + s_tr[r]) + b_e
 *     a[r, :]   = softmax of e[r, :] over j < src_lens[q(r)];  a[r, j] = 0 for the other j
 *     accum_out = accum_in + a   (0 at j >= src_lens[q(r)])
 *     att[r]    = sum_j a[r, j] enc[j, q(r)]
 * Values stored at positions j >= src_lens[q] in enc, enc_ctx or accum_in are never read; a sentence of length 0
 * gives a = 0, att = 0.  The cell that produces s is lstm_fwd with T = 1 and LSTM_FLAG_INFERENCE.
 *   desc: S source positions (1..1024), Q sentences, beam hypotheses per sentence (1..16), A attention width,
 *         E encoder state width (even), n cell width, workspace_bytes as lstm_attention_query() returns.
 *   enc      bfloat16 [S][Q][E]      enc_ctx  bfloat16 [S][Q][A]      src_lens int32 [Q] or NULL (all S)
 *   s        bfloat16 [Q*beam][ld_s >= n]                W_s bfloat16 [A][n] (a row per output feature)
 *   b_s, w_fb, b_fb, v   float [A]   b_e float (passed by value)
 *   accum_in, accum_out, a   float [Q*beam][S] (a may be NULL; accum_out must not overlap accum_in)
 *   att      bfloat16 [Q*beam][ld_att >= E], ld_att even, 4-byte aligned: may point into a wider row, e.g. the
 *            concatenated input of lstm_readout or of the next step's cell.
 * All pointers are device pointers owned by the caller; arithmetic is float.  The call only enqueues work.
 * Errors: LSTM_ERR_NULL, LSTM_ERR_DIM, LSTM_ERR_UNSUPPORTED (beam > 16, S > 1024, odd E), LSTM_ERR_ALIGN,
 * LSTM_ERR_SIZE (workspace), LSTM_ERR_HIP. */
typedef struct lstm_att_desc {
  int32_t S, Q, beam, A, E, n;
  uint64_t workspace_bytes;
} lstm_att_desc;
int lstm_attention_query(const lstm_att_desc* desc, uint64_t* workspace_bytes);
int lstm_attention_step(const lstm_att_desc* desc, const void* enc, const void* enc_ctx, const int32_t* src_lens,
                        const void* s, int64_t ld_s, const void* W_s, const float* b_s, const float* w_fb,
                        const float* b_fb, const float* v, float b_e, const float* accum_in, float* accum_out,
                        float* a, void* att, int64_t ld_att, void* workspace, void* stream);

/* The decoder's readout (Listing 1, "readout": a linear layer with relu over the cell output s, the previous target
 * embedding trg and the attention context att):  out[r] = max(0, [s[r] | trg[r] | att[r]] W_r + b_r).
 *   s bfloat16 [B][ld_s >= n], trg bfloat16 [B][ld_trg >= n_trg], att bfloat16 [B][ld_att >= E]: three separate
 *   arrays with their own row strides (att may be where lstm_attention_step wrote it, trg and att may be the two
 *   halves of the cell's input rows); trg may be NULL if n_trg = 0, att if E = 0.
 *   W_r bfloat16 [R][n + n_trg + E] (a row per output feature, columns ordered s | trg | att), b_r float [R] or NULL,
 *   out bfloat16 [B][ld_out >= R]; workspace of lstm_readout_query(B, R, n, n_trg, E) bytes.
 *   flags: 0, or LSTM_FLAG_WEIGHTS_PACKED from the second call on: the caller states that W_r and the workspace
 *   are unchanged since the previous call, which left a copy of W_r with padded rows there (as for the stepped cell).
 *   Float accumulation, one rounding at the end.  Device pointers owned by the caller; the call only enqueues work.
 * Errors: LSTM_ERR_NULL, LSTM_ERR_DIM, LSTM_ERR_UNSUPPORTED (other flag bits), LSTM_ERR_ALIGN (element alignment),
 * LSTM_ERR_SIZE, LSTM_ERR_HIP. */
int lstm_readout_query(int B, int R, int n, int n_trg, int E, uint64_t* workspace_bytes);
int lstm_readout(int flags, int B, int R, const void* s, int64_t ld_s, int n, const void* trg, int64_t ld_trg, int n_trg,
                 const void* att, int64_t ld_att, int E, const void* W_r, const float* b_r, void* out, int64_t ld_out,
                 void* workspace, uint64_t workspace_bytes, void* stream);

/* One step of batched beam search, entirely on the device (Sec. 3 and Table 2: the decoder is a batched beam search that runs on
 * the GPU, beam size 12; Listing 1: "output_prob" is a softmax over the labels, "output" chooses from it, "trg" embeds
 * the choice).  The paper gives no further detail; this library's reading, with q a sentence, b one of its `beam`
 * hypotheses (row r = q * beam + b of the decoder batch) and v a label:
 *     cand[q, b, v] = score_in[q, b] + logits[r, v] - log sum_v' exp(logits[r, v'])
 *     the `beam` largest cand[q, :, :] become the new hypotheses of sentence q, best first: score_out[q, k], the
 *     hypothesis it extends src[q, k] in [0, beam) and its label[q, k] in [0, V); equal candidates are ordered by the
 *     smaller b * V + v.  A hypothesis with score -inf (the unused slots of the first step) never beats a finite one.
 * Finished hypotheses and length normalisation are not part of this step.  All arithmetic is float.
 *   logits float [Q*beam][ld >= V] (e.g. lstm_gemm of the readout with the output weights), score_in, score_out float
 *   [Q][beam], src, label int32 [Q][beam]; beam <= 16, V <= 2^26; workspace of lstm_beam_query() bytes.
 * lstm_beam_gather moves per-hypothesis state behind the choice: out[q*beam + k][0..width) = in[q*beam + src[q, k]][..]
 *   for rows of `width` elements of elem_bytes (2 or 4) bytes; in and out must be different buffers; values of src
 *   outside [0, beam) are clamped.
 * lstm_beam_gather_many does the same for `count` (1 .. 8) arrays in ONE launch: `items` is a HOST array, read during the
 *   call; every array follows the same `src`.  Rows are copied in the widest units their alignment allows.
 * lstm_embed is Listing 1's "trg": out[r] = W_trg[label[r]] + b_trg with W_trg bfloat16 [V][n], b_trg float [n] or NULL,
 *   out bfloat16 [B][ld_out >= n]; a label outside [0, V) gives the bias alone.
 * Device pointers owned by the caller; the calls only enqueue work and nothing is copied to the host.
 * Errors: LSTM_ERR_NULL, LSTM_ERR_DIM, LSTM_ERR_UNSUPPORTED (beam > 16, V > 2^26, elem_bytes, in == out),
 * LSTM_ERR_ALIGN, LSTM_ERR_SIZE, LSTM_ERR_HIP. */
int lstm_beam_query(int Q, int beam, int V, uint64_t* workspace_bytes);
int lstm_beam_step(int Q, int beam, int V, const float* logits, int64_t ld, const float* score_in, float* score_out,
                   int32_t* src, int32_t* label, void* workspace, uint64_t workspace_bytes, void* stream);
int lstm_beam_gather(int elem_bytes, int Q, int beam, int width, const void* in, int64_t ld_in, const int32_t* src,
                     void* out, int64_t ld_out, void* stream);
typedef struct lstm_gather_item {
  int32_t elem_bytes;          /* 2 or 4 */
  int32_t width;               /* elements per row */
  const void* in;              /* device [Q*beam][ld_in] */
  int64_t ld_in;               /* elements */
  void* out;                   /* device [Q*beam][ld_out], not `in` */
  int64_t ld_out;
} lstm_gather_item;
int lstm_beam_gather_many(int Q, int beam, int count, const lstm_gather_item* items, const int32_t* src, void* stream);
/* lstm_beam_step for callers that cannot allocate device memory or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  Same arguments without the workspace, same results (the
 * same kernels run).  The step's scratch - the beam survivors of every row - lives in a device array of 512 KiB that is
 * part of the library's image on every GPU it runs on; the call allocates and frees nothing.
 *   Limit: Q * beam * beam <= 65536 (e.g. 256 sentences at beam 16), else LSTM_ERR_SIZE.
 *   Every call on one GPU uses that GPU's one array: calls that may overlap in time on the same GPU (different
 *   streams, different host threads) race and must be serialised by the caller.  Nothing in the array has to survive
 *   between calls and nothing needs clearing: a call writes every entry it later reads.
 * Other errors as lstm_beam_step. */
int lstm_beam_step_static(int Q, int beam, int V, const float* logits, int64_t ld, const float* score_in, float* score_out,
                          int32_t* src, int32_t* label, void* stream);
int lstm_embed(int B, int n, int V, const int32_t* label, const void* W_trg, const float* b_trg, void* out,
               int64_t ld_out, void* stream);

/* Diagnostic for the single-launch (persistent) recurrent kernels, whose work-groups wait for each
 * other between time steps with BOUNDED waits.  If a wait ever expired, the kernel drained early, the
 * results of that call are invalid and a word in the workspace says so.  This call copies that word
 * to the host (it SYNCHRONISES the device) and stores 1 in *timed_out if it is set, else 0.  It refers
 * to the last *_fwd / *_bwd call that used `workspace` (every call clears the word first). */
int lstm_sync_status(const void* workspace, int32_t* timed_out);

/* Phase timing for benchmarks.  While enabled, every *_fwd / *_bwd call brackets its phases with
 * hipEvents recorded on the call's own stream (the only resource the library ever creates):
 * lstm_profile_enable(1) the recurrent loops and the hoisted products (LSTM_PHASE_GEMM_*, LSTM_PHASE_LOOP_*),
 * lstm_profile_enable(2) also the short phases around them (LSTM_PHASE_PREP, LSTM_PHASE_DB), 0 none.  An event
 * between two kernels costs a few microseconds of idle device, which is why the short phases are optional.
 * lstm_profile_read() waits for the recorded events, adds each phase's elapsed milliseconds and
 * kernel-launch count into ms[LSTM_PHASE_COUNT] / launches[LSTM_PHASE_COUNT] (caller zeroes them),
 * and releases the events.  Not thread-safe; meant for a single benchmarking thread. */
enum {
  LSTM_PHASE_PREP = 0,      /* weight / state packing, state initialisation and copies            */
  LSTM_PHASE_GEMM_ZX = 1,   /* Zx = X W_x + b for all frames                                      */
  LSTM_PHASE_LOOP_FWD = 2,  /* forward recurrence                                                 */
  LSTM_PHASE_LOOP_BWD = 3,  /* backward recurrence                                                */
  LSTM_PHASE_GEMM_DX = 4,   /* dX = DZ W_x^T                                                      */
  LSTM_PHASE_GEMM_DWX = 5,  /* dW_x = X^T DZ                                                      */
  LSTM_PHASE_GEMM_DWH = 6,  /* dW_h = Hprev^T DZ                                                  */
  LSTM_PHASE_DB = 7,        /* db = column sums of DZ                                             */
  LSTM_PHASE_COUNT = 8
};
int lstm_profile_enable(int on);
int lstm_profile_read(double* ms, int64_t* launches);

/* Static, human-readable text for a status code (never NULL). */
const char* lstm_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif
