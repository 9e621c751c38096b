/*
 * fmha_varlen -- fused multi-head attention over packed, unpadded
 * variable-length sequences for AMD MI355X (gfx950), forward and backward.
 *
 * The operation is the paper's Eq. 1, softmax(Q K^T / sqrt(d_k)) V, applied to
 * every sequence of a batch and every head on its own, on the paper's unpadded
 * storage (Section IV-A-1): the batch and sequence dimensions are merged, only
 * valid tokens are stored, and a prefix-sum array (the paper's batch_offset,
 * here cu_seqlens) says where each sequence begins.  The backward pass is the
 * derivative of Eq. 1 (the paper reports backward timings in Section IV-A-2
 * but prints no formula).
 *
 * In place of the paper's length groups run on separate streams and joined
 * with events (Section IV-A-2), all sequences are cut into tiles, the tiles
 * are ordered longest sequence first by a small device kernel, and one launch
 * per direction on the caller's stream consumes that list; stream order then
 * gives the "after the producer, before the consumer" guarantee the paper
 * needs events for.
 *
 * Besides the attention calls the library holds the operations the paper places around
 * them on the unpadded storage, each documented where it is declared: dropout on the
 * attention probabilities, the padded <-> unpadded conversions (Sections IV-A-1, IV-B-2),
 * the fused Dropout + Add + LayerNorm (Section IV-C-1) and the embedding backward
 * (Section IV-C-3).
 *
 * Conventions
 *   - Every pointer named "device" is GPU memory owned by the caller; the
 *     library never allocates, frees or copies to the host, and never
 *     synchronises: all work is enqueued on `stream` and the call returns.
 *   - Tensors are token-major: element (t, h, c) of Q is at
 *     q[t * q_stride + h * 64 + c], 0 <= t < total_tokens, 0 <= h < heads,
 *     0 <= c < 64, 16-bit elements (IEEE half or bfloat16).  A stride of 0
 *     means heads * 64 (dense).  Strides are in elements, must be
 *     multiples of 8 and at most 2^24; base pointers must be 16-byte aligned.
 *   - Sequence i owns rows cu_seqlens[i] .. cu_seqlens[i+1]-1.  Rows of
 *     different sequences never interact.  Empty sequences are allowed.
 *   - Inputs are read-only.  Outputs are fully overwritten for all rows.
 *   - Arithmetic: 16-bit operands, fp32 accumulation and fp32 softmax state;
 *     the probabilities are rounded to the operand type before they are
 *     multiplied with V (and dO), as is dS before it meets K and Q.
 *   - The workspace carries state from the forward to the backward call and
 *     between the two backward passes: calls that may overlap in time (other
 *     streams, other threads) need workspaces of their own.  The library keeps
 *     no other state, so such calls are safe.
 *   - Errors are return codes; fmha_last_error() gives a message for the last
 *     failing call on the calling thread.  Validation reads only host memory.
 */
#ifndef FMHA_VARLEN_H_
#define FMHA_VARLEN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FMHA_OK = 0,
  FMHA_ERR_INVALID_ARG = 1, /* null / misaligned pointer, bad size, bad stride, bad prefix sums */
  FMHA_ERR_UNSUPPORTED = 2, /* head_dim != 64, unknown dtype */
  FMHA_ERR_WORKSPACE = 3,   /* workspace missing or smaller than fmha_varlen_workspace_size() */
  FMHA_ERR_HIP = 4          /* a HIP launch failed */
} fmha_status_t;

typedef enum { FMHA_F16 = 0, FMHA_BF16 = 1 } fmha_dtype_t;

/* The workspace already holds the tile list for exactly this cu_seqlens /
 * seqused / batch: skip rebuilding it.  A training step calls attention once
 * per layer and direction with the same batch, as the paper computes its
 * batch_offset once per mini-batch (Section IV-B-2). */
#define FMHA_FLAG_REUSE_SCHEDULE 1u
/* fmha_varlen_bwd only: run one of the two backward passes.  The dQ pass also
 * writes the per-row statistics into the workspace; the dK/dV pass reads them,
 * so a dK/dV-only call must follow a dQ pass on the same workspace and inputs.
 * The output pointers of the skipped pass are still validated but not written. */
#define FMHA_FLAG_BWD_ONLY_DQ 2u
#define FMHA_FLAG_BWD_ONLY_DKV 4u

typedef struct fmha_varlen_params {
  int32_t batch;        /* number of sequences B >= 0 */
  int32_t total_tokens; /* T = cu_seqlens[B] */
  int32_t heads;        /* H >= 1 */
  int32_t head_dim;     /* must be 64 */
  int32_t max_seqlen;   /* upper bound on the longest sequence, or <= 0 if unknown.  It only
                           sizes the launch (the kernels stride over the tile list, so a
                           wrong value costs time, not correctness); a value smaller than a
                           length seen in cu_seqlens_host is reported as an error */
  int32_t dtype;        /* fmha_dtype_t */
  uint32_t flags;       /* FMHA_FLAG_* */
  float scale;          /* multiplies Q K^T; 1/sqrt(64) = 0.125 for Eq. 1 */
  int64_t q_stride, k_stride, v_stride, o_stride;     /* elements between tokens, 0 = dense */
  int64_t do_stride, dq_stride, dk_stride, dv_stride; /* backward only, 0 = dense */
  const int32_t* cu_seqlens;      /* device, B+1 entries, cu[0] = 0, non-decreasing */
  const int32_t* cu_seqlens_host; /* optional host copy: lets the call validate the prefix sums */
  const int32_t* seqused;         /* optional device, B entries: only keys j < seqused[i] of
                                     sequence i are attended (padded layout with a key mask);
                                     NULL = all L_i keys.  Values are clamped to [0, L_i]; with no
                                     key attended the rows get O = 0, LSE = -inf and zero
                                     gradients.  All L_i query rows are computed. */
  void* workspace;                /* device, 256-byte aligned, see fmha_varlen_workspace_size */
  size_t workspace_bytes;
} fmha_varlen_params_t;

/* Bytes of device workspace for a batch of this shape (tile list; plus, if
 * need_bwd, two fp32 per (token, head): the row sums of dO o O and the
 * log-sum-exp in base-2 units).  Pure host arithmetic; returns 0 on invalid sizes. */
size_t fmha_varlen_workspace_size(int32_t batch, int32_t total_tokens, int32_t heads,
                                  int32_t need_bwd);

/* Forward: O = softmax(scale * Q K^T) V per sequence and head (Eq. 1).
 *   q, k, v : device, [T, H, 64] with the strides in p (read)
 *   o       : device, [T, H, 64] (written)
 *   lse     : device, fp32 [H, T]: natural-log sum of exp of the scaled scores of each row
 *             (written; needed by the backward call)
 *   stream  : hipStream_t (NULL = default stream)
 * Returns an fmha_status_t. */
int fmha_varlen_fwd(const fmha_varlen_params_t* p, const void* q, const void* k, const void* v,
                    void* o, float* lse, void* stream);

/* fmha_varlen_fwd for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the tile list lives in a
 * device array built into the library instead of a caller workspace, and the call makes no
 * hipMalloc / hipFree and calls no allocating routine.  p->workspace and
 * p->workspace_bytes are ignored; everything else (arguments, results, error codes) is as
 * for fmha_varlen_fwd, whose kernels it shares.
 *   - Limit: fmha_varlen_workspace_size(batch, total_tokens, heads, 0) must not exceed
 *     fmha_varlen_static_scratch_bytes() (1 MiB: about 65 000 tiles); larger batches are
 *     rejected with FMHA_ERR_WORKSPACE and nothing is launched.
 *   - Every GPU the library runs on holds its own copy of that array until the process
 *     ends; its address is looked up on the first call on a device.
 *   - All calls on one GPU share the array, which keeps the previous call's tile list:
 *     every call rebuilds the list before using it (FMHA_FLAG_REUSE_SCHEDULE reuses the
 *     list the previous such call on this GPU left there), and calls that overlap in time
 *     on one GPU (other streams, other threads) race on it - serialise them, or use
 *     fmha_varlen_fwd with separate workspaces. */
size_t fmha_varlen_static_scratch_bytes(void);
int fmha_varlen_fwd_static(const fmha_varlen_params_t* p, const void* q, const void* k, const void* v,
                           void* o, float* lse, void* stream);

/* Backward: given dO, recompute the probabilities from q, k and lse and write
 *   dV = P^T dO,  dP = dO V^T,  dS = P o (dP - rowsum(dO o O)),
 *   dQ = scale dS K,  dK = scale dS^T Q.
 *   q, k, v, o, d_o : device [T, H, 64] (read);  lse : device fp32 [H, T] from the forward call
 *   dq, dk, dv      : device [T, H, 64] (written; rows of keys masked by seqused get zeros)
 * Needs a workspace sized with need_bwd = 1. */
int fmha_varlen_bwd(const fmha_varlen_params_t* p, const void* q, const void* k, const void* v,
                    const void* o, const void* d_o, const float* lse, void* dq, void* dk,
                    void* dv, void* stream);

/* ---- Dropout on the attention probabilities -------------------------------
 * BERT trains with dropout on the attention probabilities (the model of the
 * paper's Section V-A); the paper does not describe how its attention kernel
 * draws it.  Here the mask is a pure function of (seed, sequence start, head,
 * query, key), so the backward call regenerates the mask the forward call used
 * and nothing is stored:
 *   - the 4 x 4 block (Q4, K4) = (q >> 2, k >> 2) of the score matrix of the
 *     sequence that starts at packed row r0, head h (q, k counted from the start
 *     of the sequence) owns one call of the counter-based generator Philox4x32
 *     with 10 rounds (Salmon, Moraes, Dror, Shaw, SC 2011), counter words
 *     (K4, Q4, r0, h), key words (seed & 0xffffffff, seed >> 32);
 *   - with B[x][y] = byte y (little endian) of output word x, element (q, k)
 *     reads x = ((q & 3) - (k >> 3)) & 3 and y = ((k & 3) - (q >> 3)) & 3;
 *   - the element is kept iff that byte >= t, t = round(256 p) clamped to
 *     [0, 255]: the probability applied is t / 256, and what is kept is
 *     multiplied by 256 / (256 - t).
 * Forward:  O = (P o M) V with M the scaled mask; LSE is that of the undropped
 * softmax.  Backward: dV = (P o M)^T dO, dP = (dO V^T) o M, the rest as without
 * dropout.  A caller wanting a fresh mask per layer and step passes a fresh seed. */
typedef struct fmha_dropout {
  float p;       /* drop probability, 0 <= p < 1; applied as round(256 p) / 256 */
  uint64_t seed; /* generator key */
} fmha_dropout_t;

/* fmha_varlen_fwd / fmha_varlen_bwd with dropout; `dropout` is host memory, read
 * during the call.  All other arguments, conventions and error codes as above;
 * p outside [0, 1) or a null `dropout` -> FMHA_ERR_INVALID_ARG.  The backward call
 * must be given the p and seed of the forward call that produced o and lse. */
int fmha_varlen_fwd_dropout(const fmha_varlen_params_t* p, const fmha_dropout_t* dropout,
                            const void* q, const void* k, const void* v, void* o, float* lse,
                            void* stream);
int fmha_varlen_bwd_dropout(const fmha_varlen_params_t* p, const fmha_dropout_t* dropout,
                            const void* q, const void* k, const void* v, const void* o,
                            const void* d_o, const float* lse, void* dq, void* dk, void* dv,
                            void* stream);

/* Writes the keep mask itself, for tests and debugging: mask is device memory,
 * heads * total_tokens rows of row_bytes bytes (row_bytes >= the longest sequence,
 * and >= max_seqlen if that is given); byte k of row h * total_tokens + t becomes 1 if
 * key k of token t's sequence is kept for query t under head h, else 0, for k < L of
 * that sequence; other bytes are left alone.  orientation 0 / 1 selects the code path
 * of the forward and dQ kernels / of the dK/dV kernel; both write the same mask.
 * Uses the workspace for the tile list like the other calls. */
int fmha_dropout_keep_mask(const fmha_varlen_params_t* p, const fmha_dropout_t* dropout,
                           int32_t orientation, int32_t row_bytes, uint8_t* mask, void* stream);

/* ---- Between the padded input format and the unpadded storage -----------------
 * The paper compresses the [batch, max_seq_len] inputs to the unpadded format with a
 * gather before the embedding and restores the padded format with a scatter before
 * the pooler (Section IV-A-1); the positions to keep are where input_mask is non-zero
 * (nonzero_indices) and the tokens per sequence give batch_offset (Section IV-B-2).
 * The paper computes nonzero_indices and batch_offset on the CPU, one batch ahead,
 * because on the GPU the number of valid tokens is not known to the host without a
 * synchronisation.  Both routes are offered: a host routine, and a device one that
 * needs no synchronisation because every consumer reads the token count from device
 * memory (cu_seqlens[batch]) and the caller sizes buffers for the worst case.
 * The paper does not say what scatter leaves in padding rows: zeros here. */

/* Host arrays in, host arrays out (plain loops, no GPU involved).
 *   input_mask      : [batch, seqlen] row-major; a token is valid iff its entry is non-zero
 *   nonzero_indices : batch*seqlen entries of room, or NULL; receives the flat positions
 *                     b*seqlen+s of the valid tokens in ascending order
 *   inverse         : batch*seqlen entries, or NULL; receives for every flat position its
 *                     rank among the valid ones (= its packed row), or -1 for padding
 *   cu_seqlens      : batch+1 entries; receives the prefix sums of the valid tokens per row
 *   max_seqlen      : NULL or one entry; receives the largest number of valid tokens in a row */
int fmha_unpad_indices_host(const int32_t* input_mask, int32_t batch, int32_t seqlen,
                            int32_t* nonzero_indices, int32_t* inverse, int32_t* cu_seqlens,
                            int32_t* max_seqlen);

/* The same on the device: all arrays are device memory (inverse may be NULL), sizes as
 * above; three small launches on `stream`, no host synchronisation.  Entries of
 * nonzero_indices at and beyond cu_seqlens[batch] are left alone. */
int fmha_unpad_indices(const int32_t* input_mask, int32_t batch, int32_t seqlen,
                       int32_t* nonzero_indices, int32_t* inverse, int32_t* cu_seqlens,
                       void* stream);

/* gather: packed row j <- padded row nonzero_indices[j] for j < *n_rows.
 *   padded  : device, padded_rows rows of row_bytes bytes (read)
 *   packed  : device, room for packed_rows rows (written for j < min(*n_rows, packed_rows);
 *             the rest is left alone)
 *   n_rows  : device, one int32 - normally cu_seqlens + batch
 *   row_bytes must be a multiple of 16 and the buffers 16-byte aligned; an index outside
 *   [0, padded_rows) produces a row of zeros. */
int fmha_gather_rows(const void* padded, int32_t padded_rows, const int32_t* nonzero_indices,
                     const int32_t* n_rows, int32_t packed_rows, int64_t row_bytes, void* packed,
                     void* stream);

/* scatter: padded row r <- packed row inverse[r] if 0 <= inverse[r] < min(*n_rows,
 * packed_rows), else zeros; all padded_rows rows are written.  Same layout rules as gather. */
int fmha_scatter_rows(const void* packed, int32_t packed_rows, const int32_t* inverse,
                      const int32_t* n_rows, int32_t padded_rows, int64_t row_bytes, void* padded,
                      void* stream);

/* ---- Dropout + Add + LayerNorm on the packed rows ---------------------------
 * The paper fuses the Dropout, Add and LayerNorm operators of the encoder into one
 * forward and two backward kernels (Section IV-C-1) and gives no formulas; these are
 * the operators' definitions, per row of the [rows, hidden] hidden states:
 *   forward   z = dropout(x) + residual,  mu = mean(z),  rstd = 1 / sqrt(var(z) + eps)
 *             (biased variance),  y = (z - mu) rstd gamma + beta
 *   backward  g = dy gamma,  xh = (z - mu) rstd,
 *             dz = rstd (g - mean(g) - xh mean(g xh)),  dresidual = dz,  dx = dropout'(dz),
 *             dgamma = sum over rows of dy xh,  dbeta = sum over rows of dy
 * dropout(x) = x o M / (1 - p') with p' = round(256 p) / 256 and the mask regenerated
 * from the seed in both directions: element (row t, column c) is kept iff byte c & 15
 * (byte c & 3 of output word (c >> 2) & 3) of the Philox4x32-10 call with counter words
 * (c >> 4, t, 0x4C4E, 0) and key words (seed & 0xffffffff, seed >> 32) is >= round(256 p).
 * x, residual, y, z, dy, dx, dresidual are [rows, hidden] 16-bit (dtype), dense rows;
 * gamma, beta, dgamma, dbeta are fp32 [hidden]; mu, rstd fp32 [rows].  Arithmetic in
 * fp32; z is stored rounded to 16 bits and the backward works from that stored z. */
typedef struct fmha_ln_params {
  int32_t rows;          /* rows the buffers hold (T, or the worst case batch * max_seq_len) */
  int32_t hidden;        /* multiple of 16, at most 4096 */
  int32_t dtype;         /* fmha_dtype_t */
  float eps;             /* >= 0 */
  const int32_t* n_rows; /* optional device int32: rows actually present (clamped to [0, rows]),
                            e.g. cu_seqlens + batch; rows beyond it are neither read nor written */
  fmha_dropout_t dropout; /* p = 0: no dropout */
} fmha_ln_params_t;

/* Forward; y, z, mu, rstd are written, everything else read.  One launch. */
int fmha_dropout_add_ln_fwd(const fmha_ln_params_t* p, const void* x, const void* residual,
                            const float* gamma, const float* beta, void* y, void* z, float* mu,
                            float* rstd, void* stream);

/* Bytes of device workspace the backward needs (per-workgroup column sums); 0 on invalid sizes. */
size_t fmha_dropout_add_ln_bwd_workspace_size(int32_t rows, int32_t hidden);

/* Backward; z, mu, rstd are the forward's outputs; dx, dgamma, dbeta are written, and
 * dresidual unless it is NULL (without dropout it equals dx).  Two launches; the column
 * sums are added in a fixed order, so results are reproducible run to run. */
int fmha_dropout_add_ln_bwd(const fmha_ln_params_t* p, const void* dy, const void* z, const float* mu,
                            const float* rstd, const float* gamma, void* dx, void* dresidual,
                            float* dgamma, float* dbeta, void* workspace, size_t workspace_bytes,
                            void* stream);

/* ---- Backward of the embedding lookup ----------------------------------------
 * Section IV-C-3 of the paper: the rows of the output gradient that share an index are
 * accumulated into that row of the weight gradient, collisions resolved by atomic adds on
 * packed pairs of 16-bit values (two adjacent columns per operation) with a fine work
 * split.     dw[indices[t]][c] += dy[t][c]   for every row t < rows (and < *n_rows).
 *   dy      : device, [rows, hidden] 16-bit (dtype), dense (read)
 *   indices : device, int32 [rows]; entries outside [0, vocab) or equal to padding_idx
 *             (pass -1 for none) contribute nothing
 *   n_rows  : optional device int32 (rows actually present), NULL = rows
 *   dw      : device, [vocab, hidden] 16-bit, 16-byte aligned; ACCUMULATED INTO, unless
 *             FMHA_EMB_ZERO_FIRST asks for it to be cleared first (a fill kernel on `stream`)
 *   hidden must be a multiple of 8.
 * The additions happen in the 16-bit type, each rounded to nearest, in an order that is
 * not fixed: a weight row that receives n rows carries an error of at most n half-ulps of
 * the largest partial sum, and results can differ in the last bits from run to run; rows
 * that receive one gradient row are exact.
 * FMHA_EMB_PLAIN_SPLIT selects the token-major work split (wavefront w takes tokens w, w+W,
 * ...) instead of the default, in which the tokens are divided among the chip's dies by
 * index modulo 8 so that each weight row is only ever updated from one die's L2. */
#define FMHA_EMB_ZERO_FIRST 1u
#define FMHA_EMB_PLAIN_SPLIT 2u
#define FMHA_EMB_NO_DIE_SPLIT 4u
int fmha_embedding_bwd(const void* dy, const int32_t* indices, const int32_t* n_rows, int32_t rows,
                       int32_t hidden, int32_t vocab, int32_t padding_idx, int32_t dtype,
                       uint32_t flags, void* dw, void* stream);

/* The same without atomics, in two calls, for callers that know the indices before the
 * gradient arrives (the paper computes its index tensors once per mini-batch, Section
 * IV-B-2; Section IV-C-3 names the colliding additions as the cost of this step):
 *   fmha_embedding_sort        orders the token positions by index (a stable radix sort on
 *                              the device) into `workspace`;
 *   fmha_embedding_bwd_sorted  sums the gradient rows of every index in that order in fp32,
 *                              adds the weight row that is there (unless FMHA_EMB_ZERO_FIRST,
 *                              which clears all of dw first) and writes the row once, rounded
 *                              once to the 16-bit type.
 * Tokens are skipped as in fmha_embedding_bwd (index outside [0, vocab), index ==
 * padding_idx, position >= *n_rows).  Every weight row has one writer and every sum a fixed
 * order, so results are identical from run to run, and a row that receives n gradient rows
 * carries the error of an fp32 sum of n terms plus one rounding.
 *   workspace : device, 256-byte aligned, fmha_embedding_sort_workspace_size(rows, hidden)
 *               bytes; written by the sort, read and written by the backward call (partial
 *               sums), reusable for any number of backward calls on the same indices.
 * rows, hidden, vocab of the two calls must agree (the workspace layout depends on rows and
 * hidden); FMHA_EMB_PLAIN_SPLIT / NO_DIE_SPLIT have no meaning here and are rejected.
 * Errors as above, FMHA_ERR_WORKSPACE for a missing, misaligned or short workspace. */
size_t fmha_embedding_sort_workspace_size(int32_t rows, int32_t hidden);
int fmha_embedding_sort(const int32_t* indices, const int32_t* n_rows, int32_t rows, int32_t hidden,
                        int32_t vocab, int32_t padding_idx, void* workspace, size_t workspace_bytes,
                        void* stream);
int fmha_embedding_bwd_sorted(const void* dy, void* workspace, size_t workspace_bytes, int32_t rows,
                              int32_t hidden, int32_t vocab, int32_t dtype, uint32_t flags, void* dw,
                              void* stream);

/* Number of 128-row tiles the schedule holds at most for this shape (host
 * arithmetic), and a device-to-host-free way for tests to locate the tile list
 * inside the workspace: the list starts at byte offset *list_offset and holds
 * int32 quadruples (packed row at which the sequence starts, its length, its
 * number of attended keys, first row of the tile within the sequence); its
 * length is the int32 at byte offset *count_offset. */
int32_t fmha_varlen_schedule_info(int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                                  size_t* count_offset, size_t* list_offset);

/* Message for the last error returned on this thread ("" if none). */
const char* fmha_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FMHA_VARLEN_H_ */
