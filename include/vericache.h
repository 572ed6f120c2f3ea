/*
 * vericache.h - C ABI of the MI355X (gfx950) draft / verify / accept / swap-in hot path of
 * VeriCache (arXiv 2605.17613): draft tokens against a compressed KV cache, verify them against
 * the full KV cache, accept greedily.
 *
 * Conventions that hold for every call
 *   - "device" pointers are HIP device memory of the GPU the context was created on, "host"
 *     pointers are ordinary process memory.  Every data pointer is borrowed: the library neither
 *     frees nor keeps it beyond the call (vc_swap_in keeps src/dst until the tickets complete).
 *   - Scratch memory is a caller-provided device workspace, sized by the *_workspace_bytes query.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *     and return; they never synchronise the device and never allocate device memory (vc_create
 *     alone allocates: the context's counter arrays, about 2.3 MB, freed by vc_destroy).
 *   - A context is used by one host thread at a time; contexts are independent of each other.
 *   - Errors are return codes; vc_last_error() gives a message for the last failing call on the
 *     calling thread.  Arguments are validated on the host in O(1) (null pointers, 16-byte
 *     alignment, head_dim == 128, group geometry); data-dependent contents (index ranges,
 *     sortedness) are the caller's contract and are not read by the host.
 *   - head_dim is 128.  n_q_heads must be a multiple of n_kv_heads with a ratio of at most 16;
 *     query head h uses KV head h / (n_q_heads / n_kv_heads).
 *   - bf16 tensors are raw 16-bit patterns.  A "bf16 pool" is token-major: row (token t, KV
 *     head h) is 128 consecutive bf16 at element offset (t * n_kv_heads + h) * 128.
 *   - Ragged batches use prefix-sum arrays cu_x of n_seqs + 1 int32 on the DEVICE; the matching
 *     max_x is the largest per-sequence count, given on the host so grids can be sized without
 *     a device round trip.  max_x may over-estimate; it must not under-estimate.
 */
#ifndef VERICACHE_H
#define VERICACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  VC_OK = 0,
  VC_ERR_INVALID_ARG = 1,  /* null / misaligned pointer, negative size, bad geometry          */
  VC_ERR_UNSUPPORTED = 2,  /* head_dim != 128, GQA ratio > 16, window too long, bits not 4/2     */
  VC_ERR_WORKSPACE = 3,    /* workspace missing or smaller than the query says                */
  VC_ERR_HIP = 4,          /* a HIP runtime call failed (message holds hipGetErrorString)     */
  VC_ERR_NOT_READY = 5     /* vc_swap_query: the ticket's copy has not finished yet           */
} vc_status;

typedef struct vc_ctx vc_ctx; /* opaque: owns one copy stream, the chunk and mark events, and the counter
                                 arrays of the one-launch forms of vc_accept_len and vc_draft_attn */

/* Create / destroy a context bound to HIP device `device`. */
vc_status vc_create(int device, vc_ctx** out);
vc_status vc_destroy(vc_ctx* ctx);
/* Message of the last failing call on this thread (static storage, never freed by the caller). */
const char* vc_last_error(void);
/* Library version, "major.minor". */
const char* vc_version(void);
/* Launch-shape tunables (sweeps and tests; the defaults are the measured optima).  They steer how
 * work is cut into workgroups - never a result - but the workspace sizes and the chunk length that
 * vc_verify_plan reports depend on them.  Each is read from the environment variable of its name
 * once, when the library first needs one; vc_set_tunable overrides it for the process (value < 0:
 * back to the library's default).  Changing one between a *_workspace_bytes query and its call, or
 * between the calls of one streamed verify, is the caller's error.  Names:
 *   VC_DRAFT_BF16_WGS, VC_DRAFT_QUANT_WGS   workgroups a draft launch is cut for
 *   VC_DRAFT_MIN_TOK, VC_DRAFT_MIN_BLK      shortest split (tokens / block records)
 *   VC_DRAFT_FLAT                           0: ragged batches of at most 64 sequences are launched
 *                                           like larger ones (a grid over the longest sequence's splits)
 *   VC_DRAFT_ROW_WAVES                      2 or 4 waves per workgroup of the bf16 row kernel (default: 2 for
 *                                           ragged batches - two workgroups share a compute unit - else 4)
 *   VC_DRAFT_FUSED                          largest launch (workgroups) of a single-source draft call that finishes
 *                                           inside its split kernel instead of in a merge launch (default 64; 0: none)
 *   VC_DRAFT_TAIL_SPLIT                     0: the merge launch attends to the bf16 tail itself (default 1: workgroups
 *                                           of the split launch do, and hand the merge one more partial)
 *   VC_VERIFY_WGS, VC_VERIFY_MIN_TOK        workgroups a verify launch is cut for, shortest chunk
 *   VC_VERIFY_WORKLIST, VC_VERIFY_LIST_MIN, VC_VERIFY_TAPER, VC_VERIFY_QUEUE_WGS   the work-list
 *                                           launch of large ragged batches
 *   VC_ACCEPT_FUSED                         0: the accept call finishes in a second launch
 * Unknown names return VC_ERR_INVALID_ARG. */
vc_status vc_set_tunable(const char* name, int32_t value);
vc_status vc_get_tunable(const char* name, int32_t* value, int32_t* is_set);
/* State of the work enqueued on `stream` so far, without blocking: VC_OK when it has all finished,
 * VC_ERR_NOT_READY while some is in flight, VC_ERR_HIP when the runtime reports a failure of earlier
 * asynchronous work (a launch failure is returned by the call that launched; a fault inside a
 * running kernel is reported by the runtime to a later call that touches the stream - this one,
 * vc_swap_query, vc_swap_sync). */
vc_status vc_stream_status(vc_ctx* ctx, void* stream);
/* Measurement aid.  Arms two caller-owned hipEvent_t (passed as void*, created with timing
 * enabled): the next vc_draft_attn or vc_verify_attn[_range] call on this context records
 * `begin_event` on its stream just before its main attention kernel(s) and `end_event` just after
 * them, i.e. without the merge kernel that follows, then disarms.  Pass two NULLs to disarm.
 * The events must stay alive until that call has been made. */
vc_status vc_time_main_kernel(vc_ctx* ctx, void* begin_event, void* end_event);

/* ------------------------------------------------------------------------------------------
 * Compressed KV of one attention layer for a ragged batch (paper section 6: all the runtime needs
 * to know of a compressed cache is its set of dropped positions and its element width).  The drafted token of sequence b
 * attends to the union of three sources, each of which may be absent or empty:
 *
 *  (1) bf16 rows of a pool, either all rows of the sequence or the rows a kept-index list names
 *      (token dropping, bit scheme 16; every KV head of a sequence keeps the same count).
 *        pool_k, pool_v  device bf16 pools; sequence b owns rows cu_ctx[b] .. cu_ctx[b+1]-1
 *        keep_idx        device int32 or NULL.  List (b, h) is keep_idx[(cu_keep[b]*n_kv_heads
 *                        + h*nk) + i], i < nk = cu_keep[b+1]-cu_keep[b]; entries are positions
 *                        relative to the sequence start, in [0, length).  NULL = every row.
 *        max_keep        host: max over b of nk (of the length when keep_idx is NULL)
 *
 *  (2) group-quantised block records (bit scheme 4 or 2; keys quantised per channel over the TB
 *      tokens of a block, values per token over groups of TB channels; TB = 32 for 4 bit, 64 for
 *      2 bit; x = scale * code + zero with fp16 scale and zero).
 *        blocks          device, 5120-byte records.  (b, h) owns records cu_blk[b]*n_kv_heads +
 *                        h*nb + i, i < nb = cu_blk[b+1]-cu_blk[b]; record i holds tokens
 *                        i*TB .. i*TB+TB-1 of whatever token list was compressed.
 *      Record layout (all multi-byte fields little endian).  Codes are packed into 32-bit words
 *      of E = 32/bits elements; element e of a word is the `bits`-wide field at bit
 *      16*(e mod 2) + bits*(e / 2)  (even elements fill the low half-word, odd ones the high):
 *        bytes    0..2047  key codes, token-major: token t owns words 4*bits*t .. 4*bits*t +
 *                          4*bits-1; word wi of a token holds channels E*wi .. E*wi+E-1
 *        bytes 2048..4095  value codes, 128 slots of 16 bytes; slot 64*c + 16*j + n (c<2, j<4,
 *                          n<16) holds words q<4; word q is channel d = 64*c + 16*q + n and holds
 *                          tokens E*j .. E*j+E-1 of the block
 *        bytes 4096..4607  key scale[128] then key zero[128] (fp16, per channel)
 *        bytes 4608..5119  value scale[g][t] then value zero[g][t] (fp16; g = d / TB < 128/TB,
 *                          t < TB), 128 + 128 values
 *
 *      Number range.  The kernel folds scales and zero points into fp16 operands of the matrix
 *      cores (products are accumulated in fp32), so metadata must stay inside fp16 after folding:
 *        values:  value scale <= 4094 and |value zero| <= 4094 (a probability operand reaches 16);
 *        keys:    |q[d]| * softmax_scale * 1.4427 * max(key scale[d], |key zero[d]|) <= 65504.
 *      Beyond that the output is undefined (infinities).  N(0,1)-scale caches with key outlier
 *      channels of x100 and values of a few thousand are inside the range.
 *
 *  (3) a bf16 tail of recent tokens (tokens drafted in this horizon, and the remainder of a
 *      context that does not fill a whole block): pools tail_k, tail_v, rows cu_tail[b] ..
 *      cu_tail[b+1]-1.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t n_seqs, n_q_heads, n_kv_heads, head_dim;
  int32_t bits;            /* bit scheme of `blocks`: 4 or 2 (ignored when blocks is NULL) */
  int32_t max_keep, max_blk, max_tail;
  int32_t sum_keep, sum_blk;  /* host hints: sum over sequences of nk / nb (0 = unknown, n_seqs*max is
                                 assumed); they only steer the load balance, never the result */
  const void* pool_k;      /* (1) */
  const void* pool_v;
  const int32_t* cu_ctx;
  const int32_t* keep_idx;
  const int32_t* cu_keep;  /* required when keep_idx is given */
  const void* blocks;      /* (2) */
  const int32_t* cu_blk;
  const void* tail_k;      /* (3) */
  const void* tail_v;
  const int32_t* cu_tail;
} vc_comp_kv;

/* Draft attention (paper section 4.1 step 1; section 4.2.1: bounded by HBM bandwidth).
 * For every sequence b and query head h:  s_j = softmax_scale * <q, K_j>, p = softmax(s),
 * out = sum_j p_j V_j over the keys described above, accumulated in fp32.
 *   q    device bf16 [n_seqs, n_q_heads, 128]
 *   out  device bf16 [n_seqs, n_q_heads, 128]
 *   lse  device fp32 [n_seqs, n_q_heads] or NULL: natural-log sum of exp(s_j)
 * A sequence with no keys at all gets out = 0 and lse = -inf.
 * Tiny single-source calls (up to 64 workgroups, see VC_DRAFT_FUSED) are one launch that counts its
 * workgroups on one of 16 sets of counters the context owns (call i uses set i mod 16): at most 16 such
 * calls made through one context may be in flight, or captured in graphs that run, at the same time. */
vc_status vc_draft_workspace_bytes(const vc_comp_kv* kv, size_t* bytes);
vc_status vc_draft_attn(vc_ctx* ctx, const vc_comp_kv* kv, const void* q, float softmax_scale,
                        void* out, float* lse, void* workspace, size_t workspace_bytes,
                        void* stream);

/* Optional validation of the data the host cannot see (paper section 6: the runtime is handed
 * per-request offsets and position lists by the compressor; the attention calls trust them).
 * Asynchronous: a short kernel on `stream` checks the device arrays of the descriptor and writes
 *   report[0] = number of violations found
 *   report[1] = the smallest violation as (kind << 56 | sequence << 32 | index), or -1 for none
 * to `report` (device, int64[2], 8-byte aligned); the caller reads it once the stream got there.
 * Kinds: see vc_violation; `index` is the entry of the kept list for the KEEP kinds, the array
 * (0 cu_ctx, 1 cu_keep, 2 cu_blk, 3 cu_tail, 4 cu_win, 5 total_win) for the others.
 * vc_validate_comp_kv: every prefix array the descriptor uses is non-decreasing; no per-sequence
 *   count exceeds its host-side maximum (max_keep, max_blk, max_tail - launch grids are sized from
 *   them); a kept list has at most len_b entries, each in [0, len_b), strictly ascending.
 * vc_validate_full_kv: cu_ctx and cu_win (may be NULL) non-decreasing, lengths within max_ctx /
 *   max_win, cu_win[n_seqs] - cu_win[0] == total_win. */
typedef enum {
  VC_BAD_PREFIX_ORDER = 1,  /* a cu_* array decreases                                  */
  VC_BAD_HOST_MAX = 2,      /* a per-sequence count exceeds the host-side maximum        */
  VC_BAD_KEEP_COUNT = 3,    /* a kept list is longer than its sequence                   */
  VC_BAD_KEEP_RANGE = 4,    /* a kept position outside [0, len_b)                        */
  VC_BAD_KEEP_ORDER = 5     /* kept positions not strictly ascending                     */
} vc_violation;
vc_status vc_validate_comp_kv(vc_ctx* ctx, const vc_comp_kv* kv, int64_t* report, void* stream);

/* vc_draft_attn for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks,
 * kernels and results as vc_draft_attn, but the split partials go to a fixed scratch array that is
 * part of the library's device image (vc_draft_static_scratch_bytes reports its size, 8 MiB; every
 * GPU the library runs on holds one until the process ends).  The call allocates nothing.  A batch
 * whose vc_draft_workspace_bytes exceeds the scratch is refused with VC_ERR_WORKSPACE and nothing is
 * enqueued.  All calls on one GPU share that GPU's array: calls that may overlap on one GPU (two
 * streams, two threads) race - serialise them or use vc_draft_attn with separate workspaces.
 * Nothing in the scratch has to start at zero (every partial is written before it is read), so the
 * contents a previous call left behind are harmless. */
vc_status vc_draft_static_scratch_bytes(size_t* bytes);
vc_status vc_draft_attn_static(vc_ctx* ctx, const vc_comp_kv* kv, const void* q, float softmax_scale,
                               void* out, float* lse, void* stream);

/* Full KV of one layer, resident on the device (the destination of vc_swap_in). */
typedef struct {
  int32_t n_seqs, n_q_heads, n_kv_heads, head_dim;
  int32_t max_ctx, max_win;
  int32_t sum_ctx;         /* host hint: sum of context lengths (0 = unknown); load balance only.  A batch
                              whose sum is well below n_seqs * max_ctx is cut into shorter chunks, and a
                              large one (up to 512 sequences) is verified from a work list that a small
                              kernel builds in the workspace, by one workgroup per CU.  Results do not
                              depend on the hint; the workspace size does, so pass the same value to
                              every call of one verify.  Every vc_verify_attn_range call on such a
                              batch rebuilds the list (about 15 us): a caller that streams sequence by
                              sequence does better with one descriptor per sequence (n_seqs = 1). */
  int32_t chunk_tokens;    /* tokens per workgroup chunk (a multiple of 128), 0 = the library picks;
                              set it to the swap-in chunk length to verify chunk by chunk */
  const void* k;           /* device bf16 pools; sequence b owns rows cu_ctx[b] .. cu_ctx[b+1]-1 */
  const void* v;
  const int32_t* cu_ctx;
  /* Staging ring (paper section 5.1, HBM ring: the full KV that is in flight for an upcoming verify
   * but not yet consumed).  ring_slots = 0: k, v hold every token, as above.  ring_slots = R > 0: k and
   * v are R slots of chunk_tokens rows each (row s * chunk_tokens + i of the pools is token i of the
   * chunk in slot s), cu_ctx still gives the sequence lengths, and only vc_verify_attn_range /
   * vc_verify_finish may be used: a range call covers one chunk [tok_begin, tok_begin + chunk_tokens)
   * of each of its sequences (a tok_end past the end of every sequence means the rest of that chunk,
   * window tokens included), and reads that chunk of sequence b from slot ring_slot[b].  A slot may be
   * overwritten (vc_swap_in) once the range call that reads it has run: vc_mark after that call and
   * vc_swap_after before the reload order the two on the device. */
  int32_t ring_slots;
  const int32_t* ring_slot; /* device int32 [n_seqs], entries in [0, ring_slots); read by the range call */
} vc_full_kv;

/* Verify attention (paper section 4.1 step 2).  Sequence b brings w_b = cu_win[b+1]-cu_win[b]
 * drafted positions (0 allowed; w_b * n_q_heads / n_kv_heads <= 4096 rows per KV head - up to 256 rows, i.e.
 * w_b <= 64 at a GQA ratio of 4 or 32 at a ratio of 8, the full KV is streamed once; beyond that once per
 * 256 rows).  Window row i of head h attends to the sequence's
 * full KV and to window rows 0..i (its own position included):
 *   q_win         device bf16 [sum w, n_q_heads, 128]
 *   k_win, v_win  device bf16 pools [sum w, n_kv_heads, 128]
 *   out           device bf16 [sum w, n_q_heads, 128];  lse device fp32 [sum w, n_q_heads] or NULL
 * bf16 MFMA, fp32 accumulation. */
vc_status vc_validate_full_kv(vc_ctx* ctx, const vc_full_kv* kv, const int32_t* cu_win, int32_t total_win,
                              int64_t* report, void* stream);
vc_status vc_verify_workspace_bytes(const vc_full_kv* kv, int32_t total_win, size_t* bytes);
vc_status vc_verify_attn(vc_ctx* ctx, const vc_full_kv* kv, const void* q_win, const void* k_win,
                         const void* v_win, const int32_t* cu_win, int32_t total_win,
                         float softmax_scale, void* out, float* lse, void* workspace,
                         size_t workspace_bytes, void* stream);

/* Chunk-streamed verify (paper section 5.2 step (i) and the HBM ring of section 5.1: the reload is
 * in flight while the GPU works).  The key stream of sequence b is its full-KV tokens followed by
 * its window tokens.  vc_verify_attn_range attends, for sequences seq_begin .. seq_end-1, to stream
 * positions [tok_begin, tok_end) and leaves split partials in `workspace`; it can be issued as soon
 * as the swap-in ticket of those tokens has been waited for on `stream`.  tok_begin must be a
 * multiple of the chunk length that vc_verify_plan reports, tok_end a multiple of it or past the end
 * of every sequence (the window tokens belong to the last range).  vc_verify_finish merges the
 * partials once every position of every sequence has been covered exactly once; the same workspace
 * (sized by vc_verify_workspace_bytes) must be passed to all calls.  vc_verify_attn is the two calls
 * back to back over the whole stream. */
vc_status vc_verify_plan(const vc_full_kv* kv, int32_t* chunk_tokens, int32_t* n_chunks);
vc_status vc_verify_attn_range(vc_ctx* ctx, const vc_full_kv* kv, const void* q_win, const void* k_win,
                               const void* v_win, const int32_t* cu_win, int32_t total_win,
                               float softmax_scale, int32_t seq_begin, int32_t seq_end,
                               int32_t tok_begin, int32_t tok_end, void* workspace,
                               size_t workspace_bytes, void* stream);
vc_status vc_verify_finish(vc_ctx* ctx, const vc_full_kv* kv, const int32_t* cu_win, int32_t total_win,
                           void* out, float* lse, void* workspace, size_t workspace_bytes,
                           void* stream);

/* Greedy acceptance (paper section 4.1 step 3).
 *   logits      device fp32 [total_rows, vocab]; sequence b owns rows cu_rows[b]..cu_rows[b+1]-1:
 *               w_b rows (row j = full-KV prediction for drafted position j), or w_b + 1 when the
 *               bonus row is supplied.  Values are finite or -inf.
 *   draft_ids   device int32 [sum w], sequence b owns cu_win[b]..cu_win[b+1]-1
 *   argmax_ids  device int32 [total_rows] (required, written): arg-max of each row, the lowest
 *               index wins a tie
 *   accept_len  device int32 [n_seqs]: first j with draft_ids[j] != argmax(row j), else w_b
 *   next_token  device int32 [n_seqs]: argmax(row accept_len) - the correction, or the bonus
 *               token when everything matched and the bonus row exists; -1 if that row is absent
 * A short scan (up to 2048 segments of 8192 logits, up to 128 sequences) is one launch whose last workgroup finishes the batch; it counts on one
 * of 16 sets of counters the context owns (call i uses set i mod 16), so at most 16 calls made through
 * one context may be in flight, or captured in graphs that run, at the same time. */
vc_status vc_accept_workspace_bytes(int32_t total_rows, int32_t vocab, size_t* bytes);
vc_status vc_accept_len(vc_ctx* ctx, const float* logits, int32_t vocab, const int32_t* cu_rows,
                        int32_t total_rows, const int32_t* draft_ids, const int32_t* cu_win,
                        int32_t n_seqs, int32_t* accept_len, int32_t* next_token,
                        int32_t* argmax_ids, void* workspace, size_t workspace_bytes,
                        void* stream);

/* Sampling-based acceptance (the footnote of paper section 4.1 says that the method carries over to
 * sampled decoding through the usual rejection-sampling rule and gives no further text, so this is
 * the textbook speculative-sampling rule, with every random number an input).
 *   p_j = softmax(target row j / T)   full-KV distribution for drafted position j
 *   q_j = softmax(draft row j / T)    the distribution drafted token t_j was sampled from
 *   position j is accepted iff u_accept[j] * q_j(t_j) < p_j(t_j); accept_len = first rejected
 *   position, else w_b.  next_token: at a rejection, drawn from max(0, p_a - q_a) by inverse CDF
 *   (the smallest v whose running sum over v' <= v exceeds u_resample[b] * total); when everything
 *   was accepted, drawn the same way from p_w if the bonus row is supplied, else -1.
 * Probabilities are evaluated in double precision (row maximum, sum of exponentials, running
 * sums), so the integers equal a plain double-precision evaluation unless a draw lies within
 * rounding distance of a boundary.
 *   target_logits  device fp32 [total_rows, vocab]; rows per sequence as for vc_accept_len
 *   draft_logits   device fp32 [total_win, vocab]; row cu_win[b] + j belongs to drafted position j
 *   draft_ids      device int32 [total_win], in [0, vocab)
 *   u_accept       device fp32 [total_win], u_resample device fp32 [n_seqs]; values in [0, 1)
 *   temperature    T > 0
 *   accept_len, next_token   device int32 [n_seqs] */
vc_status vc_accept_sample_workspace_bytes(int32_t total_rows, int32_t total_win, int32_t n_seqs, int32_t vocab,
                                           size_t* bytes);
vc_status vc_accept_sample(vc_ctx* ctx, const float* target_logits, const float* draft_logits, int32_t vocab,
                           const int32_t* cu_rows, int32_t total_rows, const int32_t* draft_ids,
                           const int32_t* cu_win, int32_t total_win, int32_t n_seqs, float temperature,
                           const float* u_accept, const float* u_resample, int32_t* accept_len,
                           int32_t* next_token, void* workspace, size_t workspace_bytes, void* stream);

/* Full-KV reload (paper section 4.2.1 and section 5.2 step (i): the full KV lives in CPU memory
 * and is reloaded asynchronously, overlapped with draft forward passes).
 * One hipMemcpyAsync and one event per chunk, on the context's own copy stream.
 *   host_src  pinned host memory (hipHostMalloc); pageable memory is rejected
 *   dev_dst   device memory
 *   chunks    host array of n_chunks {src_off, dst_off, bytes} (byte offsets from the bases)
 *   first_ticket  receives the ticket of chunks[0]; chunk i has ticket first_ticket + i.
 * Tickets complete in issue order.  At most 4096 tickets may be outstanding (issued and
 * not yet landed); a call that would exceed that returns VC_ERR_INVALID_ARG and enqueues nothing. */
typedef struct { size_t src_off, dst_off, bytes; } vc_chunk;
vc_status vc_swap_in(vc_ctx* ctx, const void* host_src, void* dev_dst, const vc_chunk* chunks,
                     int32_t n_chunks, int64_t* first_ticket);
/* Make `stream` wait (on the device, the host does not block) until `ticket` has landed. */
vc_status vc_swap_wait(vc_ctx* ctx, int64_t ticket, void* stream);
/* Ordering in the other direction (section 5.2 step (i): a request's staging memory is reloaded only
 * after its previous verify has read it; section 5.1: a ring slot is reused once consumed).
 * vc_mark records a point on `stream` - everything enqueued on it so far - and returns its number.
 * vc_swap_after makes the copy stream wait, on the device, for that point: chunks issued by later
 * vc_swap_in / vc_swap_in_rows calls start only after the marked work has finished.  The host never
 * blocks, except that vc_mark waits for the mark issued 1024 marks earlier if that one is still
 * pending (its slot is being reused). */
vc_status vc_mark(vc_ctx* ctx, void* stream, int64_t* mark);
vc_status vc_swap_after(vc_ctx* ctx, int64_t mark);
/* VC_OK once `ticket` has landed, VC_ERR_NOT_READY before. */
vc_status vc_swap_query(vc_ctx* ctx, int64_t ticket);
/* Block the host until every issued chunk has landed. */
vc_status vc_swap_sync(vc_ctx* ctx);

/* Reload of the dropped rows only (paper appendix B.1, the transfer term of the per-iteration
 * time: with token dropping a verify needs only the extra (1 - c) * KV_full, because the kept rows
 * already sit in HBM).  The host keeps the dropped rows of every (sequence, head) list PACKED:
 * packed row cu_drop[b]*n_kv_heads + h*nd_b + i is the 256-byte row (cu_ctx[b] + t, h) of the full
 * KV, t = entry i of dropped list (b, h) - vc_pack_rows builds that buffer on the device from a
 * full pool (at compression time; the caller copies it to pinned memory).
 *
 * vc_swap_in_rows, for every sequence b in [seq_begin, seq_end) in turn: copies the sequence's
 * packed rows host -> staging with the copy engine (two contiguous copies, K and V), places them
 * into rows (cu_ctx[b] + t, h) of dev_k / dev_v with a short kernel, and records one event, all
 * on the context's copy stream; sequence b gets ticket first_ticket + (b - seq_begin) for
 * vc_swap_wait / vc_swap_query.  Rows of the destination that no list names are left alone, so a
 * pool whose kept rows are valid becomes the full KV of those sequences.
 *   host_packed_k, host_packed_v   pinned host memory (hipHostMalloc), packed rows as above
 *   stage_k, stage_v   device staging, each at least stage_rows * 256 bytes; must hold one
 *                      sequence: stage_rows >= nd_b * n_kv_heads (else VC_ERR_INVALID_ARG).  The
 *                      in-order copy stream makes reuse across sequences and calls safe.
 *   dev_k, dev_v       device bf16 pools [sum tokens][n_kv_heads][128]
 *   dropped, cu_drop, cu_ctx   device int32, as for vc_keep_from_dropped (positions relative to
 *                      the sequence start, in range: the caller's contract)
 *   cu_drop_host       host copy of cu_drop (the copy sizes are needed on the host)
 *
 * vc_pack_rows: pool rows named by index lists (any lists in the dropped / kept list layout)
 * -> packed rows, on `stream`; max_idx = host-side max list length. */
vc_status vc_pack_rows(vc_ctx* ctx, const void* k, const void* v, const int32_t* idx, const int32_t* cu_idx,
                       const int32_t* cu_ctx, int32_t n_seqs, int32_t n_kv_heads, int32_t max_idx,
                       void* packed_k, void* packed_v, void* stream);
vc_status vc_swap_in_rows(vc_ctx* ctx, const void* host_packed_k, const void* host_packed_v, void* stage_k,
                          void* stage_v, int64_t stage_rows, void* dev_k, void* dev_v, const int32_t* dropped,
                          const int32_t* cu_drop, const int32_t* cu_drop_host, const int32_t* cu_ctx,
                          int32_t n_kv_heads, int32_t seq_begin, int32_t seq_end, int64_t* first_ticket);

/* Kept-index lists from the compressor's dropped-index lists (section 6,
 * CompressedKV.dropped_indices): keep = [0, len_b) minus dropped, ascending.
 *   dropped  device int32, 16-byte aligned, cu_drop[n_seqs]*n_kv_heads entries: list (b, h) is
 *            dropped[(cu_drop[b]*n_kv_heads + h*nd) + i], ascending, i < nd = cu_drop[b+1]-cu_drop[b]
 *   cu_ctx   device int32 [n_seqs+1]: len_b = cu_ctx[b+1]-cu_ctx[b];  max_ctx host
 *   keep_idx device int32, written in the layout vc_comp_kv.keep_idx describes
 *   cu_keep  device int32 [n_seqs+1], written: prefix sums of len_b - nd */
vc_status vc_keep_from_dropped(vc_ctx* ctx, const int32_t* dropped, const int32_t* cu_drop,
                               const int32_t* cu_ctx, int32_t n_seqs, int32_t n_kv_heads,
                               int32_t max_ctx, int32_t* keep_idx, int32_t* cu_keep, void* stream);

/* ------------------------------------------------------------------------------------------
 * Compressor side (paper section 6, Compressor interface: compress / decompress for the
 * quantisation methods; section 2: keys quantised per channel, values per token).
 *
 * vc_compress_quant writes, for every sequence b and KV head h, the block records of the first
 * nb_b * TB tokens of the sequence (nb_b = cu_blk[b+1] - cu_blk[b]; TB = 32 tokens for bits 4,
 * 64 for bits 2) in the record layout and list order vc_comp_kv.blocks describes.  The caller
 * chooses nb_b <= len_b / TB; tokens beyond nb_b * TB stay bf16 (they are what vc_comp_kv's tail
 * is for).  Quantiser, every step one IEEE float32 operation, metadata rounded to fp16 (nearest
 * even), codes computed from the STORED metadata:
 *     zero = fp16(min + 0)         scale = fp16((max - min) / (2^bits - 1))
 *     code = clamp(rne((x - zero) * (1 / scale)), 0, 2^bits - 1)        (scale 0: code 0)
 * Key groups: one channel over the TB tokens of a record; value groups: one token over TB
 * consecutive channels.  A group whose range exceeds fp16 gives an infinite scale (undefined).
 *   k, v      device bf16 [sum tokens][n_kv_heads][128], 16-byte aligned (the layout of pool_k)
 *   cu_ctx    device int32 [n_seqs+1] token offsets of the sequences in k, v
 *   cu_blk    device int32 [n_seqs+1] record offsets (per head) of the sequences
 *   max_blk   host-side max of nb_b
 *   blocks    device, written: n_kv_heads * cu_blk[n_seqs] records of 5120 bytes
 *
 * vc_decompress_quant is the inverse (the remote-prefix decompress that materialises bf16 KV at
 * the drafter): token t < nb_b * TB of sequence b gets x_hat = scale * code + zero, evaluated
 * as one float32 fused multiply-add and rounded to bf16 (nearest even), written to row
 * cu_ctx[b] + t of k_out / v_out (same layout as k, v above).  Rows beyond nb_b * TB are not
 * touched.  Both calls enqueue on `stream` and need no workspace. */
vc_status vc_compress_quant(vc_ctx* ctx, const void* k, const void* v, const int32_t* cu_ctx,
                            const int32_t* cu_blk, int32_t n_seqs, int32_t n_kv_heads, int32_t bits,
                            int32_t max_blk, void* blocks, void* stream);
vc_status vc_decompress_quant(vc_ctx* ctx, const void* blocks, const int32_t* cu_blk,
                              const int32_t* cu_ctx, int32_t n_seqs, int32_t n_kv_heads, int32_t bits,
                              int32_t max_blk, void* k_out, void* v_out, void* stream);

/* Kept positions from importance scores (paper section 6: what a token-dropping compressor's
 * update() decides per request and head; scope (i): every head of a layer keeps the same number
 * of positions).  The budget cu_keep[b+1] - cu_keep[b] must not exceed len_b (the caller's contract,
 * checked by vc_validate_comp_kv on the resulting descriptor: with a larger budget only len_b entries
 * of each list are written, at the list stride of the budget, and the rest are left as they were).
 * List (b, h) keeps nk_b = min(cu_keep[b+1] - cu_keep[b], len_b) positions: the
 * first F_b = min(forced_first[b], nk_b), the last L_b = min(forced_last[b], nk_b - F_b), and the
 * nk_b - F_b - L_b highest-scoring of the others; equal scores go to the lower position (-0 equals
 * +0; NaN scores are a contract violation).  Output ascending, in the layout of
 * vc_comp_kv.keep_idx.
 *   scores        device float32: list (b, h) starts at cu_ctx[b] * n_kv_heads + h * len_b
 *   cu_ctx        device int32 [n_seqs+1]
 *   cu_keep       device int32 [n_seqs+1], read (the caller fixes the budget per sequence)
 *   forced_first, forced_last   device int32 [n_seqs], or NULL for 0
 *   keep_idx      device int32, written */
vc_status vc_topk_keep(vc_ctx* ctx, const float* scores, const int32_t* cu_ctx, const int32_t* cu_keep,
                       const int32_t* forced_first, const int32_t* forced_last, int32_t n_seqs,
                       int32_t n_kv_heads, int32_t* keep_idx, void* stream);

/* ------------------------------------------------------------------------------------------
 * Admission control (paper section 5; host code only, no GPU call, no stream).
 *
 * The runtime looks W iterations ("windows") ahead; window 0 is the current iteration.  Two
 * reserve rings (section 5.1): T[i], the interconnect time booked in window i (constraint
 * T[i] <= T_iter), and B[i], the bytes of full KV in flight in window i (constraint
 * M + KV_resident + B[i] <= HBM).  A reload of KV_full bytes takes KV_full / BW seconds and spans
 * S_r = max(1, ceil(KV_full / (BW * T_iter))) windows; it books an equal share of its time in
 * each of them and its bytes in all of them.  All quantities are doubles (seconds, bytes,
 * bytes per second).
 *
 * vc_iter_time_model: section 4.2.1, Eq. 3.  T_gpu = (M + B*KV_full*(c + 1/x)) / BW_hbm,
 *   T_xfer = B*KV_full / (x * BW_inter), T_iter = max of the two.  t_gpu / t_xfer may be NULL.
 * vc_sched_create: W windows, all empty, at iteration 0.  The caller owns the handle.
 * vc_sched_set_resident: KV_resident changes as requests come and go.
 * vc_sched_span: S_r for a request of that size.
 * vc_sched_admit (Algorithm 1): places the next verify of request `req`, which drafts x tokens
 *   per horizon.  Candidates are tried in the order anchor, anchor-1, anchor+1, anchor-2, ...,
 *   anchor = clamp(x, S_r, W-1), skipping those outside [S_r, W-1]; the first window d whose
 *   span [d-S_r+1, d] satisfies both constraints is reserved and returned in *window.  *window
 *   = -1 when none does (the request goes back to the caller's waiting queue; nothing is
 *   reserved).  A request that already holds a reservation is VC_ERR_INVALID_ARG.
 * vc_sched_cancel: gives a reservation back (a request that finished or was aborted).
 * vc_sched_step (section 5.2): one iteration.  Writes the ids (ascending) of the requests whose
 *   reload must start now (the first window of their span is the current one) to kick[0..*n_kick)
 *   and of the requests that verify now to verify[0..*n_verify); verified requests lose their
 *   reservation (the caller admits them again); then the horizon slides by one window.  If
 *   either list would exceed `capacity` entries the call fails and changes nothing.
 * vc_sched_rings: copies T[0..W) and B[0..W) (window 0 first; either may be NULL) and the
 *   absolute iteration number of window 0.
 * ------------------------------------------------------------------------------------------ */
typedef struct vc_sched vc_sched;
vc_status vc_iter_time_model(double model_bytes, double batch, double kv_full_bytes, double c, double x,
                             double bw_hbm, double bw_inter, double* t_iter, double* t_gpu, double* t_xfer);
vc_status vc_sched_create(int32_t windows, double t_iter_s, double bw_bytes_per_s, double hbm_bytes,
                          double model_bytes, double resident_bytes, vc_sched** out);
vc_status vc_sched_destroy(vc_sched* sched);
vc_status vc_sched_set_resident(vc_sched* sched, double resident_bytes);
vc_status vc_sched_span(const vc_sched* sched, double kv_full_bytes, int32_t* span);
vc_status vc_sched_admit(vc_sched* sched, int64_t req, double kv_full_bytes, int32_t x, int32_t* window);
vc_status vc_sched_cancel(vc_sched* sched, int64_t req);
vc_status vc_sched_step(vc_sched* sched, int64_t* kick, int32_t* n_kick, int64_t* verify, int32_t* n_verify,
                        int32_t capacity);
vc_status vc_sched_rings(const vc_sched* sched, double* t_ring, double* b_ring, int64_t* now);

#ifdef __cplusplus
}
#endif
#endif /* VERICACHE_H */
