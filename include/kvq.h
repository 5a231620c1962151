/*
 * kvq - low-bit KV-cache decode attention with outlier-token tracing, for gfx950.
 *
 * C ABI of the hot path of "KV Cache Quantization with Outlier Tokens Tracing"
 * (OTT).  All pointers named "device" are HIP device pointers owned by the
 * caller; the library never allocates, frees or keeps a pointer after a call
 * returns, enqueues all work on the caller's stream and never synchronises.
 * `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *
 * Cache shape follows the paper's [num_layers, batch_size, num_heads,
 * sequence_length, head_dim] (Introduction).  A "unit" is one (layer, batch,
 * kv head); unit index u = (layer * batch + b) * kv_heads + h.  Every buffer
 * below is a dense array whose leading dimension is the unit; the quantized
 * arrays may instead be a pool of pages shared by the sequences (kvq_qcache).
 * Sequence lengths are uniform over the batch in the calls that take them as
 * arguments; the *_ragged calls read each sequence's own state from a device
 * array, and kvq_prefill_quantize_seq fills the slot of one sequence.
 *
 * Return value of every call: 0 (KVQ_OK) or a negative kvq_status.  Arguments
 * are validated on the host before anything is launched, so an error return
 * means no device work was enqueued.  Data-dependent events (the auxiliary
 * pool filling up) are not errors: they set `frozen[u]` on the device.
 */
#ifndef KVQ_H
#define KVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum kvq_status {
  KVQ_OK = 0,
  KVQ_ERR_INVALID_ARG = -1, /* null pointer, out-of-range or inconsistent argument        */
  KVQ_ERR_UNSUPPORTED = -2, /* meaningful for the method but not built (e.g. head_dim 64) */
  KVQ_ERR_WORKSPACE = -3,   /* workspace smaller than kvq_query_sizes reports             */
  KVQ_ERR_LAUNCH = -4,      /* the HIP runtime refused a launch                           */
  KVQ_ERR_SCRATCH = -5      /* too large for the library's static scratch buffer          */
} kvq_status;

/* Hyper-parameters in the paper's notation (Experiments, "Details"): bit width b,
 * group size G, residual length R, outlier_num N, size of the additional pool A. */
typedef struct kvq_config {
  int32_t layers;
  int32_t batch;
  int32_t q_heads;        /* multiple of kv_heads; q_heads / kv_heads in {1,2,4,8}            */
  int32_t kv_heads;
  int32_t head_dim;       /* 128                                                              */
  int32_t max_seq;        /* token capacity of the quantized cache; multiple of group_k       */
  int32_t bits;           /* b: 2 or 4                                                        */
  int32_t group_k;        /* G: tokens per Key group and quantization cadence: 32, 64 or 128  */
  int32_t group_v;        /* channels per Value group: 32, 64 or 128                          */
  int32_t residual;       /* R >= 0: recent tokens kept in full precision                     */
  int32_t outlier_budget; /* N >= 0 per unit; 0 disables tracing                              */
  int32_t aux_capacity;   /* A >= 0: slots for tokens evicted from the outlier pool           */
  int32_t untraced_layers; /* the first so many layers trace no outliers: their budget is 0   */
                          /* whatever outlier_budget says (Experiments, "Details": layers 0   */
                          /* and 1 of the paper's models; 0 <= untraced_layers <= layers).    */
                          /* Buffer sizes do not depend on it                                 */
  int32_t value_per_step; /* 0: Keys and Values of a group are quantized together when the    */
                          /* ring fills, every G steps (the paper's schedule).  1: the        */
                          /* schedule the paper compares itself with (Experiments, "Details": */
                          /* Keys every G steps, Values at each step): a token's Values are   */
                          /* quantized, token-wise, when the token leaves the window of the R */
                          /* most recent tokens (kvq_quantize_value_tokens), and the group    */
                          /* steps quantize Keys only.  Needs outlier_budget == 0 and         */
                          /* residual >= 1 (KVQ_ERR_UNSUPPORTED otherwise); the *_ragged and  */
                          /* *_seq entry points do not support it.  Buffer sizes are the same */
} kvq_config;

/* Sizes (bytes unless said otherwise) of every caller-allocated buffer. */
typedef struct kvq_sizes {
  int64_t units;            /* layers * batch * kv_heads                                      */
  int64_t res_rows;         /* rows per unit of the residual ring: G * ceil((R + G) / G)      */
  int64_t pool_slots;       /* N + A: slots [0,N) outlier pool, [N,N+A) auxiliary pool        */
  int64_t k_codes_bytes;    /* [units][max_seq/32][512*bits] packed Key codes                 */
  int64_t k_meta_bytes;     /* [units][max_seq/G][2][head_dim] fp16: steps, zeros              */
  int64_t v_codes_bytes;    /* [units][max_seq/32][512*bits] packed Value codes               */
  int64_t v_meta_bytes;     /* [units][max_seq/32][128*NV bytes] fp16 steps, zeros (see below) */
  int64_t mask_bytes;       /* [units][max_seq/32] u32, bit t%32 set: token lives in a pool   */
  int64_t res_bytes;        /* each of k_res, v_res: [units][res_rows][head_dim] fp16         */
  int64_t pool_rows_bytes;  /* each of pool_k, pool_v: [units][pool_slots][head_dim] fp16     */
  int64_t pool_idx_bytes;   /* [units][pool_slots] int32 token index                          */
  int64_t pool_score_bytes; /* [units][pool_slots] fp64 L1 score                              */
  int64_t counter_bytes;    /* each of pool_count, aux_count, frozen: [units] int32           */
  int64_t selected_bytes;   /* [batch*kv_heads][G] uint8, one layer                           */
  int64_t workspace_bytes;  /* decode-attention workspace for one layer                       */
  int64_t prefill_selected_bytes; /* [batch*kv_heads][max_seq/G][G] uint8: flags of a whole prompt */
} kvq_sizes;

/*
 * Quantized cache (device).  Packed format.  Codes are stored in blocks of 32 tokens x 128
 * channels = 512*bits bytes, block i of a unit holding tokens 32i .. 32i+31.  A block is
 * 64 "lanes" of 8 "fields" of 8 codes.  Code x = 2v + e (v in 0..3, e in 0..1) of field f
 * of lane l occupies `bits` bits of a little-endian u32 word, starting at
 *     bits = 2:  bit (16e + 2(v+1) + 8(f&1)) mod 32        of the word at byte  16 l + 4 (f>>1)
 *     bits = 4:  bit (16e + 2 + 4(v&1) + 8(v>>1)) mod 32   of the word at byte  1024 (f>>2) + 16 l + 4 (f&3)
 * and continuing at bit 0 of the same word after bit 31 (the code is rotated into place; only
 * the 4-bit code x = 7 wraps).  Read as two fp16 halves, the word - or the word rotated right by
 * 8 - thus shows a field's codes at bits 2..9 of each half.
 * Key block:   token t = 16 th + m, channel c = 32 cb + 8 r + x  ->  lane 16 r + m, field 4 th + cb.
 * Value block: channel c = 16 ct + n, token t = 8 r + x          ->  lane 16 r + n, field ct.
 * (A lane's 16 bytes are what one wavefront lane loads with one dwordx4; a field is one
 * lane's share of a 16x16x32 matrix-core operand.)
 * Steps and zeros are fp16; the dequantized value is zero + code * step.
 *   k_meta[u][group]  (512 bytes): step[128 channels], then zero[128 channels].
 *   v_meta[u][block]  (128*NV bytes, NV = head_dim / group_v): step[16 token pairs][NV][2], i.e.
 *                     the step of token 2p+e and value group j at index (p*NV + j)*2 + e; then
 *                     zero[16 token pairs][NV][2], indexed the same way.
 * mask[u][block] bit t%32 is set when token
 * 32*block + t was selected as an outlier (it then lives in the outlier or auxiliary pool and
 * its codes are placeholders).
 *
 * Paged cache (page_table != NULL; what a serving stack needs, the paper uses fixed lengths): the
 * five arrays are a pool of pages shared by the sequences.  A page holds one Key group (group_k
 * tokens) of one sequence, for every layer and kv head: the arrays are laid out as above with the
 * "unit" replaced by the plane p = layer * kv_heads + h and max_seq by n_pages * group_k, i.e. they
 * have the sizes kvq_query_sizes gives for the same configuration with batch = 1 and
 * max_seq = n_pages * group_k.  Key group j (tokens j*group_k ...) of sequence b is stored as group
 * page_table[b * table_stride + j] of its planes.  The table is device memory, int32, read by the
 * kernels when they run; table_stride >= max_seq / group_k, 0 < n_pages <= 2^20 and
 * n_pages * (group_k / 32) * 512 * bits < 2^32 (the codes of one plane stay below 4 GiB: the kernels
 * address them with 32-bit offsets); otherwise KVQ_ERR_INVALID_ARG.  An entry outside
 * [0, n_pages) is clamped to that range by the kernels (results are then wrong, accesses stay inside
 * the arrays); entries of groups that no call touches are not read, with one exception: entry 0 of
 * a sequence is read even while the sequence has no quantized token.  Two sequences must not name
 * the same page.  Every entry point that takes a kvq_qcache accepts both forms; page_table == NULL
 * (n_pages and table_stride ignored) is the dense form.
 */
typedef struct kvq_qcache {
  void* k_codes;
  void* k_meta;
  void* v_codes;
  void* v_meta;
  void* mask;
  const int32_t* page_table;
  int32_t table_stride;
  int32_t n_pages;
} kvq_qcache;

/* Outlier pool and auxiliary pool (device).  Occupied slots are [0, pool_count[u]) and
 * [N, N + aux_count[u]).  Must be zero-initialised (counts and frozen) by the caller. */
typedef struct kvq_pool {
  void* pool_k;
  void* pool_v;
  int32_t* pool_idx;
  double* pool_score;
  int32_t* pool_count;
  int32_t* aux_count;
  int32_t* frozen;
} kvq_pool;

/* Full-precision residual ring (device): res_rows rows per unit; the live rows are
 * res_start, res_start+1, ... (mod res_rows), oldest first. */
typedef struct kvq_residual {
  void* k_res;
  void* v_res;
} kvq_residual;

/* Fill `out` with the buffer sizes for `cfg`.  Host only. */
int32_t kvq_query_sizes(const kvq_config* cfg, kvq_sizes* out);

/*
 * Append the new token's Key and Value (K = K_<n || K_n, V likewise: Background,
 * decoding phase) of one layer to the residual ring.
 *   k_new, v_new : device fp16 [batch][kv_heads][head_dim], 4-byte aligned (as must be the ring)
 *   res_start    : ring row of the oldest live token, in [0, res_rows)
 *   n_res        : live rows before the append, in [0, res_rows)
 * Writes ring row (res_start + n_res) mod res_rows of every unit of `layer`.
 */
int32_t kvq_append_residual(const kvq_config* cfg, int32_t layer, const void* k_new, const void* v_new,
                            kvq_residual res, int32_t res_start, int32_t n_res, void* stream);

/*
 * Outlier-token competition for one group of G tokens of one layer (Method,
 * "Quantization"; Appendix "Competition Mechanism"): score each token by the L1
 * norm of its Key, rank pool and group together (score, then token index,
 * ascending), keep the N smallest as the new pool, move members that fall out to
 * the auxiliary pool; if those do not fit, set frozen[u] and change nothing else.
 *   group_index  : index of the group in the sequence; its tokens are
 *                  group_index*G .. group_index*G + G - 1; must be < max_seq / G
 *   k_group, v_group : device fp16; unit (b,h) of this layer has its G rows of head_dim
 *                  contiguous at element offset (b*kv_heads + h) * unit_stride
 *   unit_stride  : in fp16 elements, >= G * head_dim, multiple of 8; k_group and v_group
 *                  16-byte aligned
 *   pool         : updated in place (rows are bit-exact copies of the group's rows)
 *   selected     : device uint8 [batch*kv_heads][G], out: 1 = token entered the pool now
 */
int32_t kvq_trace_outliers(const kvq_config* cfg, int32_t layer, int32_t group_index, const void* k_group,
                           const void* v_group, int64_t unit_stride, kvq_pool pool, uint8_t* selected,
                           void* stream);

/*
 * Quantize one group of G tokens of one layer and store it as group `group_index`
 * of the quantized cache: rows flagged in `selected` are first replaced by the
 * per-channel mean of the group (Method, "Quantization"), then Keys are quantized
 * channel-wise over the G tokens and Values token-wise over group_v channels with
 * Eq. 2 (step = (max - min) / (2^b - 1) stored in fp16, zero = min, round to
 * nearest), packed, and the mask words of the group are written.
 *   k_group, v_group, unit_stride : as in kvq_trace_outliers (read only)
 *   selected     : device uint8 [batch*kv_heads][G] or NULL (= none selected)
 */
int32_t kvq_quantize_group(const kvq_config* cfg, int32_t layer, int32_t group_index, const void* k_group,
                           const void* v_group, int64_t unit_stride, const uint8_t* selected,
                           kvq_qcache qcache, void* stream);

/*
 * Per-step Value quantization (cfg->value_per_step == 1; the schedule of the paper's comparison,
 * Experiments, "Details": "compressing the Values at each step").  Tokens first_token ..
 * first_token + count - 1 of every sequence, which live in ring rows ring_row, ring_row + 1, ...
 * (mod res_rows) of the Value ring, are quantized token-wise with Eq. 2 (one step and zero per
 * group_v channels of the token, exactly what kvq_quantize_group computes for the same row): their
 * codes, steps and zeros are stored at their places in v_codes / v_meta (other tokens' bits of the
 * same words are kept), and each ring row is overwritten with its dequantized row, zero + code * step
 * evaluated in fp32 and rounded to fp16.  From then on the decode calls, which read those tokens from
 * the ring until their Key group is quantized, attend them with their quantized Values.  A decode
 * step under this schedule: this call for the one token that leaves the window (token n - R - 1 with
 * n tokens in the cache after the append, once n > R), then the step's other calls as usual;
 * kvq_quantize_group, kvq_append_trace_quantize and kvq_prefill_quantize's group pass then leave the
 * Value arrays alone, and kvq_prefill_quantize ends with this call for the tokens between the last
 * whole group and the window.
 *   first_token, count : 0 <= first_token, 1 <= count <= res_rows, first_token + count <= max_seq (under
 *                        this schedule max_seq must cover n - R tokens: Values run up to group_k - 1
 *                        tokens ahead of the Keys)
 *   ring_row           : in [0, res_rows)
 *   v_res              : device fp16 ring of the Values (read and written), 4-byte aligned
 *   qcache             : dense or paged (the pages of the tokens' groups must be in the table)
 * Tokens of one call are processed in order by one workgroup per unit; two calls that touch tokens
 * of the same 32-token block must not overlap in time.
 */
int32_t kvq_quantize_value_tokens(const kvq_config* cfg, int32_t layer, int32_t first_token, int32_t count,
                                  void* v_res, int32_t ring_row, kvq_qcache qcache, void* stream);

/*
 * Decode-step attention of one layer (Eq. 1) over the three cache kinds (Method,
 * "Decoding"): the first n_quant tokens from the quantized cache, except those
 * whose mask bit is set, which come from the outlier / auxiliary pool in full
 * precision; then the n_res residual tokens in full precision.  One softmax over
 * all of them, scale 1/sqrt(head_dim).  Query head j reads kv head j / (q_heads /
 * kv_heads).
 *   q        : device fp16 [batch][q_heads][head_dim], 16-byte aligned (as must be the code arrays,
 *              the residual ring and the pool rows; steps/zeros and mask words 4-byte aligned)
 *   n_quant  : multiple of G, <= max_seq
 *   res_start, n_res : live part of the residual ring, n_res <= res_rows; res_start a multiple of 16
 *              (it is a multiple of group_k under the schedule of kvq_append_trace_quantize): the
 *              residual rows are read 16 at a time, and such a run must not wrap; n_quant + n_res >= 1
 *   qcache   : all five arrays must be valid device memory of the sizes kvq_query_sizes gives, also
 *              when n_quant == 0: every workgroup loads a first block whether or not it has quantized
 *              tokens to work on.  Likewise pool.pool_k / pool_v whenever outlier_budget +
 *              aux_capacity > 0 (every slot is loaded, filled or not, 16 slots at a time: up to 15 rows
 *              past a unit's last slot are read, never used; kvq_sizes.pool_rows_bytes includes those
 *              15 rows behind the last unit) and pool_count, aux_count
 *   Range    : the products run on fp16 operands with fp32 accumulation.  Results are finite and within
 *              2e-3 (absolute, for outputs of order 1) of the exact attention over the dequantized
 *              cache while |q_c| * step_c < 32 000 for every channel c and Key group
 *              (step = the group's quantization step of that channel) and every Value step < 4000;
 *              beyond that an operand overflows fp16 and outputs become infinite or NaN
 *   out      : device fp16 [batch][q_heads][head_dim]
 *   workspace: device scratch of at least kvq_sizes.workspace_bytes, 256-byte aligned.  It must
 *              be zero-filled once before its first use; every call leaves the part it relies on
 *              (per-unit arrival counters) zero again, so it can be reused call after call.  Two
 *              calls that overlap in time must not share it
 */
int32_t kvq_decode_attention(const kvq_config* cfg, int32_t layer, const void* q, kvq_qcache qcache,
                             int32_t n_quant, kvq_residual res, int32_t res_start, int32_t n_res,
                             kvq_pool pool, void* out, void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * The same attention for several consecutive query tokens at once (verification of drafted tokens,
 * a short continuation of the prompt; the paper decodes one token per step): the q_tokens newest
 * tokens of every sequence, whose Keys and Values are already in the cache.  Token i of them (0 = the
 * oldest) attends to every token up to and including itself, i.e. to everything but the q_tokens - 1 - i
 * newest residual rows.  The cache is read once for all of them.
 *   q, out    : device fp16 [batch][q_tokens][q_heads][head_dim]
 *   q_tokens  : q_tokens * (q_heads / kv_heads) must be 1, 2, 4 or 8 (KVQ_ERR_UNSUPPORTED otherwise);
 *               n_res >= q_tokens - 1 (the tokens to hide must be residual rows)
 *   workspace : at least kvq_decode_workspace_bytes(cfg, q_tokens) (host only; a negative kvq_status
 *               for a configuration or token count that is not supported); for q_tokens = 1 that is
 *               kvq_sizes.workspace_bytes
 * Everything else as kvq_decode_attention, which is the case q_tokens = 1.
 */
int64_t kvq_decode_workspace_bytes(const kvq_config* cfg, int32_t q_tokens);
int32_t kvq_decode_attention_multi(const kvq_config* cfg, int32_t layer, const void* q, int32_t q_tokens,
                                   kvq_qcache qcache, int32_t n_quant, kvq_residual res, int32_t res_start,
                                   int32_t n_res, kvq_pool pool, void* out, void* workspace,
                                   size_t workspace_bytes, void* stream);

/*
 * kvq_decode_attention for callers that cannot allocate or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  The launch's workspace (arrival
 * counters and partial results of units that are split over several workgroups) is a 4 MiB array
 * inside the library, one per device, held from its first use until the process ends.  The call
 * allocates nothing and frees nothing; its first call on a device looks up the array's address once.
 *   arguments : as kvq_decode_attention, without workspace and workspace_bytes; `stream` must be a
 *               stream of the current device
 *   limit     : kvq_decode_workspace_bytes(cfg, 1) <= 4 MiB (4 194 304), else KVQ_ERR_SCRATCH and
 *               nothing is launched
 * The result equals kvq_decode_attention's bit for bit.  All calls on one device share the array:
 * calls that overlap in time on one device (different streams, different threads) race on it; calls
 * on one stream, or otherwise ordered, do not.  What must start at zero (the counters) is cleared by
 * the call itself, with a small fill kernel ahead of the decode launch when a unit is split.
 */
int32_t kvq_decode_attention_static(const kvq_config* cfg, int32_t layer, const void* q, kvq_qcache qcache,
                                    int32_t n_quant, kvq_residual res, int32_t res_start, int32_t n_res,
                                    kvq_pool pool, void* out, void* stream);

/*
 * How kvq_decode_attention (and its variants) would split a launch, host only: the quantized tokens
 * of a unit go to the wavefronts of `splits` workgroups of `waves` wavefronts each in mini-chunks of
 * 128 tokens, `minichunks_per_split` per workgroup; with splits > 1 the workgroups of a unit exchange
 * partial results (m, l, o) through the workspace and the last one to arrive merges them (the
 * chunk-wise form of Eq. 1's softmax: the result does not depend on the split).  For tests and
 * benchmarks that must know which launch shape they exercise; the kernels need no such call.
 *   q_tokens : as in kvq_decode_attention_multi (1 for a plain decode step)
 *   n_quant  : quantized tokens (multiple of group_k, <= max_seq)
 *   fp_rows  : full-precision rows the launch reads per unit: n_res (+ 1 with k_new) + outlier_budget
 *              + aux_capacity
 * Returns KVQ_OK or the status kvq_decode_attention would return for the same cfg / q_tokens / n_quant.
 */
int32_t kvq_decode_launch_shape(const kvq_config* cfg, int32_t q_tokens, int32_t n_quant, int32_t fp_rows,
                                int32_t* splits, int32_t* waves, int32_t* minichunks_per_split);

/*
 * Quantize a whole prompt of one layer in one call (Method, "Quantization", prefill phase: the
 * prompt's Keys and Values are quantized group by group, the last tokens stay in full precision).
 * The result is the state that appending the n_tokens tokens one by one would leave: groups
 * 0 .. n_q/G - 1 of the quantized cache with n_q = G * floor((n_tokens - R) / G) (0 if n_tokens <
 * R + G), pool and auxiliary pool after the n_q/G competitions in order, and the last
 * n_tokens - n_q rows in ring rows 0 .. (the caller continues with res_start = 0, n_res =
 * n_tokens - n_q).  The layer's cache must be empty before the call (counts and frozen zero).
 *   k_rows, v_rows : device fp16, unit (b, h)'s n_tokens rows of head_dim contiguous at element
 *                    offset (b*kv_heads + h) * unit_stride; 16-byte aligned
 *   unit_stride    : in fp16 elements, >= n_tokens * head_dim, multiple of 8
 *   n_tokens       : 1 .. max_seq + R + G - 1, with n_q <= max_seq
 *   selected       : device uint8 scratch of kvq_sizes.prefill_selected_bytes; on return
 *                    selected[(unit * (n_q/G) + group) * G + t] = 1 if token t of that group entered
 *                    the pool at its competition
 * The competitions of a unit run in order in one wavefront, on scores that the other wavefronts of its
 * workgroup compute a stretch of tokens ahead; the groups are then quantized in parallel over units and
 * groups.
 */
int32_t kvq_prefill_quantize(const kvq_config* cfg, int32_t layer, const void* k_rows, const void* v_rows,
                             int64_t unit_stride, int32_t n_tokens, kvq_pool pool, uint8_t* selected,
                             kvq_qcache qcache, kvq_residual res, void* stream);

/*
 * The same for ONE sequence of the batch, for a serving loop in which sequences join a running batch
 * (the paper's experiments use batches of equal length): the prompt of sequence `seq` (0 .. batch-1) is
 * quantized into that sequence's units of `layer`, whatever they held before - its pools are emptied
 * first, its ring rows and, for a paged cache, the pages its table row names are overwritten.  Other
 * sequences are not touched.
 *   k_rows, v_rows : device fp16, kv head h's n_tokens rows at element offset h * unit_stride
 *   selected       : device uint8 scratch, at least kv_heads * n_q bytes
 * Everything else as kvq_prefill_quantize.  With per-sequence state (kvq_decode_attention_ragged) the
 * caller then writes {n_q, 0, n_tokens - n_q, active} into the sequence's entry of that array.
 */
int32_t kvq_prefill_quantize_seq(const kvq_config* cfg, int32_t layer, int32_t seq, const void* k_rows,
                                 const void* v_rows, int64_t unit_stride, int32_t n_tokens, kvq_pool pool,
                                 uint8_t* selected, kvq_qcache qcache, kvq_residual res, void* stream);

/*
 * The whole group step in one launch, for the decode steps on which the ring fills: append the
 * new token's Key and Value as kvq_append_residual does, then, on the oldest G rows of the ring,
 * the outlier competition of kvq_trace_outliers and the quantization of kvq_quantize_group
 * (Method, "Quantization": every G steps the oldest group is traced and quantized).  Results are
 * those of the three calls in sequence.
 *   res_start, n_res : as in kvq_append_residual (state before the append); the ring must be
 *                      full after the append: n_res + 1 == residual + group_k, and res_start must
 *                      be a multiple of group_k (the oldest group is one contiguous block)
 *   n_quant          : tokens already quantized, a multiple of group_k, n_quant + group_k <= max_seq;
 *                      the group is stored as group n_quant / group_k
 *   selected         : device uint8 [batch*kv_heads][G], out, or NULL if the flags are not wanted
 * Errors: as the three calls; KVQ_ERR_INVALID_ARG if the ring is not full after the append.
 */
int32_t kvq_append_trace_quantize(const kvq_config* cfg, int32_t layer, const void* k_new, const void* v_new,
                                  kvq_residual res, int32_t res_start, int32_t n_res, int32_t n_quant,
                                  kvq_pool pool, uint8_t* selected, kvq_qcache qcache, void* stream);

/*
 * A decode step on which the ring does not fill, in one launch: the attention of
 * kvq_decode_attention over the cache as it is plus the token being decoded (Background, decoding
 * phase: K = K_<n || K_n), whose rows come with the call and are also stored in the ring, as
 * kvq_append_residual would have stored them before.  Result and ring contents equal those of
 * kvq_append_residual followed by kvq_decode_attention with n_res + 1.
 *   k_new, v_new     : device fp16 [batch][kv_heads][head_dim], 4-byte aligned
 *   res_start, n_res : the ring's state BEFORE the token; n_res + 1 < residual + group_k (on the
 *                      step that fills the ring call kvq_append_trace_quantize, then
 *                      kvq_decode_attention).  The caller counts the token: n_res + 1 afterwards
 *   other arguments, workspace and errors as kvq_decode_attention.
 */
int32_t kvq_append_decode_attention(const kvq_config* cfg, int32_t layer, const void* q, const void* k_new,
                                    const void* v_new, kvq_qcache qcache, int32_t n_quant, kvq_residual res,
                                    int32_t res_start, int32_t n_res, kvq_pool pool, void* out,
                                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same step for callers that hand over the query and the new Key BEFORE their rotary position
 * embedding: the launch rotates both, then does what kvq_append_decode_attention does with the
 * rotated rows (the rotated Key row is what the ring receives; Values are not rotated).  Not part of
 * the paper's method: it is the step its models (LLaMA-2/3, Mistral) apply ahead of the cache
 * (Su et al., "RoFormer", Eq. 34), fused here so that a decode step stays one launch.
 * Channel i < head_dim/2 is paired with channel i + head_dim/2:
 *     y_i = x_i cos_i - x_{i+hd/2} sin_i        y_{i+hd/2} = x_{i+hd/2} cos_i + x_i sin_i
 * each product and the sum rounded to fp32 on its own, the result to fp16 (nearest-even).
 *   q, k_new         : as kvq_append_decode_attention, unrotated; neither buffer is written
 *   rope             : device fp32, 16-byte aligned: for the new token's position the head_dim/2
 *                      cosines, then the head_dim/2 sines (frequencies, base and scaling are the
 *                      caller's).  Sequence b reads the head_dim floats at rope + b * rope_stride
 *   rope_stride      : elements (floats) between the rows of consecutive sequences: 0 (every
 *                      sequence is at the same position and shares one row) or a multiple of 4
 *                      that is >= head_dim
 *   other arguments, workspace and errors as kvq_append_decode_attention.
 */
int32_t kvq_append_decode_attention_rope(const kvq_config* cfg, int32_t layer, const void* q, const void* k_new,
                                         const void* v_new, const float* rope, int64_t rope_stride,
                                         kvq_qcache qcache, int32_t n_quant, kvq_residual res, int32_t res_start,
                                         int32_t n_res, kvq_pool pool, void* out, void* workspace,
                                         size_t workspace_bytes, void* stream);

/*
 * The rotation of kvq_append_decode_attention_rope on its own, for the steps on which the new Key
 * goes through kvq_append_trace_quantize first (the ring fills): rotate k_new and q with it, then
 * call the unrotated entry points.  Same pairing and the same arithmetic, bit for bit.
 *   x, out           : device fp16 [batch][heads][head_dim], 4-byte aligned; out may be x
 *   heads            : rows per sequence (q_heads for a query, kv_heads for Keys)
 *   rope, rope_stride: as above
 * Errors: KVQ_ERR_INVALID_ARG (NULL or misaligned pointers, heads < 1, a bad stride).
 */
int32_t kvq_rope_rotate(const kvq_config* cfg, const void* x, int32_t heads, const float* rope, int64_t rope_stride,
                        void* out, void* stream);

/*
 * Batches whose sequences differ in length (the paper's runs use one length per batch; a serving
 * loop does not).  The per-sequence state lives in device memory so that a step needs no host
 * decision:
 *   seq_state : device int32 [batch][4], 16-byte aligned: {n_quant, res_start, n_res, active} of
 *               each sequence, with the meanings and invariants of the uniform calls (n_quant a
 *               multiple of group_k; res_start a multiple of group_k below res_rows; n_res <
 *               residual + group_k between steps).  A sequence with active == 0 is skipped by
 *               kvq_append_trace_quantize_ragged and kvq_seq_advance.
 * The kernels clamp what they read to the buffers' sizes, so a corrupt array gives wrong results
 * for its sequence but no access outside the buffers.
 *
 * kvq_append_trace_quantize_ragged: one decode step's cache update of one layer, in one launch.
 * Every active sequence's new row (k_new, v_new as in kvq_append_residual) is appended to its ring;
 * the sequences whose ring is full with it (n_res + 1 == residual + group_k, and n_quant + group_k
 * <= max_seq) have their oldest group traced and quantized as in kvq_append_trace_quantize.
 * seq_state is read only: call it for every layer with the same array, then kvq_seq_advance once.
 *   selected : device uint8 [batch*kv_heads][G] or NULL; written only for sequences that quantized
 *
 * kvq_seq_advance: applies the same rule to the array itself: n_res + 1, and where the ring filled,
 * n_quant + group_k, res_start + group_k (mod res_rows), n_res - group_k.
 *
 * kvq_decode_attention_ragged: kvq_decode_attention with each sequence's own state.
 *   max_n_quant : upper bound of the sequences' n_quant, a multiple of group_k, <= max_seq
 *   max_n_res   : upper bound of the sequences' n_res, <= res_rows; max_n_quant + max_n_res >= 1
 *                 (the two bounds size the launch; a longer sequence is truncated to them).  A
 *                 sequence with no token at all gets an all-zero output row.
 *   other arguments, workspace and errors as kvq_decode_attention.
 */
int32_t kvq_append_trace_quantize_ragged(const kvq_config* cfg, int32_t layer, const void* k_new,
                                         const void* v_new, kvq_residual res, const int32_t* seq_state,
                                         kvq_pool pool, uint8_t* selected, kvq_qcache qcache, void* stream);
int32_t kvq_seq_advance(const kvq_config* cfg, int32_t* seq_state, void* stream);
int32_t kvq_decode_attention_ragged(const kvq_config* cfg, int32_t layer, const void* q, kvq_qcache qcache,
                                    kvq_residual res, const int32_t* seq_state, int32_t max_n_quant,
                                    int32_t max_n_res, kvq_pool pool, void* out, void* workspace,
                                    size_t workspace_bytes, void* stream);

/*
 * kvq_decode_attention_ragged sizes its launch by the longest sequence, so it lasts as long as that
 * sequence's units.  A launch PLAN deals the workgroups by length instead: every sequence gets a number
 * of workgroups in proportion to its tokens and full-precision rows (at least one), all of them resident
 * at once; the workgroups of a sequence share its quantized tokens equally and merge their partial
 * results (m, l, o) like the splits of kvq_decode_attention.
 *   kvq_seq_plan_bytes : host only; size of a plan for cfg, or KVQ_ERR_UNSUPPORTED when the batch has more
 *                than 1024 sequences or more sequences than workgroups fit per kv head on the device
 *   kvq_seq_plan : one small launch; writes the plan for the sequences' CURRENT state (a copy of it is
 *                part of the plan).  Call it after kvq_seq_advance, once per decode step, before the
 *                step's kvq_decode_attention_planned calls of all layers (the state is the same for all)
 *     seq_state, max_n_quant, max_n_res : as in kvq_decode_attention_ragged
 *     plan      : device int32, kvq_seq_plan_bytes(cfg) bytes, 16-byte aligned.  Word 0: entries in use;
 *                from word 8 on, 8 words per entry (= per workgroup of a kv head): {sequence, split,
 *                splits of the sequence, first mini-chunk of 128 quantized tokens, n_quant, res_start,
 *                n_res, end of the mini-chunks}
 *   kvq_decode_attention_planned : kvq_decode_attention_ragged on the state the plan holds
 *     plan      : as written by kvq_seq_plan with the same cfg and bounds.  Its entries are clamped to the
 *                bounds like seq_state's; a plan that is inconsistent (not written by kvq_seq_plan) gives
 *                wrong or missing outputs, no access outside the buffers and no hang
 *     workspace : at least kvq_sizes.workspace_bytes (which covers this launch shape too)
 *   other arguments and errors as kvq_decode_attention_ragged.
 */
int64_t kvq_seq_plan_bytes(const kvq_config* cfg);
int32_t kvq_seq_plan(const kvq_config* cfg, const int32_t* seq_state, int32_t max_n_quant, int32_t max_n_res,
                     int32_t* plan, void* stream);
int32_t kvq_decode_attention_planned(const kvq_config* cfg, int32_t layer, const void* q, kvq_qcache qcache,
                                     kvq_residual res, const int32_t* plan, int32_t max_n_quant,
                                     int32_t max_n_res, kvq_pool pool, void* out, void* workspace,
                                     size_t workspace_bytes, void* stream);

/*
 * The quantized segment as fp16 rows, for consumers that need the cache as a matrix (attention of
 * several query tokens at once, inspection): x^ = X_min + Q * q, the inverse of Eq. 2, evaluated in
 * fp32 (the product is exact there, the sum rounds once) and rounded to nearest fp16.  A token that
 * lives in the outlier or auxiliary pool comes out as its stored full-precision row (Method,
 * "Decoding").  Tokens t0 .. t0+n-1 of every unit of `layer`:
 *   n_quant      : quantized tokens of the layer (multiple of group_k, <= max_seq)
 *   t0, n        : multiples of 32, n >= 32, t0 + n <= n_quant
 *   k_out, v_out : device fp16, out; token t of unit (b,h) at element offset
 *                  (b*kv_heads + h) * out_unit_stride + (t - t0) * head_dim
 *   out_unit_stride : in fp16 elements, >= n * head_dim
 * The pools are read only.  Not on the decode path: the decode entry points never form these rows.
 */
int32_t kvq_dequantize(const kvq_config* cfg, int32_t layer, kvq_qcache qcache, int32_t n_quant, kvq_pool pool,
                       int32_t t0, int32_t n, void* k_out, void* v_out, int64_t out_unit_stride, void* stream);

/*
 * Measurement aid, not part of the method: read `bytes` bytes (a multiple of 16) of device memory
 * at `buf` (16-byte aligned) once with 16-byte loads, in one launch that fills the chip, and fold
 * them into the 4 bytes at `sink` (device).  The benchmark times it over a buffer larger than the
 * last-level cache to measure the read bandwidth a trivial kernel reaches on the device at hand.
 * Returns KVQ_ERR_INVALID_ARG for a null pointer, a misaligned buffer or a size that is zero or not
 * a multiple of 16.
 */
int32_t kvq_stream_read(const void* buf, size_t bytes, void* sink, void* stream);

/* Static string for a kvq_status value. */
const char* kvq_status_string(int32_t status);

/* Version of this interface (structure layouts and entry points), for the binding's load check: 6. */
int32_t kvq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_H */
