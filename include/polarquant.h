/*
 * polarquant.h -- C ABI of libpolarquant: polar-quantized key cache for decode
 * attention on AMD MI355X (gfx950).
 *
 * The library packs post-RoPE keys into radius/angle codes (paper Section 3.2)
 * and runs one decode step of attention against the packed cache through a
 * per-query lookup table (Section 3.3, Appendix A).  All kernels are HIP; there
 * is no CPU fallback.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates nothing, frees nothing and keeps no state between calls except
 *     the last HIP error code (thread-local, see pq_last_hip_error).
 *   - Calls enqueue work on the given HIP stream (a hipStream_t passed as
 *     void*; NULL = the default stream) and return without waiting for it.
 *   - Every entry point returns a pq_status; argument errors are found on the
 *     host before anything is launched.  Nothing throws or aborts.
 *   - Inputs must be finite; for non-finite keys or queries the output is
 *     unspecified (but no out-of-bounds access happens).  The per-group parameters
 *     are stored as fp16 (Appendix B.1), so pair radii must stay below the fp16
 *     maximum (65504) to be representable.
 *
 * Pairing.  A key (or query) of head_dim d is d/2 pairs; pair j is the two
 * elements (j, j + d/2) that rotate-half RoPE turns together (footnote 2 of
 * Section 3.1).  x = element j, y = element j + d/2.
 *
 * What is stored per pair (Section 3.2, with a uniform angle grid)
 *   radius code c = Clamp(floor((rho - z) / s), 0, 2^r - 1),  rho = sqrt(x^2 + y^2) in fp32,
 *       z = min and s = (max - min) / 2^r of rho over the tokens of the pair's
 *       group (= page), both rounded to fp16 and used as rounded; c = 0 if s == 0
 *   angle code  a = Clamp(floor((atan2(y, x) + pi) * 2^t / (2 pi)), 0, 2^t - 1);
 *       bins are half-open arcs of the uniform grid over [-pi, pi); x = y = 0 -> 2^(t-1)
 *   reconstruction rho~ = (c + 1/2) s + z,  theta~ = -pi + (a + 1/2) 2 pi / 2^t
 *
 * Packed layout (all little-endian).  A page holds group_tokens (g) tokens of
 * every KV head.  P = d/2, w = r + t.
 *   codes pool  : [page][kv_head][pair_block = P/16][token g][unit 2*w bytes]
 *                 unit = the 16 symbols of pairs 16*block .. 16*block+15 of one
 *                 token as a bit string; symbol k = (a << r) | c sits in bits
 *                 [k*w, (k+1)*w); bit i of the string = bit (i % 8) of byte (i / 8).
 *                 For r = t = 4 byte k of a unit is simply (a_k << 4) | c_k.
 *   params pool : [page][kv_head][pair P]{fp16 s, fp16 z}
 *   value pool  : [page][kv_head][token g][d] fp16        (values stay fp16, Section 4.1)
 * Slots of a sequence's last page beyond its length hold zero bytes in the
 * codes pool; their values are never read.
 *
 * Optional quantized values (Section 2's token-wise quantizer, used in Section 6.3): b = 4 or 2
 * bits per element, code = Clamp(round((v - z) / s), 0, 2^b - 1) with z = min and
 * s = (max - min) / (2^b - 1) over the d values of one token of one head (round half to even;
 * s, z stored as fp16 and used as stored); dequantized value = code * s + z.
 *   vq pool     : [page][kv_head][token block = token / T][dim slice = dim / 8][unit 16 bytes],
 *                 T = 16 / b tokens per unit.  A unit is four 32-bit words; a word holds the codes of
 *                 two consecutive tokens, the even one in its low 16 bits and the odd one in its high
 *                 16 bits, the same dims in both halves, dim after dim from bit 0 up.  b = 4: a half
 *                 holds 4 dims, word j = 2 * (token pair) + (0: dims 0-3 of the slice, 1: dims 4-7);
 *                 b = 2: a half holds the slice's 8 dims, word j = token pair.  (Two tokens per word so
 *                 that one mask yields the fp16 pair a two-term dot-product instruction takes.)
 *   vq params   : [page][kv_head][token g]{fp16 s, fp16 z}
 *
 * Optional grouped angle quantizer (pq_layout.angle_quantizer = PQ_ANGLE_GROUPED): the angle
 * quantizer exactly as Section 3.2 prints it, asymmetric and group-wise like the radius, instead of
 * the uniform grid.  theta = atan2(y, x) in float64 (the printed "+ pi" would only shift every
 * zero-point and is dropped); per pair and group z = min theta, s = (max - min) / 2^t over the
 * valid tokens, rounded once to fp16 and used as rounded;
 *   angle code a = Clamp(floor((theta - z) / s), 0, 2^t - 1) in float64, a = 0 if s == 0
 *   reconstruction theta~ = (a + 1/2) s + z
 * so the lookup table of Section 3.3 is rebuilt from (s, z) for every group (the appendix listing
 * does the same from "tscale" and "tmn").  The parameter block of a page doubles:
 *   params pool : [page][kv_head][2][pair P]{fp16 s, fp16 z}   radius parameters, then angle parameters
 */
#ifndef POLARQUANT_H
#define POLARQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PQ_OK = 0,
  PQ_ERR_INVALID_ARG = -1,   /* null pointer, negative size, inconsistent shapes */
  PQ_ERR_UNSUPPORTED = -2,   /* a layout this build has no kernel for */
  PQ_ERR_WORKSPACE = -3,     /* workspace missing, misaligned or too small */
  PQ_ERR_HIP = -4,           /* a HIP call failed; see pq_last_hip_error() */
  PQ_ERR_STATIC_LIMIT = -5   /* pq_decode_attention_static: the shape needs more scratch than
                                PQ_STATIC_SCRATCH_BYTES */
} pq_status;

typedef enum { PQ_F16 = 0, PQ_F32 = 1 } pq_dtype;

typedef enum {
  PQ_ANGLE_UNIFORM = 0,      /* uniform grid of 2^t bins over [-pi, pi), no angle parameters */
  PQ_ANGLE_GROUPED = 1       /* per-group min / scale (Section 3.2 as printed) */
} pq_angle_quantizer;

/* Shape of the packed cache.  Plain data, passed by const pointer.
 * Supported: head_dim 128; (r_bits, t_bits) with r + t in {6, 8}, 2 <= r, t <= 5
 * -- (4,4) and (3,3) are the paper's main settings, the others its bit
 * allocation ablation (Section 6.1); group_tokens 128; any n_kv_heads >= 1;
 * angle_quantizer PQ_ANGLE_UNIFORM or PQ_ANGLE_GROUPED. */
typedef struct {
  int32_t head_dim;         /* d */
  int32_t r_bits;           /* radius bits r */
  int32_t t_bits;           /* angle bits t */
  int32_t group_tokens;     /* g: tokens per quantization group = tokens per page */
  int32_t n_kv_heads;
  int32_t angle_quantizer;  /* a pq_angle_quantizer */
} pq_layout;

int pq_version(void);
const char* pq_strerror(int status);
/* hipError_t of the last failing HIP call on this host thread (0 if none). */
int pq_last_hip_error(void);

/* Bytes of one page in each pool; 0 if the layout is not supported. */
size_t pq_codes_bytes_per_page(const pq_layout* layout);
size_t pq_params_bytes_per_page(const pq_layout* layout);
size_t pq_values_bytes_per_page(const pq_layout* layout);

/* Quantized values: bytes of one page of the code pool (v_bits 4 or 2) and of the parameter pool. */
size_t pq_vq_bytes_per_page(const pq_layout* layout, int32_t v_bits);
size_t pq_vq_params_bytes_per_page(const pq_layout* layout);

/* Bytes of scratch pq_decode_attention needs for n_seqs sequences of at most
 * max_seq_len tokens (256-byte aligned device memory); 0 on invalid arguments. */
size_t pq_decode_workspace_bytes(const pq_layout* layout, int32_t n_seqs, int32_t n_q_heads,
                                 int32_t max_seq_len);

/*
 * pq_encode_keys -- prefill-time encoder (Section 3.2: pair, radius, angle,
 * group-wise radius quantization, bit-pack).
 *
 *   keys          device, post-RoPE keys of ONE sequence; element i of KV head h of
 *                 token n is keys[n * token_stride + h * head_stride + i] (strides in
 *                 elements; the d elements of a head are contiguous)
 *   key_dtype     PQ_F16 or PQ_F32
 *   n_tokens      tokens 0 .. n_tokens-1; group k = tokens [k*g, min((k+1)*g, n_tokens));
 *                 statistics of a partial last group run over its valid tokens
 *   page_ids      device int32 [ceil(n_tokens / g)]: destination page of each group
 *   codes_pool, params_pool   device, written for the named pages only (whole pages:
 *                 padded slots are zero-filled); n_pool_pages is the pool size in pages
 *                 and page ids outside [0, n_pool_pages) are skipped (nothing is written)
 *
 * n_tokens == 0 is a no-op.  Returns PQ_OK once the kernel is enqueued.
 */
int pq_encode_keys(const pq_layout* layout, const void* keys, pq_dtype key_dtype,
                   int64_t token_stride, int64_t head_stride, int64_t n_tokens,
                   const int32_t* page_ids, void* codes_pool, void* params_pool,
                   int64_t n_pool_pages, void* hip_stream);

/*
 * pq_encode_values -- token-wise value quantizer (Section 2; see the layout above).
 *   values        device fp16, element i of KV head h of token n at values[n * token_stride +
 *                 h * head_stride + i] (strides in elements, multiples of 8; 16-byte aligned)
 *   v_bits        4 or 2
 *   page_ids      device int32 [ceil(n_tokens / g)]; pages outside [0, n_pool_pages) are skipped
 *   vq_pool, vq_params_pool   device; whole pages are written, slots past n_tokens with zeros
 */
int pq_encode_values(const pq_layout* layout, int32_t v_bits, const void* values, int64_t token_stride,
                     int64_t head_stride, int64_t n_tokens, const int32_t* page_ids, void* vq_pool,
                     void* vq_params_pool, int64_t n_pool_pages, void* hip_stream);

/*
 * pq_decode_attention -- one decode step per sequence against the packed cache
 * (Section 3.3 / Appendix A for the table-lookup query-key product; softmax and
 * fp16 value aggregation are standard attention, Section 2).
 *
 *   q             device [n_seqs][n_q_heads][d], post-RoPE, q_dtype PQ_F16 or PQ_F32.
 *                 Query head h reads KV head h / (n_q_heads / n_kv_heads); the ratio may be
 *                 1 .. 16.  Kernels serve 8, 4, 2 or 1 query heads per pass over the cache (8
 *                 with fp16 values, in launches large enough for the role-specialised kernel,
 *                 see pq_decode_kernel_name), so a ratio of 1, 2, 4 (or 8) reads the cache once,
 *                 6 = 4 + 2 twice, 12 = 8 + 4 twice, ...
 *   block_table   device int32 [n_seqs][max_pages_per_seq]: page of tokens
 *                 [i*g, (i+1)*g) of each sequence; entries past a sequence's last page
 *                 are ignored
 *   seq_lens      device int32 [n_seqs]; a length <= 0 gives an all-zero output row;
 *                 lengths above max_seq_len are treated as max_seq_len
 *   max_seq_len   host-known upper bound of seq_lens (sizes the launch);
 *                 ceil(max_seq_len / g) <= max_pages_per_seq
 *   v_pool, v_bits, v_params_pool
 *                 v_bits 16: v_pool is the fp16 value pool, v_params_pool is ignored (NULL);
 *                 v_bits 4 or 2: v_pool is the quantized value pool and v_params_pool its
 *                 parameter pool
 *   n_pool_pages  pool size in pages; a block-table entry outside [0, n_pool_pages)
 *                 makes that page count as masked (no read happens)
 *   sm_scale      softmax scale (1/sqrt(d) for standard attention)
 *   out           device fp32 [n_seqs][n_q_heads][d]
 *   scores        optional device fp32 [n_seqs][n_q_heads][scores_stride]: raw q . k~
 *                 (before sm_scale) of tokens < seq_len; NULL to skip (timed runs)
 *   residual_keys optional device fp16 [n_seqs][n_kv_heads][g][d] (16-byte aligned), see
 *                 pq_append_keys: when given, the keys of a sequence's last, incomplete group
 *                 (tokens floor(len/g)*g .. len-1) are read from it un-quantized and scored by
 *                 plain dot products; packed pages then hold complete groups only.  NULL: the
 *                 incomplete group, if any, is read from its packed page (as pq_encode_keys
 *                 writes it).  Values always come from the value pool.
 *   workspace     device, >= pq_decode_workspace_bytes(layout, n_seqs, n_q_heads, max_seq_len),
 *                 256-byte aligned; contents are scratch
 *
 * Scores, softmax statistics and outputs are fp32.  The probabilities that weight the values are
 * fp32 too, except with quantized values and in 8-head passes, where they are rounded to fp16
 * (pairs of tokens for the two-term fp16 dot product with an fp32 accumulator; with quantized
 * values the token's fp16 scale is folded in before the rounding).
 */
int pq_decode_attention(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                        int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                        const void* v_pool, int32_t v_bits, const void* v_params_pool,
                        int64_t n_pool_pages, const int32_t* block_table,
                        int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len,
                        float sm_scale, float* out, float* scores, int64_t scores_stride,
                        const void* residual_keys, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/*
 * pq_decode_attention_static -- pq_decode_attention for callers that cannot allocate device
 * memory and have no workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, kernels and results as pq_decode_attention,
 * without `workspace` / `workspace_bytes`: the chunk partials go to a static device array of
 * PQ_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process ends).
 * The call allocates and frees nothing.
 *   - A shape whose pq_decode_workspace_bytes(...) exceeds PQ_STATIC_SCRATCH_BYTES is rejected with
 *     PQ_ERR_STATIC_LIMIT before anything is launched.  8 MiB covers e.g. 16 sequences x 32 query
 *     heads x 32K tokens (2.1 MiB), 64 ragged sequences of up to 16K tokens (4.2 MiB), one
 *     sequence of 4M tokens.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on the same GPU
 *     (two streams, two host threads) race on it and give wrong results.  Calls ordered on one
 *     stream are safe; the array's contents after a call are scratch and nothing in it needs to be
 *     cleared between calls (every slot a call reads it has written before).
 *   - The array's device address is looked up (hipGetSymbolAddress) on the first call on each
 *     device, with that device current; make that first call outside a graph capture.
 */
#define PQ_STATIC_SCRATCH_BYTES (8u << 20)
int pq_decode_attention_static(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                               int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                               const void* v_pool, int32_t v_bits, const void* v_params_pool,
                               int64_t n_pool_pages, const int32_t* block_table,
                               int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len,
                               float sm_scale, float* out, float* scores, int64_t scores_stride,
                               const void* residual_keys, void* hip_stream);

/*
 * The two stages of pq_decode_attention, callable on their own (the benchmark
 * times them separately).  pq_decode_partials runs the split-sequence kernel:
 * every (sequence, KV head, chunk of pages) work-group writes its softmax
 * partial (running maximum, denominator, un-normalised output) into the
 * workspace.  pq_decode_merge combines the chunks of each (sequence, query
 * head) into `out`.  Arguments as in pq_decode_attention; the merge must be given the same
 * layout, n_seqs, n_q_heads, seq_lens, max_seq_len and workspace as the partials call it follows
 * (they fix how the sequences were cut into chunks).
 */
int pq_decode_partials(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                       int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                       const void* v_pool, int32_t v_bits, const void* v_params_pool,
                       int64_t n_pool_pages, const int32_t* block_table,
                       int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len,
                       float sm_scale, float* scores, int64_t scores_stride, const void* residual_keys,
                       void* workspace, size_t workspace_bytes, void* hip_stream);
int pq_decode_merge(const pq_layout* layout, int32_t n_seqs, int32_t n_q_heads,
                    const int32_t* seq_lens, int32_t max_seq_len, float* out,
                    const void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * pq_decode_kernel_name -- name of the attention kernel pq_decode_partials / pq_decode_attention
 * launch for this shape ("" on invalid arguments).  The choice depends on the launch shape (see
 * pq_decode_partials); profiles and the benchmark use this to name the kernel that really ran.
 * The string is static storage.
 */
const char* pq_decode_kernel_name(const pq_layout* layout, int32_t n_seqs, int32_t n_q_heads,
                                  int32_t max_seq_len, int32_t v_bits);

/*
 * pq_decode_merges_in_kernel -- 1 if pq_decode_attention serves this shape with one kernel that
 * shares the launch out evenly and combines the partial results itself, 0 if it launches one
 * work-group per chunk followed by the merge kernel; a negative pq_status on invalid arguments.
 * Launches of few (sequence, KV head) units and the kernels without role specialisation take the
 * second form.  For profiles and the benchmark, like pq_decode_kernel_name.
 */
int pq_decode_merges_in_kernel(const pq_layout* layout, int32_t n_seqs, int32_t n_q_heads,
                               int32_t max_seq_len, int32_t v_bits);

/*
 * pq_append_keys -- one decode step's new key per sequence.  Methods of this kind keep the most
 * recent keys un-quantized until a full group exists (the "residual" of Appendix B.1): the key of
 * token len (len = seq_lens[s], the length BEFORE the append) is rounded to fp16 and stored in slot
 * len % g of the sequence's residual buffer; when that completes a group (len % g == g - 1) the g
 * residual keys are encoded, exactly as pq_encode_keys would encode them, into page
 * block_table[s][len / g] of the pools.  The caller increments seq_lens afterwards and files the
 * new value row into the value pool itself.
 *
 *   new_keys      device [n_seqs][n_kv_heads][d], post-RoPE, PQ_F16 or PQ_F32 (16-byte aligned)
 *   residual      device fp16 [n_seqs][n_kv_heads][g][d] (16-byte aligned), owned by the caller
 *   seq_lens      device int32 [n_seqs]; a negative length skips the sequence
 *   A group whose page index is >= max_pages_per_seq or whose page id is outside the pool is not
 *   encoded (nothing is written to the pools).
 */
int pq_append_keys(const pq_layout* layout, const void* new_keys, pq_dtype key_dtype, int32_t n_seqs,
                   void* residual, const int32_t* seq_lens, const int32_t* block_table,
                   int32_t max_pages_per_seq, void* codes_pool, void* params_pool,
                   int64_t n_pool_pages, void* hip_stream);

/*
 * pq_score_keys -- the query-key product alone: raw scores q . k~ of every cached token
 * through the lookup table (Section 3.3, Appendix A).  This is the operation whose latency
 * the paper reports in Section 5.2 (query-key multiplication kernel).  Arguments as in
 * pq_decode_attention; `scores` (device fp32 [n_seqs][n_q_heads][scores_stride], scores_stride
 * >= max_seq_len, < 2^28: PQ_ERR_UNSUPPORTED beyond) receives the scores of tokens < seq_len,
 * other elements are left untouched.  A score equals, bit for bit, the one pq_decode_attention
 * computes (and reports through its own `scores` argument) for the same cache and query.
 * No workspace is needed.  residual_keys as in pq_decode_attention (NULL: every group is read
 * from the packed pages).
 */
int pq_score_keys(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                  int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                  int64_t n_pool_pages, const int32_t* block_table, int32_t max_pages_per_seq,
                  const int32_t* seq_lens, int32_t max_seq_len, float* scores, int64_t scores_stride,
                  const void* residual_keys, void* hip_stream);

/*
 * pq_probe_read_stream -- measurement aid, not part of the method: a streaming read of
 * `bytes` (multiple of 16) device bytes with non-temporal 128-bit loads, each wavefront taking
 * 40 KB blocks as the decode kernel takes pages, XOR-folded into sink[0..63] (device uint32[64],
 * so the loads cannot be elided).  Timed by the benchmark to report what this device streams
 * from HBM when no arithmetic is in the way.
 */
int pq_probe_read_stream(const void* src, size_t bytes, uint32_t* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* POLARQUANT_H */
