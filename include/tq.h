/* tq.h - C ABI of the MI355X (gfx950) int4 compressed-domain decode-attention library.
 *
 * The library computes single-query (decode) scaled-dot-product attention directly on a
 * KV cache stored as packed int4 codes with one fp16 scale and one fp16 zero-point per
 * group of 32 consecutive head_dim elements (Sec. 2.1, Eq. 2-3; groups of 64 and 128 are offered
 * too, see tq_kv_cache), dequantising in registers
 * and never writing a dequantised K or V matrix (Sec. 3.1, Alg. 1), with the sequence split
 * into chunks whose partial results are merged by an online-softmax correction
 * (Sec. 3.2, Eq. 6).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library allocates
 *     nothing, frees nothing and never synchronises: work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and the call returns.
 *   - Arguments are validated on the host before anything is launched.  A call that fails
 *     validation launches nothing and touches no device memory.
 *   - Return value: TQ_OK (0) or a negative TQ_ERR_* code.  Nothing is thrown across the ABI.
 *   - Inputs must be finite; NaN/Inf are not scanned for and give unspecified output.
 *   - fp16 is IEEE binary16.  Arrays are dense, row-major, no padding, in the shapes given,
 *     and every data pointer is 16-byte aligned.
 */
#ifndef TQ_H_
#define TQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  TQ_OK = 0,
  TQ_ERR_NULL = -1,        /* a required pointer is NULL                                        */
  TQ_ERR_SHAPE = -2,       /* head_dim not in {128,256,512}, group_size not in {32,64,128}, batch/heads < 1,
                              n_q_heads not a multiple of n_kv_heads, unknown layout            */
  TQ_ERR_EMPTY = -3,       /* seq_len < 1 or n_new < 1                                          */
  TQ_ERR_CAPACITY = -4,    /* pos < 0, pos + n_new > capacity, or seq_len > capacity            */
  TQ_ERR_WORKSPACE = -5,   /* workspace / dense scratch smaller than the *_bytes() query says   */
  TQ_ERR_UNSUPPORTED = -6, /* a shape or option the kernels do not cover (e.g. an unknown variant) */
  TQ_ERR_HIP = -7,         /* the HIP runtime reported an error at launch                       */
  TQ_ERR_ALIGN = -8        /* a data pointer is not 16-byte aligned (workspace: 256-byte)        */
};

enum { TQ_LAYOUT_CANONICAL = 0 };

/* One layer's caller-owned cache (Sec. 2.1).  Canonical layout:
 *   k_codes, v_codes : uint8 [batch][n_kv_heads][capacity][head_dim/2]
 *                      byte b of a token holds element 2b in its low nibble and element 2b+1
 *                      in its high nibble (element j of a 16-bit word sits in bits 4j..4j+3,
 *                      the order the masks of Eq. 5 assume)
 *   k_scale, k_zero,
 *   v_scale, v_zero  : fp16  [batch][n_kv_heads][capacity][head_dim/group_size]
 * 4 + 32/group_size bits per element in total: 5.0 at the paper's group size of 32 (its 3.2x against fp16),
 * 4.5 at 64, 4.25 at 128.  Tokens [0, seq_len) are valid; the rest is never read.
 * group_size 32 is what the matrix-core kernels are built for (one matrix instruction per group).  Sec. 2.1
 * states the scheme for groups of g consecutive elements: 64 and 128 are accepted by every call (same
 * arithmetic per group, same bit-exact stores).  At head_dim 128 they take the matrix-core kernel as well
 * (group_size 128: with an even capacity and no sliding window); otherwise the generic vector-ALU kernels,
 * where options that only the matrix-core kernels offer (variant 2, n_queries > 1) answer UNSUPPORTED.
 * (With group_size 128 that kernel reads the scale / zero-point arrays two tokens at a time: up to one token
 * past seq_len, inside the row.) */
typedef struct tq_kv_cache {
  void* k_codes;
  void* v_codes;
  void* k_scale;
  void* k_zero;
  void* v_scale;
  void* v_zero;
  int32_t batch;
  int32_t n_kv_heads;
  int32_t head_dim;    /* 128, 256 or 512 */
  int32_t group_size;  /* 32 (the paper's), 64 or 128 */
  int32_t capacity;    /* tokens allocated per (batch, kv head) */
  int32_t layout;      /* TQ_LAYOUT_CANONICAL */
} tq_kv_cache;

/* Optional tuning knobs for the decode entry points; NULL or zeros = library defaults. */
typedef struct tq_decode_opts {
  int32_t n_splits;  /* chunks the sequence is split into (Sec. 3.2); 0 = heuristic            */
  int32_t variant;   /* 0 = default kernel, 1 = generic vector-ALU kernel, 2 = matrix-core kernel
                        (head_dim 512 has a matrix-core kernel of its own: 0 and 2 both take it)    */
  int32_t window;    /* sliding-window attention (the Gemma local layers of Appendix A): > 0 = every
                        sequence attends only its last `window` tokens, [len - window, len); 0 = all.
                        tq_dequant_then_attend does not offer it (UNSUPPORTED).                  */
  int32_t n_queries; /* query tokens per sequence, 0 or 1 = one (the decode step of Sec. 3.3, S_q = 1).
                        2..8 = a short run of new tokens (speculative verification, a chunk of prefill),
                        which Sec. 3.3 sends to the unfused path and this library attends in the fused
                        kernel: the queries are the LAST n_queries tokens of the sequence (already in the
                        cache, or appended by the call) and causal among themselves, i.e. query t attends
                        tokens [0, len - (n_queries - 1 - t)).  q and out are then fp16
                        [batch][n_queries][n_q_heads][head_dim]; size the workspace with
                        tq_workspace_bytes(batch * n_queries, ...) and pass batch * n_queries as `batch`
                        to tq_sdpa_int4_reduce; k_new / v_new of tq_sdpa_int4_append_decode are
                        [batch][n_kv_heads][n_queries][head_dim].  Every sequence length must be at least
                        n_queries.  With a window, query t attends the last `window` of its tokens.
                        Matrix-core kernels only (variant 1, tq_dequant_then_attend and, at head_dim
                        128 / 256, attn_scale <= 0 answer UNSUPPORTED).                            */
} tq_decode_opts;

/* Quantise and append (Sec. 2.1, Eq. 2-3; "quantize -> store" arm of Sec. 3.3).
 * k_new, v_new: fp16 [batch][n_kv_heads][n_new][head_dim].  Tokens are written at positions
 * pos .. pos+n_new-1 of every (batch, kv head).  Per token, per group of 32 elements, K and V
 * independently:  s = fp16((max-min)/15) computed in fp32 (s := 1.0 if that rounds to 0),
 * z = fp16(-min / s) from the stored s (saturated to +-65504, -0 stored as +0),
 * code = clamp(rint_half_even(x/s + z), 0, 15) with fp32 divide then fp32 add.
 * Errors: NULL, SHAPE, EMPTY (n_new < 1), CAPACITY, HIP. */
int tq_quantize_kv(const tq_kv_cache* cache, const void* k_new, const void* v_new, int32_t pos,
                   int32_t n_new, void* stream);

/* The same with one position per sequence, as a decode server appends: sequence b is written at
 * positions[b] .. positions[b]+n_new-1.  positions: DEVICE int32 [batch], read by the kernel (the
 * host never sees the values): a sequence whose tokens would not fit into [0, capacity) is skipped,
 * nothing of it is written.  Errors: NULL, SHAPE, EMPTY, CAPACITY (n_new > capacity), ALIGN, HIP. */
int tq_quantize_kv_varlen(const tq_kv_cache* cache, const void* k_new, const void* v_new,
                          const int32_t* positions, int32_t n_new, void* stream);

/* Fused compressed-domain decode attention (Sec. 3.1 Alg. 1 + Sec. 3.2 Eq. 6).
 * q, out: fp16 [batch][n_q_heads][head_dim]; query head h reads KV head h / (n_q_heads /
 * n_kv_heads) (GQA rule of Sec. 3.1).  out = softmax(attn_scale * q.K^) V^ over tokens
 * [0, seq_len), fp32 accumulation, fp16 result.  workspace: at least tq_workspace_bytes()
 * bytes, 256-byte aligned, holds the per-chunk partial results; contents undefined on return.
 * Same result as tq_sdpa_int4_partial followed by tq_sdpa_int4_reduce on the same stream (up to the
 * order of the fp32 sums of the merge).  For short sequences, where launch overhead outweighs the
 * stream (see tq_decode_launches), the matrix-core kernel does both in ONE launch: the block that
 * finishes a (batch, KV head) last merges its chunks in place (a sequence that is a single chunk
 * needs no merge: its block writes out).  That path counts the blocks in with arrival counters in device
 * memory owned by the library, one set per WORKSPACE address (kept for the life of the process, left zero by
 * every launch).  Calls that may run at the same time must not share a workspace (they would overwrite each
 * other's partials), so they never share counters either, whether issued eagerly or replayed from a captured
 * graph.  There are 256 sets; a call whose workspace is the 257th distinct address the library sees takes the
 * merge kernel (two launches) instead, with the same result up to the summation order of the merge: results are
 * bit-for-bit repeatable per workspace, not across workspaces.
 * Errors: NULL, SHAPE, EMPTY (seq_len < 1), CAPACITY (seq_len > capacity), WORKSPACE,
 * UNSUPPORTED, HIP. */
int tq_sdpa_int4_decode(const tq_kv_cache* cache, const void* q, int32_t n_q_heads, int32_t seq_len,
                        float attn_scale, void* out, void* workspace, size_t workspace_bytes,
                        const tq_decode_opts* opts, void* stream);

/* tq_sdpa_int4_decode for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same call without the workspace arguments.  The
 * per-chunk partial results go to an array of TQ_STATIC_SCRATCH_BYTES bytes that is part of the library's
 * device code (one copy per GPU, held until the process ends); the call allocates and frees nothing, neither
 * itself nor through the runtime.  Same kernels, same chunking, same result bits as tq_sdpa_int4_decode.
 * A configuration whose tq_workspace_bytes(batch * n_queries, n_q_heads, head_dim) exceeds
 * TQ_STATIC_SCRATCH_BYTES is rejected with TQ_ERR_WORKSPACE (the 70B shape at head_dim 128 fits up to batch 4).
 * All calls on one GPU share that GPU's array: two of them in flight at the same time (different streams) race
 * and give undefined output; calls on one stream are ordered and safe.  The array keeps the last call's
 * contents; nothing in it has to be cleared between calls.  The first call on a device looks the array's address
 * up (hipGetSymbolAddress), so make one call on each device before capturing a graph there.
 * Errors: those of tq_sdpa_int4_decode; WORKSPACE as above; HIP if the address cannot be resolved. */
#define TQ_STATIC_SCRATCH_BYTES ((size_t)20 << 20)
int tq_sdpa_int4_decode_static(const tq_kv_cache* cache, const void* q, int32_t n_q_heads, int32_t seq_len,
                               float attn_scale, void* out, const tq_decode_opts* opts, void* stream);

/* One decode step in one call: tq_quantize_kv(cache, k_new, v_new, seq_len - 1, 1) followed by
 * tq_sdpa_int4_decode(cache, q, ..., seq_len, ...), i.e. the new token of every sequence (k_new,
 * v_new: fp16 [batch][n_kv_heads][1][head_dim]) is quantised, written at position seq_len - 1 and
 * attended together with the seq_len - 1 cached ones (with opts->n_queries = n > 1: n new tokens,
 * written at seq_len - n .. seq_len - 1, each attended by its own query).  Same stored bits and same
 * result as the two calls.  With one query token the append costs no launch of its own: the decode
 * kernel attends the cached tokens, and the merge kernel quantises the new one, stores it and adds
 * its attention term from registers.  Otherwise (several query tokens, a window or sequence of one
 * token) the append kernel is launched first.
 * Errors: those of the two calls. */
int tq_sdpa_int4_append_decode(const tq_kv_cache* cache, const void* k_new, const void* v_new,
                               const void* q, int32_t n_q_heads, int32_t seq_len, float attn_scale,
                               void* out, void* workspace, size_t workspace_bytes,
                               const tq_decode_opts* opts, void* stream);

/* The same with one length per sequence (continuous batching; the paper's kernel takes one
 * common N, Alg. 1): sequence b attends tokens [0, seq_lens[b]).  seq_lens: DEVICE int32 [batch],
 * read by the kernels (the host never sees the values); each is clamped to [1, max_seq_len].
 * max_seq_len (host, <= capacity) only bounds them.  With opts->n_splits == 0 the kernels plan the
 * chunks themselves from the lengths, so that every block gets about the same number of tokens
 * whatever the mix (the cost follows the SUM of the lengths); with n_splits > 0 the sequence range
 * [0, max_seq_len) is cut into that many chunks and those past a sequence's end do no work.  Always
 * two launches (partial kernel + merge kernel).  Other arguments and errors as for
 * tq_sdpa_int4_decode (EMPTY / CAPACITY refer to max_seq_len). */
int tq_sdpa_int4_decode_varlen(const tq_kv_cache* cache, const void* q, int32_t n_q_heads,
                               const int32_t* seq_lens, int32_t max_seq_len, float attn_scale,
                               void* out, void* workspace, size_t workspace_bytes,
                               const tq_decode_opts* opts, void* stream);

/* One decode step with per-sequence lengths, in one call: as tq_sdpa_int4_append_decode, but seq_lens[b]
 * (DEVICE int32 [batch], each in [n_queries, max_seq_len]) is sequence b's length INCLUDING its new token(s),
 * which are written at its last position(s) and attended together with its cached ones; the same result and
 * the same stored bits as tq_quantize_kv_varlen at seq_lens[b] - n followed by tq_sdpa_int4_decode_varlen.
 * With one query token (and no window of a single token) the merge kernel takes the token in: two launches
 * instead of three.  tq_sdpa_int4_append_decode_paged (declared with the paged calls below) is the same over a
 * pool of pages.  Errors: those of the two calls. */
int tq_sdpa_int4_append_decode_varlen(const tq_kv_cache* cache, const void* k_new, const void* v_new,
                                      const void* q, int32_t n_q_heads, const int32_t* seq_lens,
                                      int32_t max_seq_len, float attn_scale, void* out, void* workspace,
                                      size_t workspace_bytes, const tq_decode_opts* opts, void* stream);

/* Paged cache (what a decode server keeps: sequences grow page by page out of one pool).
 * pool: a tq_kv_cache whose `batch` field counts PAGES and whose `capacity` is the page length in
 * tokens (a power of two >= 32), arrays [n_pages][n_kv_heads][page_tokens][...] in the canonical
 * layout.  block_table: DEVICE int32 [batch][max_blocks]; token t of sequence b lives in page
 * block_table[b][t / page_tokens] at row t % page_tokens; only the entries a sequence's tokens
 * reach are read, and they must name pages of the pool (not checked).  `batch` counts sequences
 * (q, out, seq_lens, positions, k_new, v_new and the workspace are sized by it).
 * tq_quantize_kv_paged: as tq_quantize_kv_varlen; a sequence whose tokens would not fit into its
 * max_blocks pages is skipped.  tq_sdpa_int4_decode_paged: as tq_sdpa_int4_decode_varlen (device
 * seq_lens, chunks planned on the device, two launches, opts->window and opts->n_queries as there);
 * max_seq_len <= max_blocks * page_tokens.  Errors as for the varlen calls; SHAPE also for a page
 * length that is not a power of two >= 32. */
int tq_quantize_kv_paged(const tq_kv_cache* pool, const int32_t* block_table, int32_t max_blocks,
                         int32_t batch, const void* k_new, const void* v_new,
                         const int32_t* positions, int32_t n_new, void* stream);
int tq_sdpa_int4_append_decode_paged(const tq_kv_cache* pool, const int32_t* block_table, int32_t max_blocks,
                                     int32_t batch, const void* k_new, const void* v_new, const void* q,
                                     int32_t n_q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                                     float attn_scale, void* out, void* workspace, size_t workspace_bytes,
                                     const tq_decode_opts* opts, void* stream);
int tq_sdpa_int4_decode_paged(const tq_kv_cache* pool, const int32_t* block_table, int32_t max_blocks,
                              int32_t batch, const void* q, int32_t n_q_heads,
                              const int32_t* seq_lens, int32_t max_seq_len, float attn_scale,
                              void* out, void* workspace, size_t workspace_bytes,
                              const tq_decode_opts* opts, void* stream);

/* The two phases of Sec. 3.2, separately callable (used for per-kernel timing).
 * partial: every chunk c writes (o_c, m_c, l_c) for each query head into workspace and
 * *n_splits_out (host int, may be NULL) receives the chunk count used.  reduce: merges
 * n_splits chunks from workspace by Eq. 6 and writes out.  Same errors as above. */
int tq_sdpa_int4_partial(const tq_kv_cache* cache, const void* q, int32_t n_q_heads, int32_t seq_len,
                         float attn_scale, void* workspace, size_t workspace_bytes,
                         const tq_decode_opts* opts, int32_t* n_splits_out, void* stream);
int tq_sdpa_int4_reduce(int32_t batch, int32_t n_q_heads, int32_t head_dim, int32_t n_splits,
                        const void* workspace, size_t workspace_bytes, void* out, void* stream);

/* Unfused comparator (the "dequantize-then-attend" baseline of Sec. 3.1 / Table 2):
 * phase 1 writes dense fp16 K^ and V^ [batch][n_kv_heads][seq_len][head_dim] (K^ first, then V^)
 * into dense_scratch, phase 2 runs fp16 decode attention over them with the same split/merge.
 * (The paper's baseline materialises FP32; fp16 is used here, which only favours the baseline.)
 * Phase 2 runs on the matrix cores for head_dim 128 / 256 with up to 16 query heads per KV head and a
 * positive scale, else (and with opts->variant = 1) on the generic vector-ALU kernel; variant 2 means the same
 * as 0 here.  dense_scratch: at least tq_dense_scratch_bytes() bytes.  Other arguments and errors as for
 * tq_sdpa_int4_decode. */
int tq_dequant_then_attend(const tq_kv_cache* cache, const void* q, int32_t n_q_heads, int32_t seq_len,
                           float attn_scale, void* out, void* workspace, size_t workspace_bytes,
                           void* dense_scratch, size_t dense_scratch_bytes,
                           const tq_decode_opts* opts, void* stream);

/* Size queries (host only, no HIP calls).  Return 0 for invalid shapes.
 * tq_kv_bytes: bytes of one layer's cache, K and V, codes + scales + zero-points
 * (= 2 * batch * n_kv_heads * capacity * (head_dim/2 + 4*head_dim/32); Eq. 1 with 5 bits/element). */
size_t tq_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t head_dim);
size_t tq_dense_scratch_bytes(int32_t batch, int32_t n_kv_heads, int32_t seq_len, int32_t head_dim);
size_t tq_kv_bytes(int32_t batch, int32_t n_kv_heads, int32_t capacity, int32_t head_dim);
/* The same for a group size of 32, 64 or 128: 2 * batch * n_kv_heads * capacity * (head_dim/2 + 4*head_dim/group_size). */
size_t tq_kv_bytes_grouped(int32_t batch, int32_t n_kv_heads, int32_t capacity, int32_t head_dim, int32_t group_size);

/* Chunk count the heuristic would pick (host only). */
int32_t tq_plan_splits(int32_t batch, int32_t n_kv_heads, int32_t seq_len);

/* Kernel launches one tq_sdpa_int4_decode call makes for this cache shape, query head count,
 * seq_len, attn_scale and opts (host only): 1 = partial results and chunk merge in one kernel,
 * 2 = partial kernel + merge kernel, 0 = invalid arguments. */
int32_t tq_decode_launches(const tq_kv_cache* cache, int32_t n_q_heads, int32_t seq_len,
                           float attn_scale, const tq_decode_opts* opts);

/* Static, NUL-terminated description of a status code. */
const char* tq_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TQ_H_ */
