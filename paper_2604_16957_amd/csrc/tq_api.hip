// C ABI of the library: host-side validation, chunk planning and kernel dispatch.
// Every argument check happens here, on the host, before any HIP call, so a rejected call
// launches nothing (and the checks themselves can be exercised on a machine without a GPU).
#include <algorithm>
#include <cmath>
#include <mutex>

#include "tq_internal.h"

namespace {

using tq::DecodeParams;
using tq::half_t;

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// head dimensions the kernels are built for
inline bool head_dim_ok(int d) { return d == 128 || d == 256 || d == 512; }

int check_cache(const tq_kv_cache* c) {
  if (!c) return TQ_ERR_NULL;
  if (!c->k_codes || !c->v_codes || !c->k_scale || !c->k_zero || !c->v_scale || !c->v_zero) return TQ_ERR_NULL;
  if (!head_dim_ok(c->head_dim)) return TQ_ERR_SHAPE;
  if (c->group_size != 32 && c->group_size != 64 && c->group_size != 128) return TQ_ERR_SHAPE;
  if (c->head_dim % c->group_size != 0) return TQ_ERR_SHAPE;
  if (c->batch < 1 || c->n_kv_heads < 1 || c->capacity < 1) return TQ_ERR_SHAPE;
  if (c->layout != TQ_LAYOUT_CANONICAL) return TQ_ERR_SHAPE;
  const void* ptrs[] = {c->k_codes, c->v_codes, c->k_scale, c->k_zero, c->v_scale, c->v_zero};
  for (const void* p : ptrs)
    if (!aligned(p, 16)) return TQ_ERR_ALIGN;
  return TQ_OK;
}

struct Plan { int n_splits, tokens_per_split; };

constexpr int kBlocksMfma = 256;   // matrix-core kernel: 8-wave blocks, one per compute unit
constexpr int kBlocksValu = 512;   // generic kernel: 4-wave blocks, two per compute unit
constexpr int kBlocksWide = 512;   // head_dim 512 matrix-core kernel: 4-wave blocks, two per compute unit

// A chunk is never longer than this many tokens under the heuristic: the fp32 accumulators of one wave
// then take in at most 64 tiles, which bounds the rounding they pick up however long the sequence is.
constexpr int kMaxChunkTokens = 16384;

// Chunks of whole 32-token tiles, never an empty chunk.  The blocks of a launch run in rounds of
// `target_blocks` (what the chip holds at once): as many chunks as fill one round without spilling into a
// second (a 257th block would wait for a whole block's time), or, where that makes chunks longer than
// kMaxChunkTokens, as many as fill the fewest rounds that do not.  With `tiles_per_block_min` > 1 short
// sequences get fewer, fuller blocks (one tile per wave at least).
Plan plan_splits(int batch, int n_kv_heads, int seq_len, int requested, int target_blocks, int tiles_per_block_min) {
  const int tiles = (seq_len + tq::kTile - 1) / tq::kTile;
  int n = requested;
  if (n <= 0) {
    const int64_t rows = (int64_t)batch * n_kv_heads;
    const int64_t need = (seq_len + kMaxChunkTokens - 1) / kMaxChunkTokens;
    const int64_t rounds = std::max<int64_t>(1, (need * rows + target_blocks - 1) / target_blocks);
    n = (int)std::max<int64_t>({1, need, rounds * target_blocks / rows});
    n = std::min(n, std::max(1, tiles / tiles_per_block_min));
    n = (int)std::max<int64_t>(n, need);
  }
  n = std::max(1, std::min({n, tiles, tq::kMaxSplits}));
  const int tiles_per = (tiles + n - 1) / n;
  Plan p;
  p.tokens_per_split = tiles_per * tq::kTile;
  p.n_splits = (seq_len + p.tokens_per_split - 1) / p.tokens_per_split;
  return p;
}

// query tokens per sequence the options ask for
int queries_of(const tq_decode_opts* opts) { return (opts && opts->n_queries > 1) ? opts->n_queries : 1; }
// query rows that share one KV head
int rows_of(const tq_kv_cache* c, int n_q_heads, const tq_decode_opts* opts) {
  return n_q_heads / c->n_kv_heads * queries_of(opts);
}

// `room`: tokens a sequence can hold (the cache's capacity, or max_blocks pages of a paged pool)
int check_decode(const tq_kv_cache* c, const void* q, int n_q_heads, int seq_len, const void* out,
                 const void* workspace, size_t workspace_bytes, const tq_decode_opts* opts, bool need_out,
                 int64_t room = -1) {
  int rc = check_cache(c);
  if (rc == TQ_ERR_NULL) return rc;
  if (!q || (need_out && !out) || !workspace) return TQ_ERR_NULL;
  if (rc != TQ_OK && rc != TQ_ERR_ALIGN) return rc;
  if (n_q_heads < 1 || n_q_heads % c->n_kv_heads != 0) return TQ_ERR_SHAPE;
  if (seq_len < queries_of(opts)) return TQ_ERR_EMPTY;   // (every query token is one of the sequence's tokens)
  if (seq_len > (room >= 0 ? room : (int64_t)c->capacity)) return TQ_ERR_CAPACITY;
  if (rc == TQ_ERR_ALIGN) return rc;
  if (!aligned(q, 16) || (need_out && !aligned(out, 16)) || !aligned(workspace, 256)) return TQ_ERR_ALIGN;
  if (opts) {
    if (opts->variant < 0 || opts->variant > 2 || opts->n_splits < 0 || opts->window < 0) return TQ_ERR_UNSUPPORTED;
    if (opts->n_queries < 0 || opts->n_queries > tq::kMaxQueries) return TQ_ERR_UNSUPPORTED;
    if (opts->n_queries > 1 && opts->variant == 1) return TQ_ERR_UNSUPPORTED;   // matrix-core kernels only
    if (opts->variant == 2 && !tq::wide_supported(c->head_dim) &&
        !tq::mfma_supported(c->head_dim, rows_of(c, n_q_heads, opts)))
      return TQ_ERR_UNSUPPORTED;
  }
  if (workspace_bytes < tq_workspace_bytes(c->batch * queries_of(opts), n_q_heads, c->head_dim)) return TQ_ERR_WORKSPACE;
  return TQ_OK;
}

DecodeParams make_params(const tq_kv_cache* c, const void* q, int n_q_heads, int seq_len, float attn_scale,
                         void* out, void* workspace, const Plan& plan, int n_queries = 1) {
  DecodeParams p{};
  p.k_codes = static_cast<const uint8_t*>(c->k_codes);
  p.v_codes = static_cast<const uint8_t*>(c->v_codes);
  p.k_scale = static_cast<const half_t*>(c->k_scale);
  p.k_zero = static_cast<const half_t*>(c->k_zero);
  p.v_scale = static_cast<const half_t*>(c->v_scale);
  p.v_zero = static_cast<const half_t*>(c->v_zero);
  p.q = static_cast<const half_t*>(q);
  p.out = static_cast<half_t*>(out);
  p.part_o = static_cast<float*>(workspace);
  p.part_ml = p.part_o + tq::workspace_o_floats(c->batch * n_queries, n_q_heads, c->head_dim);
  p.plan = reinterpret_cast<int32_t*>(p.part_ml + tq::workspace_ml_floats(c->batch * n_queries, n_q_heads));
  p.n_q_heads = n_q_heads;
  p.n_queries = n_queries;
  p.n_kv_heads = c->n_kv_heads;
  p.gqa = n_q_heads / c->n_kv_heads;
  p.group = c->group_size;
  p.row_stride = c->capacity;
  p.seq_len = seq_len;
  p.n_splits = plan.n_splits;
  p.tokens_per_split = plan.tokens_per_split;
  p.scale_log2 = attn_scale * 1.4426950408889634f;
  return p;
}

int hip_rc(hipError_t e) { return e == hipSuccess ? TQ_OK : TQ_ERR_HIP; }

// Which kernel a decode call takes, and whether that kernel can also do the chunk merge.
// single: every sequence is one chunk (no merge needed at all); wide: the head_dim 512 matrix-core kernel
struct Route { bool ok, use_mfma, merge, single, wide; };
// The in-kernel merge ends the kernel with a chain of device-wide round trips (publish the partial,
// count in, read all partials) that one block walks alone: about 5 us, against about 3.5 us for the
// separate merge kernel plus its launch.  It pays where the call is bound by launch overhead, not by
// the stream: below this many packed bytes per call.
constexpr int64_t kMergeInKernelMaxBytes = 48ll << 20;

// tokens a sequence of length seq_len attends under the options' sliding window
// (several query tokens: the span all rows together attend, the earliest row's window start to the end)
int windowed(int seq_len, const tq_decode_opts* opts) {
  return (opts && opts->window > 0) ? std::min(seq_len, opts->window + queries_of(opts) - 1) : seq_len;
}
// blocks of the matrix-core kernel that stream one KV head
int mfma_share_of(const tq_kv_cache* cache, int n_q_heads, const tq_decode_opts* opts) {
  return tq::mfma_kv_share(cache->head_dim, rows_of(cache, n_q_heads, opts));
}

Route route_of(const tq_kv_cache* cache, int n_q_heads, int seq_len, float attn_scale, const tq_decode_opts* opts) {
  const int variant = opts ? opts->variant : 0;
  // groups of 64 or 128 elements: the matrix-core kernel at head_dim 128 (see mfma_supports_group), else the
  // generic vector-ALU kernel with one query token per sequence
  // (groups of 128 under a sliding window: a window may start at an odd token, in the middle of a pair)
  const bool pairs_split = cache->group_size == 4 * tq::kGroup && opts && opts->window > 0;
  if (!tq::mfma_supports_group(cache->head_dim, cache->group_size, cache->capacity) || pairs_split) {
    const bool ok = variant != 2 && queries_of(opts) == 1;
    return {ok, false, false, false, false};
  }
  // the matrix-core kernel folds attn_scale into its exp2 argument and needs it positive and finite
  const bool scale_ok = attn_scale > 0.0f && std::isfinite(attn_scale);
  if (variant == 2 && !scale_ok) return {false, false, false, false, false};
  // head_dim 512: its own matrix-core kernel (any finite scale), partials merged by the merge kernel
  if (variant != 1 && tq::wide_supported(cache->head_dim) && std::isfinite(attn_scale))
    return {true, false, false, false, true};
  // the matrix-core kernel addresses a (batch, KV head) row of codes with 32-bit byte offsets
  const bool offsets_ok = (int64_t)seq_len * (cache->head_dim / 2) < (1ll << 31);
  if (variant == 2 && !offsets_ok) return {false, false, false, false, false};
  const int rows = rows_of(cache, n_q_heads, opts);
  const bool use_mfma = variant == 2 || (variant == 0 && scale_ok && offsets_ok &&
                                         tq::mfma_supported(cache->head_dim, rows));
  if (!use_mfma && queries_of(opts) > 1) return {false, false, false, false, false};
  // (more query rows than the kernel's tile holds: several blocks stream each KV head, counted as rows of their own)
  const int rows_per_batch = cache->n_kv_heads * std::max(1, use_mfma ? mfma_share_of(cache, n_q_heads, opts) : 1);
  const int64_t bytes = (int64_t)tq_kv_bytes(cache->batch, rows_per_batch, windowed(seq_len, opts), cache->head_dim);
  // a sequence that is one chunk needs no merge at all: the kernel writes the output itself, whatever the size
  const bool single = use_mfma && plan_splits(cache->batch, rows_per_batch, windowed(seq_len, opts),
                                               opts ? opts->n_splits : 0, kBlocksMfma, 8).n_splits == 1;
  // (a 16-row tile leaves the last block twice the partials to fetch: there the merge kernel is the faster end,
  //  measured 21.8 against 24.1 us with 16 heads per KV head at 32K tokens)
  const bool small_tile = rows_per_batch == 0 || rows * cache->n_kv_heads / rows_per_batch <= 8;
  const bool merge = use_mfma && (single || (bytes <= kMergeInKernelMaxBytes && small_tile &&
                                             tq::mfma_can_merge(cache->batch, rows_per_batch)));
  return {true, use_mfma, merge, single && merge, false};
}

// waves that share one (sequence, KV head) row where single-chunk rows are packed several to a block
int waves_per_packed_row(int64_t total_rows, int target) {
  return total_rows > 4 * target ? 1 : total_rows > 2 * target ? 2 : total_rows > target ? 4 : 8;
}

// Many short sequences with their own lengths: where the (sequence, KV head) rows fill at least two rounds of
// blocks and the longest sequence is no more than about a thousand tokens per wave that will work on it, every
// row is ONE chunk of its own length: the decode kernel writes the output itself, and neither the device-side
// chunk plan nor the merge kernel (one block per sequence and query head) is needed.
bool rows_as_chunks(const tq_kv_cache* cache, int n_q_heads, int seq_len, float attn_scale, const tq_decode_opts* opts,
                    bool paged) {
  if (paged || queries_of(opts) > 1 || (opts && opts->n_splits > 0)) return false;
  const Route r = route_of(cache, n_q_heads, seq_len, attn_scale, opts);
  if (!r.ok || !r.use_mfma) return false;
  const int64_t total = (int64_t)cache->batch * cache->n_kv_heads * mfma_share_of(cache, n_q_heads, opts);
  return total >= 2 * kBlocksMfma && windowed(seq_len, opts) <= 1024 * waves_per_packed_row(total, kBlocksMfma);
}

// One launch of phase 1: what to attend, and what came of it.
struct PartialRequest {
  const tq_kv_cache* cache;            // validated; for a paged pool: the view with batch = sequences
  const void* q;
  int32_t n_q_heads, seq_len;          // seq_len: the common length, or the bound of seq_lens
  const int32_t* seq_lens = nullptr;   // device, per-sequence lengths
  float attn_scale = 0.0f;
  void* out = nullptr;                 // non-null: the kernel may merge the chunks itself and write it
  void* workspace = nullptr;
  const tq_decode_opts* opts = nullptr;
  const void* k_new = nullptr;         // append-and-attend: the step's new token (then seq_len includes it),
  const void* v_new = nullptr;         // taken in by the merge kernel, which then has to run
  const tq::PagedView* paged = nullptr;
  void* stream = nullptr;
  // results
  int32_t n_splits = 0;
  bool merged = false;                 // `out` has been written
  DecodeParams params{};               // what the kernel was given (the merge kernel takes the same)
};

// Phase 1 (and, with `out`, the whole decode where the matrix-core kernel can merge in place).
int run_partial(PartialRequest& rq) {
  const tq_kv_cache* cache = rq.cache;
  const tq_decode_opts* opts = rq.opts;
  const int32_t* seq_lens = rq.seq_lens;
  const int n_q_heads = rq.n_q_heads, seq_len = rq.seq_len;
  const Route r = route_of(cache, n_q_heads, seq_len, rq.attn_scale, opts);
  if (!r.ok) return TQ_ERR_UNSUPPORTED;
  const bool use_mfma = r.use_mfma;
  const int target = use_mfma ? kBlocksMfma : r.wide ? kBlocksWide : kBlocksValu;
  int attended = windowed(seq_len, opts);         // chunks cover the attended tokens only
  // (paged cache: counted from the supertile boundary before the window, see var_start)
  if (rq.paged && attended < seq_len) attended = std::min(seq_len, attended + tq::kTile - 1);
  // append-and-attend: the new token (the last attended one) does not come from the cache
  const bool append_in_merge = rq.k_new != nullptr;
  const int first = seq_len - attended;           // first attended token
  if (append_in_merge) --attended;
  const int row_tiles = r.wide ? tq::wide_row_tiles(rows_of(cache, n_q_heads, opts),
                                                    (int64_t)cache->batch * cache->n_kv_heads, std::max(1, attended))
                               : 1;
  const int mfma_share = use_mfma ? mfma_share_of(cache, n_q_heads, opts) : 1;
  const int rows_per_batch = cache->n_kv_heads * (use_mfma ? mfma_share : row_tiles);
  const bool one_chunk_rows = seq_lens && rq.out != nullptr && !append_in_merge &&
                              rows_as_chunks(cache, n_q_heads, seq_len, rq.attn_scale, opts, rq.paged != nullptr);
  const Plan plan = plan_splits(cache->batch, rows_per_batch, attended, one_chunk_rows ? 1 : opts ? opts->n_splits : 0,
                                target, use_mfma ? 8 : r.wide ? 2 : 1);
  DecodeParams p = make_params(cache, rq.q, n_q_heads, seq_len, rq.attn_scale, rq.out, rq.workspace, plan,
                               queries_of(opts));
  p.seq_lens = seq_lens;
  p.batch = cache->batch;
  if (seq_lens) {
    // the kernels window every sequence's own length (append-and-attend: the lengths count the new token, the
    // chunks and the window over them do not)
    p.len_bias = append_in_merge ? -1 : 0;
    p.window = (opts && opts->window > 0) ? opts->window + queries_of(opts) - 1 + p.len_bias : 0;
  } else {
    p.seq_len = attended;
    p.start = first;
  }
  p.row_window = (opts && queries_of(opts) > 1) ? opts->window : 0;
  if (rq.paged) {
    p.block_table = rq.paged->block_table;
    p.max_blocks = rq.paged->max_blocks;
    p.page_shift = rq.paged->page_shift;
  }
  if (seq_lens && !(opts && opts->n_splits > 0) && !one_chunk_rows) {
    // per-sequence lengths, no chunk count asked for: the kernels plan the chunks themselves from the lengths,
    // `target` chunks over all sequences of a KV head (a requested n_splits keeps the fixed chunking)
    // per KV head: r rounds of target / H_kv chunks, r the smallest count that leaves at least half of them
    // once every sequence has been granted its partial last chunk
    const int per_round = std::max(1, target / rows_per_batch);          // (one round never spills into a second)
    const int rounds = std::max(1, (2 * cache->batch + per_round - 1) / per_round);
    p.var_chunks = rounds * per_round;
    p.var_min_chunk = use_mfma ? 8 * tq::kTile : r.wide ? 2 * tq::kTile : tq::kTile;
    p.n_splits = tq::kMaxSplits;
    // many sequences: the slots of several rounds share blocks (2, 4 or 8 to a block) and run in one
    if (use_mfma) p.waves_per_row = rounds > 4 ? 1 : rounds > 2 ? 2 : rounds > 1 ? 4 : 8;
  }
  rq.params = p;
  if (append_in_merge) {
    rq.params.k_new = static_cast<const half_t*>(rq.k_new);
    rq.params.v_new = static_cast<const half_t*>(rq.v_new);
    rq.params.append_pos = seq_len - 1;
  }
  rq.n_splits = plan.n_splits;
  hipStream_t s = static_cast<hipStream_t>(rq.stream);
  rq.merged = one_chunk_rows || (rq.out != nullptr && r.merge && !seq_lens && !append_in_merge);
  int merge_slot = -1;
  if (rq.merged) {
    // several chunks: the arrival counters of this workspace (none left: the merge kernel does it); rows that are
    // single chunks count nothing
    merge_slot = plan.n_splits > 1 ? tq::mfma_merge_slot_of(rq.workspace) : 0;
    if (merge_slot < 0) rq.merged = false;
  }
  if (rq.merged && use_mfma && plan.n_splits == 1 && !rq.paged) {
    // more single-chunk rows than the chip holds blocks: pack 2, 4 or 8 of them into a block
    p.waves_per_row = waves_per_packed_row((int64_t)cache->batch * rows_per_batch, target);
  }
  if (use_mfma) {
    p.kv_share = mfma_share;
    return hip_rc(tq::launch_partial_mfma(p, cache->batch, cache->head_dim, merge_slot, s));
  }
  if (r.wide) {
    p.kv_share = row_tiles;
    return hip_rc(tq::launch_partial_wide(p, cache->batch, cache->head_dim, s));
  }
  return hip_rc(tq::launch_partial_valu(p, cache->batch, cache->head_dim, false, s));
}

// Phase 2 after run_partial, unless the kernel has merged already.
int finish_decode(const PartialRequest& rq, int rc) {
  if (rc != TQ_OK || rq.merged) return rc;
  return hip_rc(tq::launch_reduce(rq.params, rq.cache->batch, rq.cache->head_dim, static_cast<hipStream_t>(rq.stream)));
}

// A pool of pages seen as a cache: `batch` sequences whose rows are pages of pool->capacity tokens.
int paged_view(const tq_kv_cache* pool, const int32_t* block_table, int32_t max_blocks, int32_t batch,
                      tq_kv_cache* view, tq::PagedView* pv) {
  const int rc = check_cache(pool);
  if (rc == TQ_ERR_NULL || !block_table) return TQ_ERR_NULL;
  if (rc != TQ_OK && rc != TQ_ERR_ALIGN) return rc;
  const int pt = pool->capacity;
  if (pt < tq::kTile || (pt & (pt - 1)) != 0 || batch < 1 || max_blocks < 1) return TQ_ERR_SHAPE;
  if (rc == TQ_ERR_ALIGN || !aligned(block_table, 4)) return TQ_ERR_ALIGN;
  *view = *pool;
  view->batch = batch;
  int shift = 0;
  while ((1 << shift) < pt) ++shift;
  *pv = tq::PagedView{block_table, max_blocks, shift, batch};
  return TQ_OK;
}

// ---- tq_sdpa_int4_decode_static: the workspace of callers that cannot allocate.
// One array per GPU the library runs on, held until the process ends.  In host code the array's name is only a
// stand-in for the symbol: the memory's address on a device is what hipGetSymbolAddress returns with that
// device current, and that pointer is what the kernels get.
constexpr size_t kScratchBytes = TQ_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices];                   // per device: where that device's copy of `scratch` lives

// The current device's copy of `scratch` (resolved once per device, on the first call with that device current).
int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TQ_ERR_HIP;
  std::lock_guard<std::mutex> guard(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TQ_ERR_HIP;
    scratch_ptr[dev] = ptr;
  }
  *out = scratch_ptr[dev];
  return TQ_OK;
}

}  // namespace

extern "C" {

size_t tq_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t head_dim) {
  if (batch < 1 || n_q_heads < 1 || !head_dim_ok(head_dim)) return 0;
  // partial outputs, their (m, l), and one cache line for the device-side chunk plan
  return (tq::workspace_o_floats(batch, n_q_heads, head_dim) + tq::workspace_ml_floats(batch, n_q_heads)) *
             sizeof(float) + 256;
}

size_t tq_dense_scratch_bytes(int32_t batch, int32_t n_kv_heads, int32_t seq_len, int32_t head_dim) {
  if (batch < 1 || n_kv_heads < 1 || seq_len < 1 || !head_dim_ok(head_dim)) return 0;
  return (size_t)2 * batch * n_kv_heads * seq_len * head_dim * sizeof(half_t);
}

size_t tq_kv_bytes_grouped(int32_t batch, int32_t n_kv_heads, int32_t capacity, int32_t head_dim, int32_t group_size) {
  if (group_size != 32 && group_size != 64 && group_size != 128) return 0;
  if (batch < 1 || n_kv_heads < 1 || capacity < 1 || head_dim < group_size || head_dim % group_size != 0) return 0;
  const size_t per_token = (size_t)head_dim / 2 + 2 * sizeof(half_t) * (head_dim / group_size);
  return (size_t)2 * batch * n_kv_heads * capacity * per_token;
}

size_t tq_kv_bytes(int32_t batch, int32_t n_kv_heads, int32_t capacity, int32_t head_dim) {
  return tq_kv_bytes_grouped(batch, n_kv_heads, capacity, head_dim, tq::kGroup);
}

int32_t tq_plan_splits(int32_t batch, int32_t n_kv_heads, int32_t seq_len) {
  if (batch < 1 || n_kv_heads < 1 || seq_len < 1) return 0;
  return plan_splits(batch, n_kv_heads, seq_len, 0, kBlocksMfma, 8).n_splits;
}

int32_t tq_decode_launches(const tq_kv_cache* cache, int32_t n_q_heads, int32_t seq_len, float attn_scale,
                           const tq_decode_opts* opts) {
  const int rc = check_cache(cache);
  if (rc != TQ_OK && rc != TQ_ERR_ALIGN) return 0;
  if (n_q_heads < 1 || n_q_heads % cache->n_kv_heads != 0 || seq_len < 1 || seq_len > cache->capacity) return 0;
  if (opts && (opts->variant < 0 || opts->variant > 2)) return 0;
  if (opts && (opts->n_queries < 0 || opts->n_queries > tq::kMaxQueries || seq_len < queries_of(opts))) return 0;
  if (opts && opts->variant == 2 && !tq::wide_supported(cache->head_dim) &&
      !tq::mfma_supported(cache->head_dim, rows_of(cache, n_q_heads, opts)))
    return 0;
  const Route r = route_of(cache, n_q_heads, seq_len, attn_scale, opts);
  if (!r.ok) return 0;
  return r.merge ? 1 : 2;
}

const char* tq_status_string(int status) {
  switch (status) {
    case TQ_OK: return "ok";
    case TQ_ERR_NULL: return "a required pointer is NULL";
    case TQ_ERR_SHAPE: return "unsupported or inconsistent shape";
    case TQ_ERR_EMPTY: return "empty request (seq_len < 1 or n_new < 1)";
    case TQ_ERR_CAPACITY: return "position or sequence length exceeds the cache capacity";
    case TQ_ERR_WORKSPACE: return "workspace or dense scratch too small";
    case TQ_ERR_UNSUPPORTED: return "shape or option not covered by the kernels";
    case TQ_ERR_HIP: return "HIP runtime error at launch";
    case TQ_ERR_ALIGN: return "pointer not sufficiently aligned";
    default: return "unknown status";
  }
}

int tq_quantize_kv(const tq_kv_cache* cache, const void* k_new, const void* v_new, int32_t pos, int32_t n_new,
                   void* stream) {
  int rc = check_cache(cache);
  if (rc == TQ_ERR_NULL) return rc;
  if (!k_new || !v_new) return TQ_ERR_NULL;
  if (rc != TQ_OK && rc != TQ_ERR_ALIGN) return rc;
  if (n_new < 1) return TQ_ERR_EMPTY;
  if (pos < 0 || (int64_t)pos + n_new > cache->capacity) return TQ_ERR_CAPACITY;
  if (rc == TQ_ERR_ALIGN || !aligned(k_new, 16) || !aligned(v_new, 16)) return TQ_ERR_ALIGN;
  return hip_rc(tq::launch_quantize(*cache, k_new, v_new, pos, nullptr, n_new, static_cast<hipStream_t>(stream)));
}

int tq_quantize_kv_varlen(const tq_kv_cache* cache, const void* k_new, const void* v_new, const int32_t* positions,
                          int32_t n_new, void* stream) {
  int rc = check_cache(cache);
  if (rc == TQ_ERR_NULL) return rc;
  if (!k_new || !v_new || !positions) return TQ_ERR_NULL;
  if (rc != TQ_OK && rc != TQ_ERR_ALIGN) return rc;
  if (n_new < 1) return TQ_ERR_EMPTY;
  if (n_new > cache->capacity) return TQ_ERR_CAPACITY;
  if (rc == TQ_ERR_ALIGN || !aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(positions, 4)) return TQ_ERR_ALIGN;
  return hip_rc(tq::launch_quantize(*cache, k_new, v_new, 0, positions, n_new, static_cast<hipStream_t>(stream)));
}

int tq_sdpa_int4_partial(const tq_kv_cache* cache, const void* q, int32_t n_q_heads, int32_t seq_len,
                         float attn_scale, void* workspace, size_t workspace_bytes, const tq_decode_opts* opts,
                         int32_t* n_splits_out, void* stream) {
  const int rc = check_decode(cache, q, n_q_heads, seq_len, nullptr, workspace, workspace_bytes, opts, false);
  if (rc != TQ_OK) return rc;
  PartialRequest rq{cache, q, n_q_heads, seq_len};
  rq.attn_scale = attn_scale;
  rq.workspace = workspace;
  rq.opts = opts;
  rq.stream = stream;
  const int out_rc = run_partial(rq);
  if (n_splits_out) *n_splits_out = rq.n_splits;
  return out_rc;
}

int tq_sdpa_int4_reduce(int32_t batch, int32_t n_q_heads, int32_t head_dim, int32_t n_splits, const void* workspace,
                        size_t workspace_bytes, void* out, void* stream) {
  if (!workspace || !out) return TQ_ERR_NULL;
  if (batch < 1 || n_q_heads < 1 || !head_dim_ok(head_dim)) return TQ_ERR_SHAPE;
  if (n_splits < 1) return TQ_ERR_EMPTY;
  if (n_splits > tq::kMaxSplits) return TQ_ERR_UNSUPPORTED;
  if (!aligned(workspace, 256) || !aligned(out, 16)) return TQ_ERR_ALIGN;
  if (workspace_bytes < tq_workspace_bytes(batch, n_q_heads, head_dim)) return TQ_ERR_WORKSPACE;
  DecodeParams p{};
  p.part_o = const_cast<float*>(static_cast<const float*>(workspace));
  p.part_ml = p.part_o + tq::workspace_o_floats(batch, n_q_heads, head_dim);
  p.out = static_cast<half_t*>(out);
  p.n_q_heads = n_q_heads;
  p.n_splits = n_splits;
  return hip_rc(tq::launch_reduce(p, batch, head_dim, static_cast<hipStream_t>(stream)));
}

int tq_sdpa_int4_decode(const tq_kv_cache* cache, const void* q, int32_t n_q_heads, int32_t seq_len, float attn_scale,
                        void* out, void* workspace, size_t workspace_bytes, const tq_decode_opts* opts, void* stream) {
  int rc = check_decode(cache, q, n_q_heads, seq_len, out, workspace, workspace_bytes, opts, true);
  if (rc != TQ_OK) return rc;
  PartialRequest rq{cache, q, n_q_heads, seq_len};
  rq.attn_scale = attn_scale;
  rq.out = out;
  rq.workspace = workspace;
  rq.opts = opts;
  rq.stream = stream;
  return finish_decode(rq, run_partial(rq));
}

int tq_sdpa_int4_decode_static(const tq_kv_cache* cache, const void* q, int32_t n_q_heads, int32_t seq_len,
                               float attn_scale, void* out, const tq_decode_opts* opts, void* stream) {
  // everything that can be told without the workspace first (a fake, aligned address stands in for it), so that a
  // rejected call touches neither the device nor the runtime
  void* const fake = reinterpret_cast<void*>(uintptr_t{256});
  int rc = check_decode(cache, q, n_q_heads, seq_len, out, fake, ~size_t{0}, opts, true);
  if (rc != TQ_OK) return rc;
  if (tq_workspace_bytes(cache->batch * queries_of(opts), n_q_heads, cache->head_dim) > kScratchBytes)
    return TQ_ERR_WORKSPACE;
  void* ws = nullptr;
  rc = scratch_of_current_device(&ws);
  if (rc != TQ_OK) return rc;
  // Nothing in the array has to start at zero: every partial the merge reads has been written by the same call's
  // first phase, and the arrival counters of the one-launch route live elsewhere and reset themselves.
  PartialRequest rq{cache, q, n_q_heads, seq_len};
  rq.attn_scale = attn_scale;
  rq.out = out;
  rq.workspace = ws;
  rq.opts = opts;
  rq.stream = stream;
  return finish_decode(rq, run_partial(rq));
}

int tq_sdpa_int4_append_decode(const tq_kv_cache* cache, const void* k_new, const void* v_new, const void* q,
                               int32_t n_q_heads, int32_t seq_len, float attn_scale, void* out, void* workspace,
                               size_t workspace_bytes, const tq_decode_opts* opts, void* stream) {
  int rc = check_decode(cache, q, n_q_heads, seq_len, out, workspace, workspace_bytes, opts, true);
  if (rc != TQ_OK) return rc;
  if (!k_new || !v_new) return TQ_ERR_NULL;
  if (!aligned(k_new, 16) || !aligned(v_new, 16)) return TQ_ERR_ALIGN;
  const Route r = route_of(cache, n_q_heads, seq_len, attn_scale, opts);
  if (!r.ok) return TQ_ERR_UNSUPPORTED;
  PartialRequest rq{cache, q, n_q_heads, seq_len};
  rq.attn_scale = attn_scale;
  rq.out = out;
  rq.workspace = workspace;
  rq.opts = opts;
  rq.stream = stream;
  // The merge kernel takes the token in (one query token, at least one cached token to attend: no append launch,
  // nothing read back); else the append kernel runs first.  Where every sequence is a single chunk there is no
  // merge kernel to begin with (the decode kernel writes the output itself): the append kernel, then that.
  if (queries_of(opts) == 1 && windowed(seq_len, opts) >= 2 && !r.single && cache->group_size == tq::kGroup) {
    rq.k_new = k_new;
    rq.v_new = v_new;
  } else {                                        // the append kernel first, then the plain decode
    const int n_new = queries_of(opts);
    rc = hip_rc(tq::launch_quantize(*cache, k_new, v_new, seq_len - n_new, nullptr, n_new,
                                    static_cast<hipStream_t>(stream)));
    if (rc != TQ_OK) return rc;
  }
  return finish_decode(rq, run_partial(rq));
}

int tq_quantize_kv_paged(const tq_kv_cache* pool, const int32_t* block_table, int32_t max_blocks, int32_t batch,
                         const void* k_new, const void* v_new, const int32_t* positions, int32_t n_new, void* stream) {
  tq_kv_cache view;
  tq::PagedView pv;
  const int rc = paged_view(pool, block_table, max_blocks, batch, &view, &pv);
  if (rc != TQ_OK) return rc;
  if (!k_new || !v_new || !positions) return TQ_ERR_NULL;
  if (n_new < 1) return TQ_ERR_EMPTY;
  if ((int64_t)n_new > (int64_t)max_blocks * pool->capacity) return TQ_ERR_CAPACITY;
  if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(positions, 4)) return TQ_ERR_ALIGN;
  return hip_rc(tq::launch_quantize(view, k_new, v_new, 0, positions, n_new, static_cast<hipStream_t>(stream), &pv));
}

int tq_sdpa_int4_decode_paged(const tq_kv_cache* pool, const int32_t* block_table, int32_t max_blocks, int32_t batch,
                              const void* q, int32_t n_q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                              float attn_scale, void* out, void* workspace, size_t workspace_bytes,
                              const tq_decode_opts* opts, void* stream) {
  tq_kv_cache view;
  tq::PagedView pv;
  int rc = paged_view(pool, block_table, max_blocks, batch, &view, &pv);
  if (rc != TQ_OK) return rc;
  rc = check_decode(&view, q, n_q_heads, max_seq_len, out, workspace, workspace_bytes, opts, true,
                    (int64_t)max_blocks * pool->capacity);
  if (rc != TQ_OK) return rc;
  if (!seq_lens) return TQ_ERR_NULL;
  if (!aligned(seq_lens, 4)) return TQ_ERR_ALIGN;
  PartialRequest rq{&view, q, n_q_heads, max_seq_len};
  rq.seq_lens = seq_lens;
  rq.attn_scale = attn_scale;
  rq.out = out;
  rq.workspace = workspace;
  rq.opts = opts;
  rq.paged = &pv;
  rq.stream = stream;
  return finish_decode(rq, run_partial(rq));
}

namespace {
// One decode step with per-sequence lengths that count the step's new token: the merge kernel takes the token
// in where it can (one query token; a window, if any, of at least two tokens), else the append kernel runs first.
int append_decode_with_lengths(PartialRequest& rq, const void* k_new, const void* v_new) {
  const tq_decode_opts* opts = rq.opts;
  // (where every row is a single chunk there is no merge kernel to take the token in: the append kernel, then the decode)
  const bool one_chunk_rows = rows_as_chunks(rq.cache, rq.n_q_heads, rq.seq_len, rq.attn_scale, opts, rq.paged != nullptr);
  if (queries_of(opts) == 1 && !(opts && opts->window == 1) && rq.seq_len >= 2 && !one_chunk_rows &&
      rq.cache->group_size == tq::kGroup) {
    rq.k_new = k_new;
    rq.v_new = v_new;
  } else {
    const int n_new = queries_of(opts);
    const int rc = hip_rc(tq::launch_quantize(*rq.cache, k_new, v_new, -n_new, rq.seq_lens, n_new,
                                              static_cast<hipStream_t>(rq.stream), rq.paged));
    if (rc != TQ_OK) return rc;
  }
  return finish_decode(rq, run_partial(rq));
}
}  // namespace

int tq_sdpa_int4_append_decode_varlen(const tq_kv_cache* cache, const void* k_new, const void* v_new, const void* q,
                                      int32_t n_q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                                      float attn_scale, void* out, void* workspace, size_t workspace_bytes,
                                      const tq_decode_opts* opts, void* stream) {
  int rc = check_decode(cache, q, n_q_heads, max_seq_len, out, workspace, workspace_bytes, opts, true);
  if (rc != TQ_OK) return rc;
  if (!seq_lens || !k_new || !v_new) return TQ_ERR_NULL;
  if (!aligned(seq_lens, 4) || !aligned(k_new, 16) || !aligned(v_new, 16)) return TQ_ERR_ALIGN;
  if (!route_of(cache, n_q_heads, max_seq_len, attn_scale, opts).ok) return TQ_ERR_UNSUPPORTED;
  PartialRequest rq{cache, q, n_q_heads, max_seq_len};
  rq.seq_lens = seq_lens;
  rq.attn_scale = attn_scale;
  rq.out = out;
  rq.workspace = workspace;
  rq.opts = opts;
  rq.stream = stream;
  return append_decode_with_lengths(rq, k_new, v_new);
}

int tq_sdpa_int4_append_decode_paged(const tq_kv_cache* pool, const int32_t* block_table, int32_t max_blocks,
                                     int32_t batch, const void* k_new, const void* v_new, const void* q,
                                     int32_t n_q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                                     float attn_scale, void* out, void* workspace, size_t workspace_bytes,
                                     const tq_decode_opts* opts, void* stream) {
  tq_kv_cache view;
  tq::PagedView pv;
  int rc = paged_view(pool, block_table, max_blocks, batch, &view, &pv);
  if (rc != TQ_OK) return rc;
  rc = check_decode(&view, q, n_q_heads, max_seq_len, out, workspace, workspace_bytes, opts, true,
                    (int64_t)max_blocks * pool->capacity);
  if (rc != TQ_OK) return rc;
  if (!seq_lens || !k_new || !v_new) return TQ_ERR_NULL;
  if (!aligned(seq_lens, 4) || !aligned(k_new, 16) || !aligned(v_new, 16)) return TQ_ERR_ALIGN;
  if (!route_of(&view, n_q_heads, max_seq_len, attn_scale, opts).ok) return TQ_ERR_UNSUPPORTED;
  PartialRequest rq{&view, q, n_q_heads, max_seq_len};
  rq.seq_lens = seq_lens;
  rq.attn_scale = attn_scale;
  rq.out = out;
  rq.workspace = workspace;
  rq.opts = opts;
  rq.paged = &pv;
  rq.stream = stream;
  return append_decode_with_lengths(rq, k_new, v_new);
}

int tq_sdpa_int4_decode_varlen(const tq_kv_cache* cache, const void* q, int32_t n_q_heads, const int32_t* seq_lens,
                               int32_t max_seq_len, float attn_scale, void* out, void* workspace,
                               size_t workspace_bytes, const tq_decode_opts* opts, void* stream) {
  int rc = check_decode(cache, q, n_q_heads, max_seq_len, out, workspace, workspace_bytes, opts, true);
  if (rc != TQ_OK) return rc;
  if (!seq_lens) return TQ_ERR_NULL;
  if (!aligned(seq_lens, 4)) return TQ_ERR_ALIGN;
  PartialRequest rq{cache, q, n_q_heads, max_seq_len};
  rq.seq_lens = seq_lens;
  rq.attn_scale = attn_scale;
  rq.out = out;
  rq.workspace = workspace;
  rq.opts = opts;
  rq.stream = stream;
  return finish_decode(rq, run_partial(rq));       // the merge works out from the same lengths which chunks exist
}

int tq_dequant_then_attend(const tq_kv_cache* cache, const void* q, int32_t n_q_heads, int32_t seq_len,
                           float attn_scale, void* out, void* workspace, size_t workspace_bytes, void* dense_scratch,
                           size_t dense_scratch_bytes, const tq_decode_opts* opts, void* stream) {
  int rc = check_decode(cache, q, n_q_heads, seq_len, out, workspace, workspace_bytes, opts, true);
  if (rc != TQ_OK) return rc;
  if (!dense_scratch) return TQ_ERR_NULL;
  if (!aligned(dense_scratch, 16)) return TQ_ERR_ALIGN;
  const size_t need = tq_dense_scratch_bytes(cache->batch, cache->n_kv_heads, seq_len, cache->head_dim);
  if (dense_scratch_bytes < need) return TQ_ERR_WORKSPACE;
  if (opts && (opts->window > 0 || opts->n_queries > 1)) return TQ_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  half_t* k_dense = static_cast<half_t*>(dense_scratch);
  half_t* v_dense = k_dense + need / sizeof(half_t) / 2;
  rc = hip_rc(tq::launch_dequant_dense(*cache, seq_len, k_dense, v_dense, s));
  if (rc != TQ_OK) return rc;
  // attention over the dense tensors: on the matrix cores where that kernel covers the shape (variant 1 asks for
  // the generic vector-ALU kernel), one block per compute unit and at least a supertile per wave
  const bool on_mfma = !(opts && opts->variant == 1) && attn_scale > 0.0f && std::isfinite(attn_scale) &&
                       tq::dense_mfma_supported(cache->head_dim, n_q_heads / cache->n_kv_heads);
  const Plan plan = on_mfma ? plan_splits(cache->batch, cache->n_kv_heads, seq_len, opts ? opts->n_splits : 0,
                                          kBlocksMfma, tq::dense_mfma_waves(cache->head_dim))
                            : plan_splits(cache->batch, cache->n_kv_heads, seq_len, opts ? opts->n_splits : 0,
                                          kBlocksValu, 1);
  DecodeParams p = make_params(cache, q, n_q_heads, seq_len, attn_scale, out, workspace, plan);
  p.k_dense = k_dense;
  p.v_dense = v_dense;
  p.row_stride = seq_len;                  // the dense buffers are packed to seq_len rows
  rc = hip_rc(on_mfma ? tq::launch_partial_dense_mfma(p, cache->batch, cache->head_dim, s)
                      : tq::launch_partial_valu(p, cache->batch, cache->head_dim, true, s));
  if (rc != TQ_OK) return rc;
  return hip_rc(tq::launch_reduce(p, cache->batch, cache->head_dim, s));
}

}  // extern "C"
