// Host-side plumbing of liba3: status strings, per-thread error text, layout validation,
// workspace sizing, and the staging of chunk caches from host memory.  No kernels here.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "a3_internal.h"

#include <errno.h>
#include <unistd.h>

#include <atomic>
#include <thread>
#include <vector>

static thread_local char g_last_error[512] = "";

static std::atomic<int> g_knobs[A3_KNOB_COUNT] = {{-1}, {-1}, {-1}, {-1}, {-1}, {-1}};
static const char *const kKnobNames[A3_KNOB_COUNT] = {"attn_wgs", "attn_item_cost", "proj_ntw", "proj_k64", "gemm_tb", "gemm_k64"};

int a3_knob(int which) { return g_knobs[which].load(std::memory_order_relaxed); }

extern "C" a3_status a3_set_tuning(const char *name, int value) {
  A3_REQUIRE(name != nullptr, A3_ERR_INVALID_ARG, "a3_set_tuning: name is NULL");
  for (int i = 0; i < A3_KNOB_COUNT; ++i)
    if (strcmp(name, kKnobNames[i]) == 0) {
      g_knobs[i].store(value < 0 ? -1 : value, std::memory_order_relaxed);
      return A3_OK;
    }
  return a3_fail(A3_ERR_INVALID_ARG, "a3_set_tuning: unknown name '%s'", name);
}

a3_status a3_fail(a3_status code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
  va_end(ap);
  return code;
}

a3_status a3_check_layout(const a3_layout *L, const char *who, bool need_tables) {
  A3_REQUIRE(L != nullptr, A3_ERR_INVALID_ARG, "%s: layout is NULL", who);
  A3_REQUIRE(L->dtype == A3_F32 || L->dtype == A3_BF16, A3_ERR_INVALID_ARG, "%s: unknown dtype %d", who, L->dtype);
  A3_REQUIRE(L->rope_layout == A3_ROPE_INTERLEAVED || L->rope_layout == A3_ROPE_HALF, A3_ERR_INVALID_ARG,
             "%s: unknown rope_layout %d", who, L->rope_layout);
  A3_REQUIRE(L->n_q_heads > 0 && L->n_kv_heads > 0 && L->hidden > 0, A3_ERR_INVALID_ARG,
             "%s: head counts and hidden must be positive", who);
  A3_REQUIRE(L->n_q_heads % L->n_kv_heads == 0, A3_ERR_INVALID_ARG,
             "%s: n_q_heads %d is not a multiple of n_kv_heads %d", who, L->n_q_heads, L->n_kv_heads);
  A3_REQUIRE(L->head_dim == 64 || L->head_dim == 128, A3_ERR_UNSUPPORTED, "%s: head_dim %d (64 or 128 only)", who,
             L->head_dim);
  A3_REQUIRE(L->dtype != A3_BF16 || L->head_dim == 128, A3_ERR_UNSUPPORTED,
             "%s: bf16 kernels need head_dim 128, got %d", who, L->head_dim);
  A3_REQUIRE(L->hidden % 32 == 0, A3_ERR_UNSUPPORTED, "%s: hidden %d is not a multiple of 32", who, L->hidden);
  A3_REQUIRE(L->n_q_heads / L->n_kv_heads <= 16, A3_ERR_UNSUPPORTED, "%s: more than 16 query heads per KV head", who);
  A3_REQUIRE(L->rope_base > 1.0, A3_ERR_INVALID_ARG, "%s: rope_base must be > 1", who);
  A3_REQUIRE(L->sm_scale >= 0.f, A3_ERR_INVALID_ARG, "%s: sm_scale must be >= 0", who);
  A3_REQUIRE(L->n_req > 0 && L->n_chunks >= 0 && L->total_tokens > 0, A3_ERR_INVALID_ARG,
             "%s: n_req/total_tokens must be positive", who);
  A3_REQUIRE(L->max_ctx_len >= 0 && L->max_q_len >= 0 && L->max_ctx_len + L->max_q_len > 0, A3_ERR_INVALID_ARG,
             "%s: max_ctx_len/max_q_len invalid", who);
  A3_REQUIRE((long long)L->max_ctx_len + L->max_q_len <= L->total_tokens, A3_ERR_INVALID_ARG,
             "%s: max_ctx_len + max_q_len exceeds total_tokens", who);
  A3_REQUIRE(L->seg_start && L->ctx_len && L->q_len, A3_ERR_INVALID_ARG, "%s: seg_start/ctx_len/q_len is NULL", who);
  A3_REQUIRE(L->n_chunks == 0 || (L->chunk_start && L->chunk_len && L->chunk_delta), A3_ERR_INVALID_ARG,
             "%s: chunk arrays are NULL", who);
  if (need_tables) {
    A3_REQUIRE(L->tok_pos && L->tok_req && L->tok_chunk && L->q_start && L->rope_pos_cs, A3_ERR_INVALID_ARG,
               "%s: derived tables are NULL (allocate them and call a3_layout_prepare)", who);
    A3_REQUIRE(L->n_chunks == 0 || L->rope_chunk_cs, A3_ERR_INVALID_ARG, "%s: rope_chunk_cs is NULL", who);
  }
  return A3_OK;
}

extern "C" const char *a3_strerror(a3_status s) {
  switch (s) {
    case A3_OK: return "ok";
    case A3_ERR_INVALID_ARG: return "invalid argument";
    case A3_ERR_UNSUPPORTED: return "unsupported shape or type";
    case A3_ERR_WORKSPACE: return "workspace too small";
    case A3_ERR_HIP: return "HIP launch failed";
    case A3_ERR_IO: return "file read failed";
  }
  return "unknown status";
}

extern "C" const char *a3_last_error(void) { return g_last_error; }

// Eq. 3, p = r * n: recomputed context tokens of a request with n_ctx context tokens at ratio num / den, rounded
// down, in integer arithmetic.
extern "C" int a3_recompute_count(int n_ctx, int ratio_num, int ratio_den) {
  if (n_ctx < 0 || ratio_num < 0 || ratio_den <= 0 || ratio_num > ratio_den) {
    a3_fail(A3_ERR_INVALID_ARG, "a3_recompute_count: n_ctx %d, ratio %d / %d", n_ctx, ratio_num, ratio_den);
    return -1;
  }
  return (int)(((long long)n_ctx * ratio_num) / ratio_den);
}

// sel_start for a3_select_chunk_edges: request r holds, per chunk, min(chunk_len, n_head + n_tail) rows.  Host arrays.
extern "C" a3_status a3_chunk_edge_sel_start(int n_req, const int *seg_start, const int *ctx_len, int n_chunks,
                                             const int *chunk_start, const int *chunk_len, int n_head, int n_tail,
                                             int *sel_start) {
  A3_REQUIRE(n_req >= 0 && n_chunks >= 0 && n_head >= 0 && n_tail >= 0, A3_ERR_INVALID_ARG,
             "a3_chunk_edge_sel_start: negative count");
  A3_REQUIRE(sel_start && (n_req == 0 || (seg_start && ctx_len)) && (n_chunks == 0 || (chunk_start && chunk_len)),
             A3_ERR_INVALID_ARG, "a3_chunk_edge_sel_start: NULL argument");
  long long run = 0;
  sel_start[0] = 0;
  for (int r = 0; r < n_req; ++r) {
    const long long lo = seg_start[r], hi = lo + ctx_len[r];
    for (int c = 0; c < n_chunks; ++c)
      if (chunk_start[c] >= lo && chunk_start[c] < hi) {
        const long long edge = (long long)n_head + n_tail;
        run += chunk_len[c] < edge ? chunk_len[c] : edge;
      }
    A3_REQUIRE(run < (1LL << 31), A3_ERR_UNSUPPORTED, "a3_chunk_edge_sel_start: too many rows");
    sel_start[r + 1] = (int)run;
  }
  return A3_OK;
}
extern "C" int a3_version(void) { return A3_VERSION; }

extern "C" size_t a3_workspace_bytes(const a3_layout *L, int max_active_rows) {
  if (a3_check_layout(L, "a3_workspace_bytes", false) != A3_OK || max_active_rows < 0) return 0;
  size_t a = a3_scores_ws_bytes(L);
  size_t b = a3_attn_ws_bytes(L, max_active_rows);
  return (a > b ? a : b) + 256;
}

// The per-chunk K/V store of Eq. 1 lives outside the GPU (the paper keeps it on persistent storage and names
// its loading cost as the method's limitation).  One layer's chunks go from host memory into their packed
// slots of the concatenated cache as asynchronous copies on the caller's stream: with pinned host blocks and
// a stream of its own they run beside the kernels of the previous layer.
extern "C" a3_status a3_chunk_cache_load(const a3_layout *L, const int *chunk_start_host, const int *chunk_len_host,
                                         int n_chunks, const void *const *host_k, const void *const *host_v,
                                         void *k_cat, void *v_cat, void *stream) {
  a3_status s = a3_check_layout(L, "a3_chunk_cache_load", false);
  if (s != A3_OK) return s;
  A3_REQUIRE(n_chunks >= 0, A3_ERR_INVALID_ARG, "a3_chunk_cache_load: n_chunks %d is negative", n_chunks);
  if (n_chunks == 0) return A3_OK;
  A3_REQUIRE(chunk_start_host && chunk_len_host && host_k && host_v && k_cat && v_cat, A3_ERR_INVALID_ARG,
             "a3_chunk_cache_load: NULL argument");
  const size_t row_bytes = (size_t)L->n_kv_heads * L->head_dim * (L->dtype == A3_BF16 ? 2 : 4);
  for (int c = 0; c < n_chunks; ++c) {
    const int start = chunk_start_host[c], len = chunk_len_host[c];
    A3_REQUIRE(len >= 0 && start >= 0 && (long long)start + len <= L->total_tokens, A3_ERR_INVALID_ARG,
               "a3_chunk_cache_load: chunk %d covers rows [%d, %d) outside [0, %d)", c, start, start + len,
               L->total_tokens);
    A3_REQUIRE(len == 0 || (host_k[c] && host_v[c]), A3_ERR_INVALID_ARG, "a3_chunk_cache_load: chunk %d has no host block", c);
  }
  hipStream_t st = (hipStream_t)stream;
  for (int c = 0; c < n_chunks; ++c) {
    const size_t bytes = (size_t)chunk_len_host[c] * row_bytes, off = (size_t)chunk_start_host[c] * row_bytes;
    if (bytes == 0) continue;
    hipError_t e = hipMemcpyAsync((char *)k_cat + off, host_k[c], bytes, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync((char *)v_cat + off, host_v[c], bytes, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return a3_fail(A3_ERR_HIP, "a3_chunk_cache_load: chunk %d: %s", c, hipGetErrorString(e));
  }
  return A3_OK;
}

// The chunk store itself sits on persistent storage (Eq. 1; the paper names loading it as the method's
// limitation).  One layer's blocks are read from already opened files into host staging buffers (pinned ones, so
// that a3_chunk_cache_load / a3_chunk_cache_load_q8 can copy them on asynchronously): block c is n_bytes[c]
// bytes at file_offset[c] of descriptor fds[c].  Plain positional reads, continued after short reads, spread
// over up to n_threads threads by block; the call returns when every block is in memory.  No GPU call.
extern "C" a3_status a3_chunk_file_read(int n_blocks, const int *fds, const long long *file_offset,
                                        const size_t *n_bytes, void *const *host_dst, int n_threads) {
  A3_REQUIRE(n_blocks >= 0, A3_ERR_INVALID_ARG, "a3_chunk_file_read: n_blocks %d is negative", n_blocks);
  if (n_blocks == 0) return A3_OK;
  A3_REQUIRE(fds && file_offset && n_bytes && host_dst, A3_ERR_INVALID_ARG, "a3_chunk_file_read: NULL argument");
  for (int c = 0; c < n_blocks; ++c) {
    A3_REQUIRE(fds[c] >= 0 && file_offset[c] >= 0, A3_ERR_INVALID_ARG,
               "a3_chunk_file_read: block %d: descriptor %d, offset %lld", c, fds[c], file_offset[c]);
    A3_REQUIRE(n_bytes[c] == 0 || host_dst[c], A3_ERR_INVALID_ARG, "a3_chunk_file_read: block %d has no destination", c);
  }
  std::atomic<int> next(0), failed_block(-1), failed_errno(0);
  auto work = [&]() {
    for (int c = next.fetch_add(1); c < n_blocks; c = next.fetch_add(1)) {
      size_t done = 0;
      while (done < n_bytes[c]) {
        const ssize_t r = pread(fds[c], (char *)host_dst[c] + done, n_bytes[c] - done, (off_t)(file_offset[c] + (long long)done));
        if (r > 0) { done += (size_t)r; continue; }
        if (r < 0 && errno == EINTR) continue;
        int expected = -1;                                     // r == 0: the file ends inside the block
        if (failed_block.compare_exchange_strong(expected, c)) failed_errno.store(r < 0 ? errno : 0);
        break;
      }
    }
  };
  const int nt = n_threads < 1 ? 1 : (n_threads > 16 ? 16 : n_threads);
  std::vector<std::thread> pool;
  for (int t = 1; t < nt && t < n_blocks; ++t) pool.emplace_back(work);
  work();
  for (auto &t : pool) t.join();
  if (failed_block.load() >= 0) {
    const int e = failed_errno.load();
    return a3_fail(A3_ERR_IO, "a3_chunk_file_read: block %d: %s", failed_block.load(),
                   e ? strerror(e) : "the file ends inside the block");
  }
  return A3_OK;
}
