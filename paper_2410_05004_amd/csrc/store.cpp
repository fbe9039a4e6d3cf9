// Host store of saved hidden states in fixed-size token chunks (paper Section 4.2.1),
// and the pipelined whole-context restore that reads it (Section 3.1 pipeline, Section 5
// "Pipelined state transmission").
#include <climits>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>

#include "hcache_internal.h"

using namespace hc;

extern "C" {

hc_status hc_store_create_ex(int32_t n_layers, int32_t d_model, int32_t chunk_tokens,
                             int64_t capacity_chunks, int32_t pinned, hc_store** out) {
  clear_error();
  if (!out) return fail(HC_EINVAL, "out is null");
  *out = nullptr;
  if (n_layers <= 0 || d_model <= 0 || chunk_tokens <= 0 || capacity_chunks <= 0)
    return fail(HC_EINVAL, "store dimensions must be positive");
  if (d_model % 8 != 0) return fail(HC_EINVAL, "d_model must be a multiple of 8 (16-byte rows)");
  hc_store* st = new (std::nothrow) hc_store();
  if (!st) return fail(HC_ENOMEM, "out of host memory");
  st->n_layers = n_layers;
  st->d_model = d_model;
  st->chunk_tokens = chunk_tokens;
  st->capacity_chunks = capacity_chunks;
  st->row_bytes = (size_t)d_model * 2;
  st->chunk_bytes = st->row_bytes * chunk_tokens;
  st->rows_total = capacity_chunks / n_layers;           // whole arena rows (one chunk of every layer)
  if (st->rows_total == 0) {
    delete st;
    return fail(HC_EINVAL, "capacity_chunks must be at least n_layers (one chunk of every layer)");
  }
  st->rows_free = st->rows_total;
  st->free_extents[0] = st->rows_total;
  const size_t bytes = st->chunk_bytes * (size_t)st->rows_total * (size_t)n_layers;
  if (pinned) {
    void* p = nullptr;
    hipError_t e = hipHostMalloc(&p, bytes, hipHostMallocDefault);
    if (e != hipSuccess) {
      delete st;
      (void)hipGetLastError();
      return fail(HC_ENOMEM, std::string("hipHostMalloc of the chunk arena failed: ") +
                                 hipGetErrorString(e));
    }
    st->arena = static_cast<unsigned char*>(p);
    st->pinned = true;
  } else {
    void* p = nullptr;
    if (posix_memalign(&p, 4096, bytes) != 0) {
      delete st;
      return fail(HC_ENOMEM, "allocation of the chunk arena failed");
    }
    st->arena = static_cast<unsigned char*>(p);
  }
  *out = st;
  return HC_OK;
}

hc_status hc_store_create(int32_t n_layers, int32_t d_model, int32_t chunk_tokens,
                          int64_t capacity_chunks, hc_store** out) {
  return hc_store_create_ex(n_layers, d_model, chunk_tokens, capacity_chunks, 1, out);
}

hc_status hc_store_destroy(hc_store* st) {
  clear_error();
  if (!st) return HC_OK;
  if (st->arena) {
    if (st->pinned) (void)hipHostFree(st->arena);
    else free(st->arena);
  }
  delete st;
  return HC_OK;
}

}  // extern "C"

namespace hc {

// ---- arena rows (callers hold the index lock) ----------------------------------------------
static void growth_add(hc_store* st, int64_t row) { st->growth[row] = st->alloc_count; }
static void growth_del(hc_store* st, int64_t row) { st->growth.erase(row); }
static bool growing_into(const hc_store* st, int64_t row) {
  auto it = st->growth.find(row);
  return it != st->growth.end() && st->alloc_count - it->second < kGrowthWindow;
}

// Take one row for a context whose last row is `last` (-1: none yet).
static int64_t take_row(hc_store* st, int64_t last) {
  int64_t row;
  auto it = last >= 0 ? st->free_extents.find(last + 1) : st->free_extents.end();
  if (it == st->free_extents.end()) {
    // new run: the largest free extent; its start unless some context grows into it from below
    it = st->free_extents.begin();
    for (auto e = st->free_extents.begin(); e != st->free_extents.end(); ++e)
      if (e->second > it->second) it = e;
    if (growing_into(st, it->first) && it->second > 1) {
      const int64_t start = it->first, len = it->second, mid = start + len / 2;
      it->second = mid - start;                          // the lower half stays free
      it = st->free_extents.emplace(mid, start + len - mid).first;
    }
  }
  row = it->first;
  const int64_t rest = it->second - 1;
  st->free_extents.erase(it);
  if (rest > 0) st->free_extents[row + 1] = rest;
  --st->rows_free;
  ++st->alloc_count;
  if (last >= 0) growth_del(st, last + 1);
  growth_add(st, row + 1);
  return row;
}

static void give_row(hc_store* st, int64_t row) {
  int64_t start = row, len = 1;
  auto next = st->free_extents.find(row + 1);
  if (next != st->free_extents.end()) {
    len += next->second;
    st->free_extents.erase(next);
  }
  auto prev = st->free_extents.lower_bound(row);
  if (prev != st->free_extents.begin()) {
    --prev;
    if (prev->first + prev->second == row) {
      start = prev->first;
      len += prev->second;
      st->free_extents.erase(prev);
    }
  }
  st->free_extents[start] = len;
  ++st->rows_free;
}

// Index half of an append: under the store's lock, check the order rule and the capacity, take
// arena rows and advance the token count of (seq_id, layer) by n_tok; report where the rows
// go.  The caller copies the payload afterwards (no lock needed: the pieces are its own).
hc_status store_reserve(hc_store* st, int64_t seq_id, int32_t layer, int32_t n_tok,
                        std::vector<StorePiece>& pieces) {
  std::lock_guard<std::mutex> lock(st->index_mutex);
  auto it = st->seqs.find(seq_id);
  const bool fresh_seq = it == st->seqs.end();
  if (fresh_seq) {
    hc_seq_state fresh;
    fresh.chunks.resize(st->n_layers);
    fresh.tokens.assign(st->n_layers, 0);
    it = st->seqs.emplace(seq_id, std::move(fresh)).first;
  }
  hc_seq_state& s = it->second;
  hc_status bad = HC_OK;
  // generation order: a layer never holds more tokens than the layer below it
  if (layer > 0 && s.tokens[layer - 1] < s.tokens[layer] + n_tok)
    bad = fail(HC_ESTATE, "layer appended before the layer below it (layer-before-token order)");
  // make sure the arena can take the whole append before touching anything
  const int64_t chunks_after = (s.tokens[layer] + n_tok + st->chunk_tokens - 1) / st->chunk_tokens;
  const int64_t need_rows = chunks_after > (int64_t)s.rows.size() ? chunks_after - (int64_t)s.rows.size() : 0;
  if (bad == HC_OK && need_rows > st->rows_free) bad = fail(HC_ERANGE, "chunk arena is full");
  if (bad != HC_OK) {
    if (fresh_seq) st->seqs.erase(it);                   // a failed first append leaves no trace
    return bad;
  }

  size_t src_off = 0;
  int32_t left = n_tok;
  while (left > 0) {
    const int64_t fill = s.tokens[layer] % st->chunk_tokens;
    if (fill == 0 && s.tokens[layer] == (int64_t)s.chunks[layer].size() * st->chunk_tokens) {
      const size_t c = s.chunks[layer].size();           // chunk index this layer starts
      if (c >= s.rows.size()) s.rows.push_back(take_row(st, s.rows.empty() ? -1 : s.rows.back()));
      s.chunks[layer].push_back(s.rows[c] * st->n_layers + layer);
    }
    const int64_t room = st->chunk_tokens - fill;
    const int32_t take = left < room ? left : (int32_t)room;
    StorePiece pc;
    pc.dst = st->arena + (size_t)s.chunks[layer].back() * st->chunk_bytes + (size_t)fill * st->row_bytes;
    pc.src_off = src_off;
    pc.bytes = (size_t)take * st->row_bytes;
    pieces.push_back(pc);
    src_off += pc.bytes;
    s.tokens[layer] += take;
    left -= take;
  }
  return HC_OK;
}

}  // namespace hc

extern "C" {

hc_status hc_store_append(hc_store* st, int64_t seq_id, int32_t layer, const void* h_rows,
                          int32_t n_tok) {
  clear_error();
  if (!st) return fail(HC_EINVAL, "store is null");
  if (layer < 0 || layer >= st->n_layers) return fail(HC_ERANGE, "layer out of range");
  if (n_tok < 0) return fail(HC_EINVAL, "negative token count");
  if (n_tok == 0) return HC_OK;
  if (!h_rows) return fail(HC_EINVAL, "rows pointer is null");
  std::vector<StorePiece> pieces;
  hc_status r = store_reserve(st, seq_id, layer, n_tok, pieces);
  if (r != HC_OK) return r;
  const unsigned char* src = static_cast<const unsigned char*>(h_rows);
  for (const StorePiece& pc : pieces) memcpy(pc.dst, src + pc.src_off, pc.bytes);
  return HC_OK;
}

int64_t hc_store_tokens(const hc_store* st, int64_t seq_id, int32_t layer) {
  if (!st || layer < 0 || layer >= st->n_layers) return 0;
  std::lock_guard<std::mutex> lock(st->index_mutex);
  auto it = st->seqs.find(seq_id);
  return it == st->seqs.end() ? 0 : it->second.tokens[layer];
}

hc_status hc_store_chunk(const hc_store* st, int64_t seq_id, int32_t layer, int32_t chunk,
                         const void** h_ptr, int32_t* rows) {
  clear_error();
  if (!st || !h_ptr || !rows) return fail(HC_EINVAL, "null argument");
  if (layer < 0 || layer >= st->n_layers) return fail(HC_ERANGE, "layer out of range");
  std::lock_guard<std::mutex> lock(st->index_mutex);
  auto it = st->seqs.find(seq_id);
  if (it == st->seqs.end()) return fail(HC_ERANGE, "unknown context");
  const hc_seq_state& s = it->second;
  if (chunk < 0 || chunk >= (int64_t)s.chunks[layer].size()) return fail(HC_ERANGE, "no such chunk");
  const int64_t before = (int64_t)chunk * st->chunk_tokens;
  const int64_t r = s.tokens[layer] - before;
  *rows = (int32_t)(r < st->chunk_tokens ? r : st->chunk_tokens);
  *h_ptr = st->arena + (size_t)s.chunks[layer][chunk] * st->chunk_bytes;
  return HC_OK;
}

hc_status hc_store_drop(hc_store* st, int64_t seq_id) {
  clear_error();
  if (!st) return fail(HC_EINVAL, "store is null");
  std::lock_guard<std::mutex> lock(st->index_mutex);
  auto it = st->seqs.find(seq_id);
  if (it == st->seqs.end()) return fail(HC_ERANGE, "unknown context");
  if (!it->second.rows.empty()) hc::growth_del(st, it->second.rows.back() + 1);
  for (int64_t row : it->second.rows) hc::give_row(st, row);
  st->seqs.erase(it);
  return HC_OK;
}

// ---- pieces shared by the pipelined restores ---------------------------------------------
// Two staging buffers of at least need_bytes each, and the events of the two-way handshake.
static hc_status ensure_staging(hc_ctx* ctx, size_t need_bytes, hipStream_t cs) {
  if (ctx->stage_bytes < need_bytes) {
    for (int b = 0; b < 2; ++b) {
      if (ctx->stage[b]) { HC_HIP(hipFree(ctx->stage[b])); ctx->stage[b] = nullptr; }
    }
    ctx->stage_bytes = 0;
    for (int b = 0; b < 2; ++b) {
      hipError_t e = hipMalloc(reinterpret_cast<void**>(&ctx->stage[b]), need_bytes);
      if (e != hipSuccess) {
        (void)hipGetLastError();
        ctx->stage[b] = nullptr;
        return fail(HC_ENOMEM, "device allocation of a staging buffer failed");
      }
    }
    ctx->stage_bytes = need_bytes;
  }
  for (int b = 0; b < 2; ++b) {
    if (!ctx->h2d_done[b]) HC_HIP(hipEventCreateWithFlags(&ctx->h2d_done[b], hipEventDisableTiming));
    if (!ctx->buf_free[b]) {
      HC_HIP(hipEventCreateWithFlags(&ctx->buf_free[b], hipEventDisableTiming));
      HC_HIP(hipEventRecord(ctx->buf_free[b], cs));   // nothing uses the buffer yet
    }
  }
  return HC_OK;
}

static void build_runs(const hc_store* st, const std::vector<int64_t>& chunks, int tok_begin,
                       int n_tok, unsigned char* dst, std::vector<CopyRun>& runs) {
  for_each_run(st, chunks, tok_begin, n_tok, dst, [&](const CopyRun& r) { runs.push_back(r); return true; });
}

static hc_status enqueue_runs(const std::vector<CopyRun>& runs, hipStream_t xs) {
  for (const CopyRun& r : runs) {
    hc_status s = enqueue_run(r, xs);
    if (s != HC_OK) return s;
  }
  return HC_OK;
}

// Shared body of the whole-context restores.  Layers [0, l_h) come from the hidden-state
// store `hs` through the fused kernel; layers [l_h, n_layers) come from the KV-row store `ks`
// (layer index l - l_h there) through the row-to-page copy.  Both kinds go through the same
// two staging buffers and the same event handshake, in layer order, so the hidden states
// stream without a gap and the offloaded KV follows them (paper Section 4.1.2).
static hc_status restore_context_impl(hc_ctx* ctx, const hc_store* hs, const hc_store* ks,
                                      int32_t l_h, int64_t seq_id, int32_t tok_begin,
                                      int32_t n_tok, int32_t pos_offset,
                                      const int32_t* d_block_table, int32_t n_blocks,
                                      void* compute_stream, void* copy_stream) {
  const int L = ctx->desc.n_layers;
  if (tok_begin < 0 || n_tok < 0 || n_blocks < 0) return fail(HC_EINVAL, "negative size");
  if (n_tok == 0) return HC_OK;
  if (!d_block_table) return fail(HC_EINVAL, "block table is null");
  if (compute_stream == copy_stream) return fail(HC_EINVAL, "compute and copy streams must differ");
  // snapshot of the context's chunk lists, taken under each store's lock: appends for other
  // contexts may run on other threads while this call enqueues its copies
  hc_seq_state hcopy, kcopy;
  const hc_seq_state* hseq = nullptr;
  const hc_seq_state* kseq = nullptr;
  if (l_h > 0) {
    std::lock_guard<std::mutex> lock(hs->index_mutex);
    auto it = hs->seqs.find(seq_id);
    if (it == hs->seqs.end()) return fail(HC_ERANGE, "unknown context");
    hcopy.tokens.assign(it->second.tokens.begin(), it->second.tokens.begin() + l_h);
    hcopy.chunks.assign(it->second.chunks.begin(), it->second.chunks.begin() + l_h);
    hseq = &hcopy;
  }
  if (l_h < L) {
    std::lock_guard<std::mutex> lock(ks->index_mutex);
    auto it = ks->seqs.find(seq_id);
    if (it == ks->seqs.end()) return fail(HC_ERANGE, "unknown context in the KV store");
    kcopy = it->second;
    kseq = &kcopy;
  }
  for (int l = 0; l < L; ++l) {
    const int64_t have = l < l_h ? hseq->tokens[l] : kseq->tokens[l - l_h];
    if (have < (int64_t)tok_begin + n_tok)
      return fail(HC_ERANGE, "token range exceeds what the store holds for some layer");
    if ((l < l_h && !ctx->layers[l].wpack) || !ctx->layers[l].pool)
      return fail(HC_ESTATE, "weights or KV pool missing for some layer");
  }
  if ((int64_t)pos_offset + tok_begin + n_tok > ctx->desc.max_position || pos_offset < 0)
    return fail(HC_ERANGE, "positions exceed max_position");
  hipStream_t cs = static_cast<hipStream_t>(compute_stream);
  hipStream_t xs = static_cast<hipStream_t>(copy_stream);

  // staging buffers and events
  size_t need_bytes = 0;
  if (l_h > 0) need_bytes = (size_t)n_tok * hs->row_bytes;
  if (l_h < L && (size_t)n_tok * ks->row_bytes > need_bytes) need_bytes = (size_t)n_tok * ks->row_bytes;
  {
    hc_status r = ensure_staging(ctx, need_bytes, cs);
    if (r != HC_OK) return r;
  }

  // Segments: one per run of equally spaced chunks of a layer.  Chunks that arrive in
  // generation order are spaced n_layers slots apart (or adjacent after a long prefill), so a
  // whole layer is usually a single run: one strided copy.
  std::vector<CopyRun> runs;
  std::vector<CopySegment> segs;                        // host scratch
  auto build = [&](const hc_store* st, const hc_seq_state& s, int l, int b) {
    const int CT = st->chunk_tokens;
    const int c_first = tok_begin / CT, c_last = (tok_begin + n_tok - 1) / CT;
    unsigned char* stage = reinterpret_cast<unsigned char*>(ctx->stage[b]);
    runs.clear();
    segs.clear();
    for (int c = c_first; c <= c_last; ++c) {           // one segment per chunk (gather kernel)
      const int lo = c == c_first ? tok_begin - c * CT : 0;
      const int hi = c == c_last ? tok_begin + n_tok - c * CT : CT;
      CopySegment g;
      g.src = st->arena + (size_t)s.chunks[l][c] * st->chunk_bytes + (size_t)lo * st->row_bytes;
      g.dst = stage + (size_t)(c * CT + lo - tok_begin) * st->row_bytes;
      g.bytes = (size_t)(hi - lo) * st->row_bytes;
      segs.push_back(g);
    }
    build_runs(st, s.chunks[l], tok_begin, n_tok, stage, runs);
  };

  // The gather kernel needs device-readable arenas and reads its segment table from pinned
  // host memory; a pageable arena goes through the copy calls.
  const bool use_gather = ctx->loader_mode == 1 && (l_h == 0 || hs->pinned) && (l_h == L || ks->pinned);
  CopySegment* tab = nullptr;
  size_t tab_used = 0;
  int tab_id = 0;
  if (use_gather) {
    tab_id = ctx->seg_next;
    ctx->seg_next ^= 1;
    size_t need = 0;
    if (l_h > 0) need += (size_t)l_h * (size_t)((tok_begin + n_tok - 1) / hs->chunk_tokens - tok_begin / hs->chunk_tokens + 1);
    if (l_h < L) need += (size_t)(L - l_h) * (size_t)((tok_begin + n_tok - 1) / ks->chunk_tokens - tok_begin / ks->chunk_tokens + 1);
    if (!ctx->seg_done[tab_id]) HC_HIP(hipEventCreateWithFlags(&ctx->seg_done[tab_id], hipEventDisableTiming));
    else HC_HIP(hipEventSynchronize(ctx->seg_done[tab_id]));   // kernels of an earlier call still reading it
    if (ctx->seg_cap[tab_id] < need) {
      if (ctx->seg_tab[tab_id]) { HC_HIP(hipHostFree(ctx->seg_tab[tab_id])); ctx->seg_tab[tab_id] = nullptr; }
      ctx->seg_cap[tab_id] = 0;
      void* p = nullptr;
      hipError_t e = hipHostMalloc(&p, need * sizeof(CopySegment), hipHostMallocDefault);
      if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(HC_ENOMEM, "pinned allocation of the segment table failed");
      }
      ctx->seg_tab[tab_id] = static_cast<CopySegment*>(p);
      ctx->seg_cap[tab_id] = need;
    }
    tab = ctx->seg_tab[tab_id];
  }

  // Copy-engine transfers of odd layers go to a second copy stream the context owns: every
  // transfer has a fixed cost of 15-26 us, and with two streams the fixed cost of one layer's
  // transfer overlaps the other layer's bytes (the two staging buffers and their events already
  // order everything else).  8192 tokens of the Llama-3-8B shape: 38.35 -> 38.21 ms; 512 tokens:
  // 3.00 -> 2.69 ms.
  if (!use_gather && !ctx->copy2) HC_HIP(hipStreamCreateWithFlags(&ctx->copy2, hipStreamNonBlocking));
  hipStream_t xs_caller = xs;
  for (int l = 0; l < L; ++l) {
    const int b = l & 1;
    xs = (b && !use_gather) ? ctx->copy2 : xs_caller;
    const bool from_hidden = l < l_h;
    if (from_hidden) build(hs, *hseq, l, b);
    else build(ks, *kseq, l - l_h, b);
    // the kernel that last read stage[b] (two layers ago, or a previous call) must be done
    HC_HIP(hipStreamWaitEvent(xs, ctx->buf_free[b], 0));
    if (use_gather) {
      memcpy(tab + tab_used, segs.data(), segs.size() * sizeof(CopySegment));
      HC_HIP(launch_gather(tab + tab_used, (int)segs.size(), xs));
      tab_used += segs.size();
    } else {
      hc_status r = enqueue_runs(runs, xs);
      if (r != HC_OK) return r;
    }
    HC_HIP(hipEventRecord(ctx->h2d_done[b], xs));
    HC_HIP(hipStreamWaitEvent(cs, ctx->h2d_done[b], 0));
    hc_status r = from_hidden
        ? restore_layer(ctx, l, ctx->stage[b], nullptr, pos_offset + tok_begin, n_tok, nullptr, 1,
                        d_block_table, n_blocks, cs)
        : kv_rows_layer(ctx, l, ctx->stage[b], nullptr, pos_offset + tok_begin, n_tok,
                        d_block_table, n_blocks, true, cs);
    if (r != HC_OK) return r;
    HC_HIP(hipEventRecord(ctx->buf_free[b], cs));
  }
  xs = xs_caller;
  if (use_gather) HC_HIP(hipEventRecord(ctx->seg_done[tab_id], xs));
  return HC_OK;
}

hc_status hc_restore_context(hc_ctx* ctx, const hc_store* st, int64_t seq_id, int32_t tok_begin,
                             int32_t n_tok, int32_t pos_offset, const int32_t* d_block_table,
                             int32_t n_blocks, void* compute_stream, void* copy_stream) {
  clear_error();
  if (!ctx || !st) return fail(HC_EINVAL, "null ctx or store");
  if (st->n_layers != ctx->desc.n_layers || st->d_model != ctx->desc.d_model)
    return fail(HC_EINVAL, "store and context disagree on n_layers / d_model");
  return restore_context_impl(ctx, st, nullptr, ctx->desc.n_layers, seq_id, tok_begin, n_tok,
                              pos_offset, d_block_table, n_blocks, compute_stream, copy_stream);
}

hc_status hc_poison_staging(hc_ctx* ctx, void* compute_stream) {
  clear_error();
  if (!ctx) return fail(HC_EINVAL, "null ctx");
  if (!ctx->stage[0] || !ctx->stage[1] || !ctx->buf_free[0] || !ctx->buf_free[1])
    return fail(HC_ESTATE, "the context has no staging buffers yet");
  hipStream_t cs = static_cast<hipStream_t>(compute_stream);
  for (int b = 0; b < 2; ++b) {
    // after every kernel queued on the stream so far; the next restore's copies wait for it
    HC_HIP(hipMemsetD16Async(reinterpret_cast<hipDeviceptr_t>(ctx->stage[b]), 0x7FFF, ctx->stage_bytes / 2, cs));
    HC_HIP(hipEventRecord(ctx->buf_free[b], cs));
  }
  return HC_OK;
}

hc_status hc_restore_contexts(hc_ctx* ctx, const hc_store* st, int32_t n_seq,
                              const int64_t* h_seq_ids, const int32_t* h_n_tok,
                              const int32_t* d_block_tables, int32_t max_blocks,
                              void* compute_stream, void* copy_stream) {
  clear_error();
  if (!ctx || !st) return fail(HC_EINVAL, "null ctx or store");
  if (st->n_layers != ctx->desc.n_layers || st->d_model != ctx->desc.d_model)
    return fail(HC_EINVAL, "store and context disagree on n_layers / d_model");
  if (n_seq < 0 || max_blocks < 0) return fail(HC_EINVAL, "negative size");
  if (n_seq == 0) return HC_OK;
  if (!h_seq_ids || !h_n_tok || !d_block_tables) return fail(HC_EINVAL, "null pointer");
  if (compute_stream == copy_stream) return fail(HC_EINVAL, "compute and copy streams must differ");
  const int L = ctx->desc.n_layers;
  // snapshot of every context's chunk lists under the store's lock; row offsets
  std::vector<hc_seq_state> snap(n_seq);
  std::vector<int32_t> cu(n_seq + 1, 0);
  {
    std::lock_guard<std::mutex> lock(st->index_mutex);
    for (int i = 0; i < n_seq; ++i) {
      if (h_n_tok[i] < 0) return fail(HC_EINVAL, "negative token count");
      if (h_n_tok[i] > ctx->desc.max_position) return fail(HC_ERANGE, "positions exceed max_position");
      if ((int64_t)cu[i] + h_n_tok[i] > INT32_MAX) return fail(HC_ERANGE, "more than 2^31 rows");
      cu[i + 1] = cu[i] + h_n_tok[i];
      if (h_n_tok[i] == 0) continue;
      auto it = st->seqs.find(h_seq_ids[i]);
      if (it == st->seqs.end()) return fail(HC_ERANGE, "unknown context");
      for (int l = 0; l < L; ++l)
        if (it->second.tokens[l] < h_n_tok[i])
          return fail(HC_ERANGE, "token range exceeds what the store holds for some layer");
      snap[i] = it->second;
    }
  }
  const int32_t total = cu[n_seq];
  if (total == 0) return HC_OK;
  for (int l = 0; l < L; ++l)
    if (!ctx->layers[l].wpack || !ctx->layers[l].pool)
      return fail(HC_ESTATE, "weights or KV pool missing for some layer");
  hipStream_t cs = static_cast<hipStream_t>(compute_stream);
  hipStream_t xs = static_cast<hipStream_t>(copy_stream);
  hc_status r = ensure_staging(ctx, (size_t)total * st->row_bytes, cs);
  if (r != HC_OK) return r;

  // row offsets on the device: one of two tables, reused only after its last reader is done
  const int tab = ctx->cu_next;
  ctx->cu_next ^= 1;
  if (!ctx->cu_done[tab]) HC_HIP(hipEventCreateWithFlags(&ctx->cu_done[tab], hipEventDisableTiming));
  else HC_HIP(hipEventSynchronize(ctx->cu_done[tab]));
  if (ctx->cu_cap[tab] < n_seq + 1) {
    if (ctx->cu_host[tab]) { HC_HIP(hipHostFree(ctx->cu_host[tab])); ctx->cu_host[tab] = nullptr; }
    if (ctx->cu_dev[tab]) { HC_HIP(hipFree(ctx->cu_dev[tab])); ctx->cu_dev[tab] = nullptr; }
    ctx->cu_cap[tab] = 0;
    void* p = nullptr;
    if (hipHostMalloc(&p, (size_t)(n_seq + 1) * sizeof(int32_t), hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      return fail(HC_ENOMEM, "pinned allocation of the row-offset table failed");
    }
    ctx->cu_host[tab] = static_cast<int32_t*>(p);
    if (hipMalloc(reinterpret_cast<void**>(&ctx->cu_dev[tab]), (size_t)(n_seq + 1) * sizeof(int32_t)) != hipSuccess) {
      (void)hipGetLastError();
      return fail(HC_ENOMEM, "device allocation of the row-offset table failed");
    }
    ctx->cu_cap[tab] = n_seq + 1;
  }
  memcpy(ctx->cu_host[tab], cu.data(), (size_t)(n_seq + 1) * sizeof(int32_t));
  HC_HIP(hipMemcpyAsync(ctx->cu_dev[tab], ctx->cu_host[tab], (size_t)(n_seq + 1) * sizeof(int32_t),
                        hipMemcpyHostToDevice, cs));

  std::vector<CopyRun> runs;
  for (int l = 0; l < L; ++l) {
    const int b = l & 1;
    unsigned char* stage = reinterpret_cast<unsigned char*>(ctx->stage[b]);
    runs.clear();
    for (int i = 0; i < n_seq; ++i)
      if (h_n_tok[i] > 0)
        build_runs(st, snap[i].chunks[l], 0, h_n_tok[i], stage + (size_t)cu[i] * st->row_bytes, runs);
    HC_HIP(hipStreamWaitEvent(xs, ctx->buf_free[b], 0));
    r = enqueue_runs(runs, xs);
    if (r != HC_OK) return r;
    HC_HIP(hipEventRecord(ctx->h2d_done[b], xs));
    HC_HIP(hipStreamWaitEvent(cs, ctx->h2d_done[b], 0));
    // positions are implied: row t of context i sits at position t - cu[i]
    r = restore_layer(ctx, l, ctx->stage[b], nullptr, 0, total, ctx->cu_dev[tab], n_seq, d_block_tables,
                      max_blocks, cs);
    if (r != HC_OK) return r;
    HC_HIP(hipEventRecord(ctx->buf_free[b], cs));
  }
  HC_HIP(hipEventRecord(ctx->cu_done[tab], cs));
  return HC_OK;
}

hc_status hc_restore_context_mixed(hc_ctx* ctx, const hc_store* hidden_store,
                                   const hc_store* kv_store, int32_t l_h, int64_t seq_id,
                                   int32_t tok_begin, int32_t n_tok, int32_t pos_offset,
                                   const int32_t* d_block_table, int32_t n_blocks,
                                   void* compute_stream, void* copy_stream) {
  clear_error();
  if (!ctx) return fail(HC_EINVAL, "null ctx");
  const int L = ctx->desc.n_layers;
  if (l_h < 0 || l_h > L) return fail(HC_ERANGE, "l_h outside [0, n_layers]");
  if (l_h > 0) {
    if (!hidden_store) return fail(HC_EINVAL, "hidden-state store is null");
    if (hidden_store->n_layers < l_h || hidden_store->d_model != ctx->desc.d_model)
      return fail(HC_EINVAL, "hidden-state store has fewer than l_h layers or another d_model");
  }
  if (l_h < L) {
    if (!kv_store) return fail(HC_EINVAL, "KV store is null");
    if (kv_store->n_layers != L - l_h || kv_store->d_model != 2 * ctx->d_kv)
      return fail(HC_EINVAL, "KV store must hold n_layers - l_h layers of 2 * d_kv wide rows");
  }
  return restore_context_impl(ctx, hidden_store, kv_store, l_h, seq_id, tok_begin, n_tok,
                              pos_offset, d_block_table, n_blocks, compute_stream, copy_stream);
}

}  // extern "C"
