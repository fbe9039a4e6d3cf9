// hc_restore_context_static: the pipelined whole-context restore for callers that cannot
// allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  Same loader, same kernel and same event handshake as hc_restore_context; the
// two staging buffers are halves of a device-resident array of this file instead of hipMalloc'd
// memory, and the handshake events are created once per device at set-up.
#include <climits>
#include <mutex>

#include "hcache_internal.h"

using namespace hc;

// Two staging buffers of HC_STATIC_STAGE_BYTES each.  Every GPU the library runs on holds its
// own copy of the array until the process ends.
static __device__ __align__(256) unsigned char scratch[2 * HC_STATIC_STAGE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
constexpr int kMaxRunsPerLayer = 256;   // copy-engine transfers of one layer (stack array)

// Per-device state, filled once by static_scratch_init with that device current.  In host
// code the array's name is only a stand-in, so everything below works with `ptr`, the
// array's address on that device as the runtime reports it.
struct DeviceScratch {
  unsigned char* ptr = nullptr;
  hipEvent_t h2d_done[2] = {nullptr, nullptr};   // copy stream -> compute stream
  hipEvent_t buf_free[2] = {nullptr, nullptr};   // compute stream -> copy stream
  bool free_recorded[2] = {false, false};
  bool ready = false;
};
DeviceScratch g_dev[kMaxDevices];
std::mutex g_mutex;                               // set-up, and one static restore at a time

}  // namespace

namespace hc {

hc_status static_scratch_init() {
  int dev = 0;
  HC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(HC_ERANGE, "device index beyond the static scratch table");
  std::lock_guard<std::mutex> lock(g_mutex);
  DeviceScratch& D = g_dev[dev];
  if (D.ready) return HC_OK;
  void* p = nullptr;
  HC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
  if (!p || (reinterpret_cast<uintptr_t>(p) & 255u) != 0)
    return fail(HC_EHIP, "address of the static scratch array is null or misaligned");
  D.ptr = static_cast<unsigned char*>(p);
  for (int b = 0; b < 2; ++b) {
    if (!D.h2d_done[b]) HC_HIP(hipEventCreateWithFlags(&D.h2d_done[b], hipEventDisableTiming));
    if (!D.buf_free[b]) HC_HIP(hipEventCreateWithFlags(&D.buf_free[b], hipEventDisableTiming));
  }
  D.ready = true;
  return HC_OK;
}

}  // namespace hc

extern "C" {

int64_t hc_static_stage_bytes(void) { return HC_STATIC_STAGE_BYTES; }

hc_status hc_restore_context_static(hc_ctx* ctx, const hc_store* st, int64_t seq_id,
                                    int32_t tok_begin, int32_t n_tok, int32_t pos_offset,
                                    const int32_t* d_block_table, int32_t n_blocks,
                                    void* compute_stream, void* copy_stream) {
  clear_error();
  if (!ctx || !st) return fail(HC_EINVAL, "null ctx or store");
  const int L = ctx->desc.n_layers;
  if (st->n_layers != L || st->d_model != ctx->desc.d_model)
    return fail(HC_EINVAL, "store and context disagree on n_layers / d_model");
  if (tok_begin < 0 || n_tok < 0 || n_blocks < 0) return fail(HC_EINVAL, "negative size");
  if (n_tok == 0) return HC_OK;
  if (!d_block_table) return fail(HC_EINVAL, "block table is null");
  if (compute_stream == copy_stream) return fail(HC_EINVAL, "compute and copy streams must differ");
  if ((uint64_t)n_tok * st->row_bytes > (uint64_t)HC_STATIC_STAGE_BYTES)
    return fail(HC_ERANGE, "n_tok * d_model * 2 bytes exceeds HC_STATIC_STAGE_BYTES, the size of a "
                           "static staging buffer; use hc_restore_context or restore in pieces");
  if (pos_offset < 0 || (int64_t)pos_offset + tok_begin + n_tok > ctx->desc.max_position)
    return fail(HC_ERANGE, "positions exceed max_position");
  if (ctx->timing) return fail(HC_ESTATE, "per-launch timing creates events; end it before this call");
  if (ctx->device < 0 || ctx->device >= kMaxDevices || !g_dev[ctx->device].ready)
    return fail(HC_ESTATE, "static scratch of the context's device was not set up");
  for (int l = 0; l < L; ++l)
    if (!ctx->layers[l].wpack || !ctx->layers[l].pool)
      return fail(HC_ESTATE, "weights or KV pool missing for some layer");
  hipStream_t cs = static_cast<hipStream_t>(compute_stream);
  hipStream_t xs = static_cast<hipStream_t>(copy_stream);

  // One static restore at a time per process: the array is shared by every context of a GPU.
  std::lock_guard<std::mutex> call_lock(g_mutex);
  DeviceScratch& D = g_dev[ctx->device];
  // The context's chunk lists are read in place under the store's lock (a snapshot would
  // allocate); appends for other contexts wait for the few enqueue calls below.
  std::lock_guard<std::mutex> index_lock(st->index_mutex);
  auto it = st->seqs.find(seq_id);
  if (it == st->seqs.end()) return fail(HC_ERANGE, "unknown context");
  const hc_seq_state& seq = it->second;
  for (int l = 0; l < L; ++l)
    if (seq.tokens[l] < (int64_t)tok_begin + n_tok)
      return fail(HC_ERANGE, "token range exceeds what the store holds for some layer");

  CopyRun runs[kMaxRunsPerLayer];
  for (int l = 0; l < L; ++l) {
    const int b = l & 1;
    unsigned char* stage = D.ptr + (size_t)b * HC_STATIC_STAGE_BYTES;
    int n_runs = 0;
    const bool all = for_each_run(st, seq.chunks[l], tok_begin, n_tok, stage, [&](const CopyRun& r) {
      if (n_runs == kMaxRunsPerLayer) return false;
      runs[n_runs++] = r;
      return true;
    });
    if (!all) return fail(HC_ERANGE, "a layer's chunks need more than 256 copy-engine transfers");
    // the kernel that last read this half (two layers ago, or an earlier call on any stream)
    // must be done before the copy engines overwrite it
    if (D.free_recorded[b]) HC_HIP(hipStreamWaitEvent(xs, D.buf_free[b], 0));
    for (int i = 0; i < n_runs; ++i) {
      hc_status r = enqueue_run(runs[i], xs);
      if (r != HC_OK) return r;
    }
    HC_HIP(hipEventRecord(D.h2d_done[b], xs));
    HC_HIP(hipStreamWaitEvent(cs, D.h2d_done[b], 0));
    hc_status r = restore_layer(ctx, l, stage, nullptr, pos_offset + tok_begin, n_tok, nullptr, 1,
                                d_block_table, n_blocks, cs);
    if (r != HC_OK) return r;
    HC_HIP(hipEventRecord(D.buf_free[b], cs));
    D.free_recorded[b] = true;
  }
  return HC_OK;
}

}  // extern "C"
