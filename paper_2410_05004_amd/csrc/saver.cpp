// Two-stage saving of newly generated hidden states (paper Section 4.2.2; Section 5,
// "Pipelined state transmission" and "Storage management").
//
// Stage 1 (GPU side): the hidden states of one layer for the whole batch -- rows of several
// contexts under continuous batching -- are snapshot to pinned host memory with ONE
// device->host copy on a downstream stream; an event lets the compute stream reuse the
// activation buffer as soon as the copy has read it.
// Stage 2 (host side): daemon threads pick the snapshot up once its copy has completed and
// append every row to the chunk list of its (context, layer) in the store, so the small
// scattered writes never touch the GPU's critical path.
//
// Ordering and balance: the index half of the append (order rule, capacity, chunk slots) is
// done by the producer inside the save call, in call order, so errors surface there and the
// daemons never contend on per-context state.  What is queued is a list of contiguous pieces
// (destination in the arena, offset in the snapshot); piece i is copied by daemon thread
// i mod n_threads once the snapshot's copy event has fired, so a long prefill of a single
// context is spread over all threads just like a decode step of many contexts.
#include <atomic>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <memory>
#include <new>
#include <thread>

#include "hcache_internal.h"

using namespace hc;

namespace {

// rows of one context that fill at least this much of a chunk in one piece are copied from the
// device straight into the arena; smaller pieces go through the snapshot slot and the daemons
constexpr size_t kDirectMinBytes = 64 * 1024;

struct SaveJob {
  int slot = -1;
  std::vector<StorePiece> pieces;    // where the rows go; src_off is relative to the slot
  hipEvent_t copied = nullptr;      // null: rows were already on the host
  std::atomic<int> workers_left{0};
};

}  // namespace

struct hc_saver {
  hc_store* store = nullptr;
  int32_t max_rows = 0, n_slots = 0, n_threads = 0;
  int device = -1;                  // -1: created without a GPU (host rows only)
  size_t row_bytes = 0;
  std::vector<unsigned char*> slot_buf;
  std::vector<bool> slot_pinned;
  std::vector<hipEvent_t> ev_ready;   // recorded on the compute stream, waited by the downstream stream
  std::vector<hipEvent_t> ev_copied;  // recorded on the downstream stream after the snapshot copy
  std::vector<char> slot_busy;
  std::vector<int> unfenced;          // slots whose snapshot copy no compute stream waits for yet

  std::mutex m;
  std::condition_variable cv_work, cv_idle;
  std::vector<std::deque<std::shared_ptr<SaveJob>>> queues;   // one per daemon thread
  std::vector<std::thread> threads;
  bool stopping = false;
  int64_t jobs_in_flight = 0;
  hc_status first_error = HC_OK;
  std::string first_error_msg;
};

static void daemon_main(hc_saver* sv, int tid) {
  if (sv->device >= 0) (void)hipSetDevice(sv->device);
  for (;;) {
    std::shared_ptr<SaveJob> job;
    {
      std::unique_lock<std::mutex> lock(sv->m);
      sv->cv_work.wait(lock, [&] { return sv->stopping || !sv->queues[tid].empty(); });
      if (sv->queues[tid].empty()) return;             // stopping and drained
      job = sv->queues[tid].front();
      sv->queues[tid].pop_front();
    }
    hc_status err = HC_OK;
    std::string msg;
    if (job->copied) {
      hipError_t e = hipEventSynchronize(job->copied);
      if (e != hipSuccess) {
        err = HC_EHIP;
        msg = std::string("hipEventSynchronize in the save daemon: ") + hipGetErrorString(e);
      }
    }
    if (err == HC_OK) {
      const unsigned char* rows = sv->slot_buf[job->slot];
      for (size_t i = tid; i < job->pieces.size(); i += sv->n_threads) {
        const StorePiece& pc = job->pieces[i];
        memcpy(pc.dst, rows + pc.src_off, pc.bytes);
      }
    }
    {
      std::lock_guard<std::mutex> lock(sv->m);
      if (err != HC_OK && sv->first_error == HC_OK) {
        sv->first_error = err;
        sv->first_error_msg = msg;
      }
      if (job->workers_left.fetch_sub(1) == 1) {
        sv->slot_busy[job->slot] = 0;
        --sv->jobs_in_flight;
        sv->cv_idle.notify_all();
      }
    }
  }
}

// Take a free snapshot slot (blocks while all are in use: back-pressure on the producer).
static int acquire_slot(hc_saver* sv) {
  std::unique_lock<std::mutex> lock(sv->m);
  for (;;) {
    for (int s = 0; s < sv->n_slots; ++s)
      if (!sv->slot_busy[s]) {
        sv->slot_busy[s] = 1;
        ++sv->jobs_in_flight;
        return s;
      }
    sv->cv_idle.wait(lock);
  }
}

static void submit(hc_saver* sv, const std::shared_ptr<SaveJob>& job) {
  job->workers_left.store(sv->n_threads);
  {
    std::lock_guard<std::mutex> lock(sv->m);
    for (auto& q : sv->queues) q.push_back(job);
  }
  sv->cv_work.notify_all();
}

static hc_status check_save_args(hc_saver* sv, int32_t layer, const void* rows, int32_t n_rows,
                                 const int64_t* h_row_seq) {
  if (!sv) return fail(HC_EINVAL, "saver is null");
  if (layer < 0 || layer >= sv->store->n_layers) return fail(HC_ERANGE, "layer out of range");
  if (n_rows < 0) return fail(HC_EINVAL, "negative row count");
  if (n_rows > sv->max_rows) return fail(HC_ERANGE, "batch larger than the saver's max_rows");
  if (n_rows > 0 && (!rows || !h_row_seq)) return fail(HC_EINVAL, "null pointer");
  return HC_OK;
}

// Index half of the save, in the producer thread: one reservation per run of rows of the same
// context.  On failure nothing of this batch is queued (rows reserved before the failing run
// stay counted in the store: the context's saved state is then incomplete and should be dropped).
static hc_status reserve_batch(hc_saver* sv, int32_t layer, int32_t n_rows, const int64_t* row_seq,
                               std::vector<StorePiece>& pieces) {
  int i = 0;
  while (i < n_rows) {
    int j = i + 1;
    while (j < n_rows && row_seq[j] == row_seq[i]) ++j;
    const size_t first = pieces.size();
    hc_status r = store_reserve(sv->store, row_seq[i], layer, j - i, pieces);
    if (r != HC_OK) return r;
    for (size_t p = first; p < pieces.size(); ++p) pieces[p].src_off += (size_t)i * sv->row_bytes;
    i = j;
  }
  return HC_OK;
}

extern "C" {

hc_status hc_saver_create(hc_store* store, int32_t max_rows, int32_t n_slots, int32_t n_threads,
                          hc_saver** out) {
  clear_error();
  if (!out) return fail(HC_EINVAL, "out is null");
  *out = nullptr;
  if (!store) return fail(HC_EINVAL, "store is null");
  if (max_rows <= 0 || n_slots <= 0 || n_threads <= 0 || n_threads > 64 || n_slots > 1024)
    return fail(HC_EINVAL, "max_rows, n_slots must be positive; n_threads in 1..64");
  hc_saver* sv = new (std::nothrow) hc_saver();
  if (!sv) return fail(HC_ENOMEM, "out of host memory");
  sv->store = store;
  sv->max_rows = max_rows;
  sv->n_slots = n_slots;
  sv->n_threads = n_threads;
  sv->row_bytes = store->row_bytes;
  int dev = -1;
  if (hipGetDevice(&dev) == hipSuccess) sv->device = dev;
  else (void)hipGetLastError();
  const size_t bytes = (size_t)max_rows * sv->row_bytes;
  bool ok = true;
  for (int s = 0; s < n_slots && ok; ++s) {
    void* p = nullptr;
    bool pinned = false;
    if (sv->device >= 0 && hipHostMalloc(&p, bytes, hipHostMallocDefault) == hipSuccess) {
      pinned = true;
    } else {
      (void)hipGetLastError();
      p = nullptr;
      if (sv->device >= 0 || posix_memalign(&p, 4096, bytes) != 0) ok = false;   // a GPU host must pin
    }
    if (!ok) break;
    sv->slot_buf.push_back(static_cast<unsigned char*>(p));
    sv->slot_pinned.push_back(pinned);
    hipEvent_t a = nullptr, b = nullptr;
    if (sv->device >= 0) {
      if (hipEventCreateWithFlags(&a, hipEventDisableTiming) != hipSuccess ||
          hipEventCreateWithFlags(&b, hipEventDisableTiming) != hipSuccess)
        ok = false;
    }
    sv->ev_ready.push_back(a);
    sv->ev_copied.push_back(b);
  }
  if (!ok) {
    (void)hipGetLastError();
    for (size_t s = 0; s < sv->slot_buf.size(); ++s) {
      if (sv->slot_pinned[s]) (void)hipHostFree(sv->slot_buf[s]); else free(sv->slot_buf[s]);
      if (sv->ev_ready[s]) (void)hipEventDestroy(sv->ev_ready[s]);
      if (sv->ev_copied[s]) (void)hipEventDestroy(sv->ev_copied[s]);
    }
    delete sv;
    return fail(HC_ENOMEM, "allocation of the snapshot slots failed");
  }
  sv->slot_busy.assign(n_slots, 0);
  sv->queues.resize(n_threads);
  for (int t = 0; t < n_threads; ++t) sv->threads.emplace_back(daemon_main, sv, t);
  *out = sv;
  return HC_OK;
}

hc_status hc_saver_flush(hc_saver* sv) {
  clear_error();
  if (!sv) return fail(HC_EINVAL, "saver is null");
  std::unique_lock<std::mutex> lock(sv->m);
  sv->cv_idle.wait(lock, [&] { return sv->jobs_in_flight == 0; });
  if (sv->first_error != HC_OK) {
    const hc_status e = sv->first_error;
    const std::string msg = "save daemon: " + sv->first_error_msg;
    sv->first_error = HC_OK;
    sv->first_error_msg.clear();
    return fail(e, msg);
  }
  return HC_OK;
}

hc_status hc_saver_destroy(hc_saver* sv) {
  clear_error();
  if (!sv) return HC_OK;
  {
    std::unique_lock<std::mutex> lock(sv->m);
    sv->cv_idle.wait(lock, [&] { return sv->jobs_in_flight == 0; });
    sv->stopping = true;
  }
  sv->cv_work.notify_all();
  for (auto& t : sv->threads) t.join();
  for (size_t s = 0; s < sv->slot_buf.size(); ++s) {
    if (sv->slot_pinned[s]) (void)hipHostFree(sv->slot_buf[s]); else free(sv->slot_buf[s]);
    if (sv->ev_ready[s]) (void)hipEventDestroy(sv->ev_ready[s]);
    if (sv->ev_copied[s]) (void)hipEventDestroy(sv->ev_copied[s]);
  }
  delete sv;
  return HC_OK;
}

// Make `stream` wait for every snapshot copy no stream has been made to wait for yet.
static hipError_t fence_snapshots(hc_saver* sv, hipStream_t stream) {
  for (int slot : sv->unfenced) {
    hipError_t e = hipStreamWaitEvent(stream, sv->ev_copied[slot], 0);
    if (e != hipSuccess) return e;
  }
  sv->unfenced.clear();
  return hipSuccess;
}

static hc_status save_layer_impl(hc_saver* sv, int32_t layer, const void* d_hidden, int32_t n_rows,
                                 const int64_t* h_row_seq, void* compute_stream, void* down_stream,
                                 bool fence_now) {
  clear_error();
  hc_status s = check_save_args(sv, layer, d_hidden, n_rows, h_row_seq);
  if (s != HC_OK) return s;
  if (n_rows == 0) return HC_OK;
  if (sv->device < 0) return fail(HC_ESTATE, "saver was created without a GPU");
  if (compute_stream == down_stream) return fail(HC_EINVAL, "compute and downstream streams must differ");
  hipStream_t cs = static_cast<hipStream_t>(compute_stream);
  hipStream_t ds = static_cast<hipStream_t>(down_stream);
  auto job = std::make_shared<SaveJob>();
  s = reserve_batch(sv, layer, n_rows, h_row_seq, job->pieces);
  if (s != HC_OK) return s;
  const int slot = acquire_slot(sv);
  auto release = [&] {
    std::lock_guard<std::mutex> lock(sv->m);
    sv->slot_busy[slot] = 0;
    --sv->jobs_in_flight;
    sv->cv_idle.notify_all();
  };
  hipError_t e = hipEventRecord(sv->ev_ready[slot], cs);           // the layer's input is complete here
  if (e == hipSuccess) e = hipStreamWaitEvent(ds, sv->ev_ready[slot], 0);
  // Long runs of one context's rows (a prefill, or the prefill share of a fused step) go
  // straight from the device into their chunks of the pinned arena: no snapshot, no second
  // copy by the daemons.  Full chunks of such a run sit a fixed distance apart in the arena, so
  // they move in ONE strided transfer.  What is left -- the scattered single rows of decoding
  // contexts -- is snapshot with one copy of the batch's sub-range that holds them and
  // re-tiled by the daemon threads as before.
  std::vector<StorePiece> small;
  if (sv->store->pinned) {
    const unsigned char* src = static_cast<const unsigned char*>(d_hidden);
    std::vector<StorePiece>& pc = job->pieces;
    size_t i = 0;
    while (i < pc.size() && e == hipSuccess) {
      if (pc[i].bytes < kDirectMinBytes) {
        small.push_back(pc[i++]);
        continue;
      }
      size_t j = i + 1;                                            // group [i, j): one strided transfer
      if (j < pc.size() && pc[j].bytes == pc[i].bytes && pc[j].dst > pc[i].dst &&
          pc[j].src_off == pc[i].src_off + pc[i].bytes) {
        const size_t pitch = (size_t)(pc[j].dst - pc[i].dst);
        ++j;
        while (j < pc.size() && pc[j].bytes == pc[i].bytes && pc[j].dst == pc[j - 1].dst + pitch &&
               pc[j].src_off == pc[j - 1].src_off + pc[i].bytes)
          ++j;
        e = hipMemcpy2DAsync(pc[i].dst, pitch, src + pc[i].src_off, pc[i].bytes, pc[i].bytes, j - i,
                             hipMemcpyDeviceToHost, ds);
      } else {
        e = hipMemcpy2DAsync(pc[i].dst, pc[i].bytes, src + pc[i].src_off, pc[i].bytes, pc[i].bytes, 1,
                             hipMemcpyDeviceToHost, ds);
      }
      i = j;
    }
  } else {
    small.swap(job->pieces);
  }
  if (e == hipSuccess && !small.empty()) {
    // snapshot the sub-range of the batch that holds the remaining rows (pieces are in batch order)
    const size_t lo = small.front().src_off, hi = small.back().src_off + small.back().bytes;
    e = hipMemcpy2DAsync(sv->slot_buf[slot], hi - lo, static_cast<const unsigned char*>(d_hidden) + lo, hi - lo,
                         hi - lo, 1, hipMemcpyDeviceToHost, ds);
    for (StorePiece& q : small) q.src_off -= lo;
  }
  job->pieces.swap(small);
  if (e == hipSuccess) e = hipEventRecord(sv->ev_copied[slot], ds);
  if (e == hipSuccess) {
    // a reused slot's event has just been re-recorded; keep it listed once
    bool listed = false;
    for (int u : sv->unfenced) listed = listed || u == slot;
    if (!listed) sv->unfenced.push_back(slot);
    // later work on the compute stream may overwrite the activation buffer only after the copy
    if (fence_now) e = fence_snapshots(sv, cs);
  }
  if (e != hipSuccess) {
    release();
    return fail_hip(e, "hc_saver_save_layer");
  }
  job->slot = slot;
  job->copied = sv->ev_copied[slot];
  submit(sv, job);
  return HC_OK;
}

hc_status hc_saver_save_layer(hc_saver* sv, int32_t layer, const void* d_hidden, int32_t n_rows,
                              const int64_t* h_row_seq, void* compute_stream, void* down_stream) {
  return save_layer_impl(sv, layer, d_hidden, n_rows, h_row_seq, compute_stream, down_stream, true);
}

hc_status hc_saver_save_layer_deferred(hc_saver* sv, int32_t layer, const void* d_hidden,
                                       int32_t n_rows, const int64_t* h_row_seq,
                                       void* compute_stream, void* down_stream) {
  return save_layer_impl(sv, layer, d_hidden, n_rows, h_row_seq, compute_stream, down_stream, false);
}

hc_status hc_saver_fence(hc_saver* sv, void* stream) {
  clear_error();
  if (!sv) return fail(HC_EINVAL, "saver is null");
  if (sv->device < 0) return HC_OK;                      // host-only saver: nothing is in flight
  HC_HIP(fence_snapshots(sv, static_cast<hipStream_t>(stream)));
  return HC_OK;
}

hc_status hc_saver_save_layer_host(hc_saver* sv, int32_t layer, const void* h_rows, int32_t n_rows,
                                   const int64_t* h_row_seq) {
  clear_error();
  hc_status s = check_save_args(sv, layer, h_rows, n_rows, h_row_seq);
  if (s != HC_OK) return s;
  if (n_rows == 0) return HC_OK;
  auto job = std::make_shared<SaveJob>();
  s = reserve_batch(sv, layer, n_rows, h_row_seq, job->pieces);
  if (s != HC_OK) return s;
  const int slot = acquire_slot(sv);
  memcpy(sv->slot_buf[slot], h_rows, (size_t)n_rows * sv->row_bytes);
  job->slot = slot;
  submit(sv, job);
  return HC_OK;
}

}  // extern "C"
