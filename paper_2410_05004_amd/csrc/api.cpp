// C ABI of libhcache.so: argument validation, context state, launches.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "hcache_internal.h"

namespace hc {

static thread_local std::string g_last_error;

hc_status fail(hc_status code, const std::string& msg) {
  g_last_error = msg;
  return code;
}
hc_status fail_hip(hipError_t e, const char* what) {
  g_last_error = std::string(what) + ": " + hipGetErrorString(e);
  (void)hipGetLastError();   // clear the sticky error so the next call starts clean
  return HC_EHIP;
}
void clear_error() { g_last_error.clear(); }

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

static hc_status check_desc(const hc_model_desc* d) {
  if (!d) return fail(HC_EINVAL, "desc is null");
  if (d->n_layers <= 0) return fail(HC_EINVAL, "n_layers must be positive");
  if (d->d_model <= 0 || d->d_model % 64 != 0)
    return fail(HC_EINVAL, "d_model must be a positive multiple of 64");
  if (d->head_dim <= 0 || d->head_dim % 64 != 0)
    return fail(HC_EINVAL, "head_dim must be a positive multiple of 64");
  if (d->n_kv_heads <= 0 || d->n_q_heads <= 0 || d->n_q_heads % d->n_kv_heads != 0)
    return fail(HC_EINVAL, "n_q_heads must be a positive multiple of n_kv_heads");
  if (!is_pow2(d->block_size)) return fail(HC_EINVAL, "block_size must be a power of two");
  if (d->max_position <= 0) return fail(HC_EINVAL, "max_position must be positive");
  if ((int64_t)d->max_position * (d->head_dim / 2) * 8 > ((int64_t)1 << 34))
    return fail(HC_EINVAL, "RoPE table would exceed 16 GiB");
  if (d->rope_style < 0 || d->rope_style > 2)
    return fail(HC_EINVAL, "rope_style must be 0 (half-split), 1 (interleaved) or 2 (none)");
  if (d->norm_kind != HC_NORM_RMS && d->norm_kind != HC_NORM_LAYER)
    return fail(HC_EINVAL, "norm_kind must be HC_NORM_RMS or HC_NORM_LAYER");
  if (!(d->rope_theta > 0.f)) return fail(HC_EINVAL, "rope_theta must be positive");
  if (!(d->rms_eps >= 0.f)) return fail(HC_EINVAL, "rms_eps must be non-negative");
  if ((int64_t)d->n_kv_heads * d->head_dim > (1 << 20))
    return fail(HC_EINVAL, "n_kv_heads * head_dim too large");
  return HC_OK;
}

static hc_status check_layer(const hc_ctx* ctx, int32_t layer) {
  if (!ctx) return fail(HC_EINVAL, "ctx is null");
  if (layer < 0 || layer >= ctx->desc.n_layers) return fail(HC_ERANGE, "layer out of range");
  return HC_OK;
}

// Arguments shared by all layers of a context's launch.
static RestoreArgs shared_args(const hc_ctx* ctx, const int32_t* d_positions, int32_t pos_base,
                               int32_t n_tok, const int32_t* d_cu, int32_t n_seq,
                               const int32_t* d_tables, int32_t max_blocks) {
  RestoreArgs a{};
  a.positions = d_positions;
  a.cu_seqlens = d_cu;
  a.block_tables = d_tables;
  a.rope = ctx->rope;
  a.err = ctx->err_dev;
  a.pos_base = pos_base;
  a.n_seq = n_seq;
  a.max_blocks = max_blocks;
  a.max_position = ctx->desc.max_position;
  a.n_tok = n_tok;
  a.d_model = ctx->desc.d_model;
  a.d_kv = ctx->d_kv;
  a.d_kv_pad = ctx->d_kv_pad;
  a.head_dim = ctx->desc.head_dim;
  a.block_shift = ctx->block_shift;
  a.rope_style = ctx->desc.rope_style;
  a.inv_d = 1.0f / (float)ctx->desc.d_model;
  a.eps = ctx->desc.rms_eps;
  return a;
}

static int layer_mode(const hc_ctx* ctx, const hc_layer_state& L) {
  return ctx->desc.norm_kind == HC_NORM_LAYER ? 2 : (L.affine ? 1 : 0);
}

// One timed (when timing is on) launch.
static hc_status timed_launch(hc_ctx* ctx, const RestoreArgs& a, LayerBatch* batch, int n_layers,
                              hipStream_t stream) {
  const bool timed = ctx->timing && ctx->ev_used + 2 <= 8192;
  if (timed) {
    while ((int)ctx->ev_pool.size() < ctx->ev_used + 2) {
      hipEvent_t e;
      HC_HIP(hipEventCreate(&e));
      ctx->ev_pool.push_back(e);
    }
    HC_HIP(hipEventRecord(ctx->ev_pool[ctx->ev_used], stream));
  }
  SplitPlan sp;
  TileGrid g_main;
  const bool split = !batch && restore_would_split(a, sp, g_main);
  // the workspace is one per context: a split launch waits for the one before it, whatever its stream
  if (split) HC_HIP(hipStreamWaitEvent(stream, ctx->split_done, 0));
  HC_HIP(launch_restore(a, batch, n_layers, stream));
  if (split) HC_HIP(hipEventRecord(ctx->split_done, stream));
  if (timed) {
    HC_HIP(hipEventRecord(ctx->ev_pool[ctx->ev_used + 1], stream));
    ctx->ev_used += 2;
  }
  return HC_OK;
}

// Launch the fused kernel for one layer (shared by the single-layer restore entry points).
hc_status restore_layer(hc_ctx* ctx, int32_t layer, const void* d_hidden,
                        const int32_t* d_positions, int32_t pos_base, int32_t n_tok,
                        const int32_t* d_cu, int32_t n_seq, const int32_t* d_tables,
                        int32_t max_blocks, hipStream_t stream, bool allow_split) {
  const hc_layer_state& L = ctx->layers[layer];
  if (!L.wpack) return fail(HC_ESTATE, "hc_set_layer_weights was not called for this layer");
  if (!L.pool) return fail(HC_ESTATE, "hc_set_kv_pool was not called for this layer");
  RestoreArgs a = shared_args(ctx, d_positions, pos_base, n_tok, d_cu, n_seq, d_tables, max_blocks);
  a.hidden = static_cast<const uint16_t*>(d_hidden);
  a.wpack = L.wpack;
  a.affine = L.affine;
  a.mode = layer_mode(ctx, L);
  a.pool = L.pool;
  a.num_pages = L.num_pages;
  a.split_ws = allow_split && ctx->split_mode ? ctx->split_ws : nullptr;
  a.split_force = ctx->split_mode == 2;
  return timed_launch(ctx, a, nullptr, 1, stream);
}

hc_status restore_layers(hc_ctx* ctx, int32_t layer_begin, int32_t n_layers,
                         const void* const* d_hidden, const int32_t* d_positions, int32_t pos_base,
                         int32_t n_tok, const int32_t* d_block_table, int32_t n_blocks,
                         hipStream_t stream) {
  for (int i = 0; i < n_layers; ++i) {
    const hc_layer_state& L = ctx->layers[layer_begin + i];
    if (!L.wpack) return fail(HC_ESTATE, "hc_set_layer_weights was not called for some layer");
    if (!L.pool) return fail(HC_ESTATE, "hc_set_kv_pool was not called for some layer");
    if (!d_hidden[i]) return fail(HC_EINVAL, "null hidden-state pointer");
    if (!aligned16(d_hidden[i])) return fail(HC_EALIGN, "hidden not 16-byte aligned");
  }
  RestoreArgs a = shared_args(ctx, d_positions, pos_base, n_tok, nullptr, 1, d_block_table, n_blocks);
  const int per_launch = layers_per_launch(2 * ctx->d_kv_pad / kTileF, (n_tok + kTileT - 1) / kTileT);
  int i = 0;
  while (i < n_layers) {
    // one launch per run of layers with the same kernel mode, at most per_launch of them
    LayerBatch batch{};
    const int mode = layer_mode(ctx, ctx->layers[layer_begin + i]);
    int n = 0;
    while (i + n < n_layers && n < per_launch &&
           layer_mode(ctx, ctx->layers[layer_begin + i + n]) == mode) {
      const hc_layer_state& L = ctx->layers[layer_begin + i + n];
      batch.e[n] = LayerEntry{static_cast<const uint16_t*>(d_hidden[i + n]), L.wpack, L.affine, L.pool,
                              L.num_pages};
      ++n;
    }
    a.mode = mode;
    hc_status r = timed_launch(ctx, a, &batch, n, stream);
    if (r != HC_OK) return r;
    i += n;
  }
  return HC_OK;
}

hc_status kv_rows_layer(hc_ctx* ctx, int32_t layer, void* d_rows, const int32_t* d_positions,
                        int32_t pos_base, int32_t n_tok, const int32_t* d_block_table,
                        int32_t n_blocks, bool to_pool, hipStream_t stream) {
  const hc_layer_state& L = ctx->layers[layer];
  if (!L.pool) return fail(HC_ESTATE, "hc_set_kv_pool was not called for this layer");
  KvRowsArgs a;
  a.rows = static_cast<uint16_t*>(d_rows);
  a.pool = L.pool;
  a.positions = d_positions;
  a.block_table = d_block_table;
  a.err = ctx->err_dev;
  a.num_pages = L.num_pages;
  a.pos_base = pos_base;
  a.n_tok = n_tok;
  a.n_blocks = n_blocks;
  a.max_position = ctx->desc.max_position;
  a.d_kv = ctx->d_kv;
  a.block_shift = ctx->block_shift;
  HC_HIP(launch_kv_rows(a, to_pool, stream));
  return HC_OK;
}

}  // namespace hc

using namespace hc;

extern "C" {

const char* hc_last_error(void) { return g_last_error.c_str(); }
const char* hc_version(void) { return "hcache-mi355x 0.1"; }

hc_status hc_validate_desc(const hc_model_desc* desc) {
  clear_error();
  return check_desc(desc);
}

hc_status hc_create(const hc_model_desc* desc, hc_ctx** out) {
  clear_error();
  if (!out) return fail(HC_EINVAL, "out is null");
  *out = nullptr;
  hc_status s = check_desc(desc);
  if (s != HC_OK) return s;
  hc_ctx* ctx = new (std::nothrow) hc_ctx();
  if (!ctx) return fail(HC_ENOMEM, "out of host memory");
  ctx->desc = *desc;
  ctx->d_kv = desc->n_kv_heads * desc->head_dim;
  ctx->d_kv_pad = round_up(ctx->d_kv, kPartAlign);
  ctx->n_phys = 2 * ctx->d_kv_pad;
  for (int b = desc->block_size; b > 1; b >>= 1) ctx->block_shift++;
  ctx->layers.resize(desc->n_layers);

  hipError_t e = hipGetDevice(&ctx->device);
  if (e == hipSuccess) e = configure_kernels();
  if (e == hipSuccess && static_scratch_init() != HC_OK) {
    delete ctx;
    return HC_EHIP;                                  // message set by static_scratch_init
  }
  const bool rotary = desc->rope_style != 2;
  if (e == hipSuccess && rotary)
    e = hipMalloc(reinterpret_cast<void**>(&ctx->rope),
                  (size_t)desc->max_position * (desc->head_dim / 2) * sizeof(float2));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ctx->err_dev), 256);
  if (e == hipSuccess) e = hipMemset(ctx->err_dev, 0, 256);
  if (e == hipSuccess)
    e = hipMalloc(reinterpret_cast<void**>(&ctx->split_ws), (size_t)kSplitMaxSlots * kSplitSlotFloats * sizeof(float));
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->split_done, hipEventDisableTiming);
  if (e == hipSuccess && rotary)
    e = launch_rope_table(ctx->rope, desc->max_position, desc->head_dim, (double)desc->rope_theta,
                          nullptr);
  if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
  if (e != hipSuccess) {
    hc_status st = fail_hip(e, "hc_create");
    if (ctx->rope) (void)hipFree(ctx->rope);
    if (ctx->err_dev) (void)hipFree(ctx->err_dev);
    if (ctx->split_ws) (void)hipFree(ctx->split_ws);
    if (ctx->split_done) (void)hipEventDestroy(ctx->split_done);
    delete ctx;
    return st;
  }
  *out = ctx;
  return HC_OK;
}

hc_status hc_destroy(hc_ctx* ctx) {
  clear_error();
  if (!ctx) return HC_OK;
  (void)hipDeviceSynchronize();
  for (auto& L : ctx->layers) {
    if (L.wpack) (void)hipFree(L.wpack);
    if (L.affine) (void)hipFree(L.affine);
  }
  if (ctx->rope) (void)hipFree(ctx->rope);
  if (ctx->err_dev) (void)hipFree(ctx->err_dev);
  if (ctx->split_ws) (void)hipFree(ctx->split_ws);
  if (ctx->split_done) (void)hipEventDestroy(ctx->split_done);
  if (ctx->copy2) (void)hipStreamDestroy(ctx->copy2);
  for (int i = 0; i < 2; ++i) {
    if (ctx->stage[i]) (void)hipFree(ctx->stage[i]);
    if (ctx->h2d_done[i]) (void)hipEventDestroy(ctx->h2d_done[i]);
    if (ctx->buf_free[i]) (void)hipEventDestroy(ctx->buf_free[i]);
  }
  for (int i = 0; i < 2; ++i) {
    if (ctx->seg_tab[i]) (void)hipHostFree(ctx->seg_tab[i]);
    if (ctx->seg_done[i]) (void)hipEventDestroy(ctx->seg_done[i]);
    if (ctx->cu_host[i]) (void)hipHostFree(ctx->cu_host[i]);
    if (ctx->cu_dev[i]) (void)hipFree(ctx->cu_dev[i]);
    if (ctx->cu_done[i]) (void)hipEventDestroy(ctx->cu_done[i]);
  }
  for (hipEvent_t e : ctx->ev_pool) (void)hipEventDestroy(e);
  delete ctx;
  return HC_OK;
}

hc_status hc_set_layer_weights(hc_ctx* ctx, int32_t layer, const void* d_wkv, const void* d_gamma,
                               void* stream) {
  return hc_set_layer_weights_affine(ctx, layer, d_wkv, d_gamma, nullptr, nullptr, stream);
}

hc_status hc_set_layer_weights_affine(hc_ctx* ctx, int32_t layer, const void* d_wkv,
                                      const void* d_gamma, const void* d_beta,
                                      const void* d_bias, void* stream) {
  clear_error();
  hc_status s = check_layer(ctx, layer);
  if (s != HC_OK) return s;
  if (!d_wkv || !d_gamma) return fail(HC_EINVAL, "weight pointer is null");
  if (!aligned16(d_wkv) || !aligned16(d_gamma)) return fail(HC_EALIGN, "weights not 16-byte aligned");
  const bool layer_norm = ctx->desc.norm_kind == HC_NORM_LAYER;
  if (d_beta && !layer_norm) return fail(HC_EINVAL, "a shift needs norm_kind = HC_NORM_LAYER");
  hc_layer_state& L = ctx->layers[layer];
  // LayerNorm always needs the row sums; RMSNorm needs the table only for a bias
  const bool need_affine = layer_norm || d_bias;
  if (need_affine && !L.affine) {
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&L.affine), (size_t)ctx->n_phys * sizeof(float2));
    if (e != hipSuccess) {
      L.affine = nullptr;
      (void)hipGetLastError();
      return fail(HC_ENOMEM, "device allocation of the row constants failed");
    }
  }
  if (!need_affine && L.affine) {
    // replaced by plain weights; kernels already queued may still read the table
    HC_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    HC_HIP(hipFree(L.affine));
    L.affine = nullptr;
  }
  if (need_affine)
    HC_HIP(launch_pack_affine(static_cast<const uint16_t*>(d_wkv), static_cast<const uint16_t*>(d_gamma),
                              static_cast<const uint16_t*>(d_beta), static_cast<const uint16_t*>(d_bias),
                              L.affine, ctx->desc.d_model, ctx->d_kv, ctx->desc.head_dim,
                              ctx->desc.rope_style, static_cast<hipStream_t>(stream)));
  if (!L.wpack) {
    const size_t bytes = (size_t)ctx->n_phys * ctx->desc.d_model * sizeof(uint16_t);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&L.wpack), bytes);
    if (e != hipSuccess) {
      L.wpack = nullptr;
      (void)hipGetLastError();
      return fail(HC_ENOMEM, "device allocation of packed weights failed");
    }
  }
  HC_HIP(launch_pack_weights(static_cast<const uint16_t*>(d_wkv),
                             static_cast<const uint16_t*>(d_gamma), L.wpack, ctx->desc.d_model,
                             ctx->d_kv, ctx->desc.head_dim, ctx->desc.rope_style,
                             static_cast<hipStream_t>(stream)));
  return HC_OK;
}

hc_status hc_set_kv_pool(hc_ctx* ctx, int32_t layer, void* d_pool, int64_t num_pages) {
  clear_error();
  hc_status s = check_layer(ctx, layer);
  if (s != HC_OK) return s;
  if (!d_pool) return fail(HC_EINVAL, "pool pointer is null");
  if (!aligned16(d_pool)) return fail(HC_EALIGN, "pool not 16-byte aligned");
  // the kernels number a pool's token rows (2 * block_size per page) with 32-bit integers
  if (num_pages <= 0 || num_pages * 2 * ctx->desc.block_size > ((int64_t)1 << 31) - 1)
    return fail(HC_ERANGE, "num_pages out of range (num_pages * 2 * block_size must stay below 2^31)");
  ctx->layers[layer].pool = static_cast<uint16_t*>(d_pool);
  ctx->layers[layer].num_pages = num_pages;
  return HC_OK;
}

hc_status hc_restore_kv(hc_ctx* ctx, int32_t layer, const void* d_hidden,
                        const int32_t* d_positions, int32_t n_tok, const int32_t* d_block_table,
                        int32_t n_blocks, void* stream) {
  clear_error();
  hc_status s = check_layer(ctx, layer);
  if (s != HC_OK) return s;
  if (n_tok < 0 || n_blocks < 0) return fail(HC_EINVAL, "negative size");
  if (n_tok == 0) return HC_OK;
  if (!d_hidden || !d_positions || !d_block_table) return fail(HC_EINVAL, "null device pointer");
  if (!aligned16(d_hidden)) return fail(HC_EALIGN, "hidden not 16-byte aligned");
  return restore_layer(ctx, layer, d_hidden, d_positions, 0, n_tok, nullptr, 1, d_block_table,
                       n_blocks, static_cast<hipStream_t>(stream));
}

hc_status hc_restore_kv_layers(hc_ctx* ctx, int32_t layer_begin, int32_t n_layers,
                               const void* const* h_d_hidden, const int32_t* d_positions,
                               int32_t n_tok, const int32_t* d_block_table, int32_t n_blocks,
                               void* stream) {
  clear_error();
  if (!ctx) return fail(HC_EINVAL, "ctx is null");
  if (n_layers < 0 || n_tok < 0 || n_blocks < 0) return fail(HC_EINVAL, "negative size");
  if (layer_begin < 0 || (int64_t)layer_begin + n_layers > ctx->desc.n_layers)
    return fail(HC_ERANGE, "layer range outside the model");
  if (n_layers == 0 || n_tok == 0) return HC_OK;
  if (!h_d_hidden || !d_positions || !d_block_table) return fail(HC_EINVAL, "null pointer");
  return restore_layers(ctx, layer_begin, n_layers, h_d_hidden, d_positions, 0, n_tok, d_block_table,
                        n_blocks, static_cast<hipStream_t>(stream));
}

hc_status hc_restore_kv_ragged(hc_ctx* ctx, int32_t layer, const void* d_hidden,
                               const int32_t* d_positions, int32_t h_total_tokens,
                               const int32_t* d_cu_seqlens, int32_t n_seq,
                               const int32_t* d_block_tables, int32_t max_blocks, void* stream) {
  clear_error();
  hc_status s = check_layer(ctx, layer);
  if (s != HC_OK) return s;
  if (h_total_tokens < 0 || n_seq < 0 || max_blocks < 0) return fail(HC_EINVAL, "negative size");
  if (h_total_tokens == 0 || n_seq == 0) return HC_OK;
  if (!d_hidden || !d_positions || !d_cu_seqlens || !d_block_tables)
    return fail(HC_EINVAL, "null device pointer");
  if (!aligned16(d_hidden)) return fail(HC_EALIGN, "hidden not 16-byte aligned");
  return restore_layer(ctx, layer, d_hidden, d_positions, 0, h_total_tokens, d_cu_seqlens, n_seq,
                       d_block_tables, max_blocks, static_cast<hipStream_t>(stream));
}

static hc_status kv_rows_entry(hc_ctx* ctx, int32_t layer, void* d_rows,
                               const int32_t* d_positions, int32_t n_tok,
                               const int32_t* d_block_table, int32_t n_blocks, bool to_pool,
                               void* stream) {
  clear_error();
  hc_status s = check_layer(ctx, layer);
  if (s != HC_OK) return s;
  if (n_tok < 0 || n_blocks < 0) return fail(HC_EINVAL, "negative size");
  if (n_tok == 0) return HC_OK;
  if (!d_rows || !d_positions || !d_block_table) return fail(HC_EINVAL, "null device pointer");
  if (!aligned16(d_rows)) return fail(HC_EALIGN, "rows not 16-byte aligned");
  return kv_rows_layer(ctx, layer, d_rows, d_positions, 0, n_tok, d_block_table, n_blocks, to_pool,
                       static_cast<hipStream_t>(stream));
}

hc_status hc_gather_kv(hc_ctx* ctx, int32_t layer, void* d_rows, const int32_t* d_positions,
                       int32_t n_tok, const int32_t* d_block_table, int32_t n_blocks,
                       void* stream) {
  return kv_rows_entry(ctx, layer, d_rows, d_positions, n_tok, d_block_table, n_blocks, false,
                       stream);
}

hc_status hc_scatter_kv(hc_ctx* ctx, int32_t layer, const void* d_rows,
                        const int32_t* d_positions, int32_t n_tok, const int32_t* d_block_table,
                        int32_t n_blocks, void* stream) {
  return kv_rows_entry(ctx, layer, const_cast<void*>(d_rows), d_positions, n_tok, d_block_table,
                       n_blocks, true, stream);
}

hc_status hc_poll_device_error(hc_ctx* ctx, void* stream, int32_t* out_flags) {
  clear_error();
  if (!ctx || !out_flags) return fail(HC_EINVAL, "null argument");
  hipStream_t st = static_cast<hipStream_t>(stream);
  HC_HIP(hipMemcpyAsync(out_flags, ctx->err_dev, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  HC_HIP(hipMemsetAsync(ctx->err_dev, 0, sizeof(int32_t), st));
  HC_HIP(hipStreamSynchronize(st));
  return HC_OK;
}

hc_status hc_partition_layers(int32_t n_layers, double io_h, double io_kv, double c_h,
                              double c_token, int32_t* l_h, int32_t* l_o, int32_t* complement) {
  clear_error();
  if (!l_h || !l_o || !complement) return fail(HC_EINVAL, "null output pointer");
  if (n_layers <= 0) return fail(HC_EINVAL, "n_layers must be positive");
  if (!(io_h > 0) || !(io_kv > 0) || !(c_h > 0) || !(c_token > 0))
    return fail(HC_EINVAL, "times must be positive");
  if (!(io_kv > io_h))
    return fail(HC_EINVAL, "io_kv <= io_h: KV offload alone moves no more data than hidden states");
  if (!(c_token > c_h))
    return fail(HC_EINVAL, "c_token <= c_h: recomputation alone is no slower than projection");
  double x;
  if (c_h > io_h) {
    *complement = HC_COMPLEMENT_KV;
    x = n_layers * io_kv / (io_kv + c_h - io_h);
  } else {
    *complement = HC_COMPLEMENT_RECOMPUTE;
    x = n_layers * c_token / (c_token + io_h - c_h);
  }
  // the ceiling as printed, on the double-precision quotient
  int32_t lh = (int32_t)std::ceil(x);
  if (lh > n_layers) lh = n_layers;
  if (lh < 0) lh = 0;
  *l_h = lh;
  *l_o = n_layers - lh;
  return HC_OK;
}

hc_status hc_set_loader(hc_ctx* ctx, int32_t mode) {
  clear_error();
  if (!ctx) return fail(HC_EINVAL, "ctx is null");
  if (mode != 0 && mode != 1) return fail(HC_EINVAL, "loader mode must be 0 (copy engines) or 1 (gather kernel)");
  ctx->loader_mode = mode;
  return HC_OK;
}

hc_status hc_set_split(hc_ctx* ctx, int32_t mode) {
  clear_error();
  if (!ctx) return fail(HC_EINVAL, "ctx is null");
  if (mode < 0 || mode > 2) return fail(HC_EINVAL, "split mode must be 0 (never), 1 (when it pays) or 2 (whenever possible)");
  ctx->split_mode = mode;
  return HC_OK;
}

hc_status hc_diag_split_plan(int32_t d_model, int32_t d_kv, int32_t n_tok, int32_t mode, int32_t* out_plan) {
  clear_error();
  if (!out_plan) return fail(HC_EINVAL, "null output pointer");
  if (d_model <= 0 || d_model % 64 != 0 || d_kv <= 0 || n_tok <= 0) return fail(HC_EINVAL, "bad shape");
  if (mode < 0 || mode > 2) return fail(HC_EINVAL, "split mode must be 0, 1 or 2");
  const int nf = 2 * round_up(d_kv, kPartAlign) / kTileF, nt = (n_tok + kTileT - 1) / kTileT;
  SplitPlan sp{};
  TileGrid g{};
  const bool split = mode != 0 && plan_split(nf, nt, d_model / (2 * kTileK), mode == 2, sp, g);
  out_plan[0] = split ? 1 : 0;
  out_plan[1] = nf;
  out_plan[2] = nt;
  out_plan[3] = split ? sp.nt_main : nt;
  out_plan[4] = split ? sp.n_tail : 0;
  out_plan[5] = split ? sp.n_split : 1;
  out_plan[6] = split ? sp.main_slots : 0;
  out_plan[7] = split ? sp.n_tail * kFixupPerTile : 0;
  return HC_OK;
}

hc_status hc_diag_tile_map(int32_t d_kv, int32_t n_tok, int32_t n_layers, int32_t* out_shape,
                           int32_t* out_tiles, int64_t out_capacity) {
  clear_error();
  if (!out_shape) return fail(HC_EINVAL, "null output pointer");
  if (d_kv <= 0 || n_tok <= 0 || n_layers <= 0 || n_layers > kMaxLayersPerLaunch)
    return fail(HC_EINVAL, "d_kv > 0, n_tok > 0, 1 <= n_layers <= 8");
  TileGrid g;
  const int slots = choose_tile_grid(2 * round_up(d_kv, kPartAlign) / kTileF, (n_tok + kTileT - 1) / kTileT, g);
  out_shape[0] = g.nf;
  out_shape[1] = g.nt;
  out_shape[2] = 1 << g.gf_shift;
  out_shape[3] = 1 << (g.g_shift - g.gf_shift);
  out_shape[4] = slots;
  out_shape[5] = 0;
  if (!out_tiles) return HC_OK;
  if (out_capacity < (int64_t)n_layers * slots) return fail(HC_ERANGE, "out_tiles too small");
  for (int l = 0; l < n_layers; ++l)
    for (int wg = 0; wg < slots; ++wg) {
      int tf, tt;
      // a launch over one layer passes no rotation, a launch over several the layer's index
      const bool ok = slot_to_tile(g, wg, n_layers > 1 ? l : 0, tf, tt);
      int32_t* o = out_tiles + ((int64_t)l * slots + wg) * 2;
      o[0] = ok ? tf : -1;
      o[1] = ok ? tt : -1;
    }
  return HC_OK;
}

hc_status hc_diag_mfma_duty(double period_us, double duty, int32_t half_phase, double total_us,
                            int32_t zero_operands, int32_t op_shape, double* out_tflops) {
  clear_error();
  if (!out_tflops) return fail(HC_EINVAL, "null output pointer");
  if (op_shape != 0 && op_shape != 1) return fail(HC_EINVAL, "op_shape: 0 (32x32x16) or 1 (16x16x32)");
  if (!(period_us >= 1.0) || !(duty > 0.0) || !(duty <= 1.0) || !(total_us >= period_us) || total_us > 2e6)
    return fail(HC_EINVAL, "period_us >= 1, 0 < duty <= 1, period_us <= total_us <= 2e6");
  HC_HIP(run_mfma_duty(period_us, duty, half_phase, total_us, zero_operands, op_shape, out_tflops));
  return HC_OK;
}

hc_status hc_timing_begin(hc_ctx* ctx) {
  clear_error();
  if (!ctx) return fail(HC_EINVAL, "ctx is null");
  ctx->timing = true;
  ctx->ev_used = 0;
  return HC_OK;
}

hc_status hc_timing_end_stats(hc_ctx* ctx, void* stream, double* out_avg_ms, double* out_min_ms,
                              double* out_median_ms, int32_t* out_launches) {
  clear_error();
  if (!ctx || !out_avg_ms || !out_launches) return fail(HC_EINVAL, "null argument");
  ctx->timing = false;
  HC_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  double total = 0.0;
  const int n = ctx->ev_used / 2;
  std::vector<float> all(n);
  for (int i = 0; i < n; ++i) {
    float ms = 0.f;
    HC_HIP(hipEventElapsedTime(&ms, ctx->ev_pool[2 * i], ctx->ev_pool[2 * i + 1]));
    all[i] = ms;
    total += ms;
  }
  std::sort(all.begin(), all.end());
  *out_launches = n;
  *out_avg_ms = n ? total / n : 0.0;
  if (out_min_ms) *out_min_ms = n ? all[0] : 0.0;
  if (out_median_ms) *out_median_ms = n ? (n % 2 ? all[n / 2] : 0.5 * (all[n / 2 - 1] + all[n / 2])) : 0.0;
  ctx->ev_used = 0;
  return HC_OK;
}

hc_status hc_timing_end(hc_ctx* ctx, void* stream, double* out_avg_ms, int32_t* out_launches) {
  return hc_timing_end_stats(ctx, stream, out_avg_ms, nullptr, nullptr, out_launches);
}

}  // extern "C"
