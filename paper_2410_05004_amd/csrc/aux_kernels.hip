// One-time kernels: weight packing (per layer) and the RoPE (cos, sin) table (per context).
#include "hcache_internal.h"

namespace hc {

// ---- weight packing -------------------------------------------------------------------
// Physical row order of the packed weights [2 * d_kv_pad, d_model], d_kv_pad = d_kv rounded
// up to 128:
//   rows come in "pair groups" of 64; K groups and V groups alternate (K0 V0 K1 V1 ...), so
//   that every 128-row wave tile carries one K group (which needs RoPE) and one V group
//   (which does not) and all waves have the same amount of epilogue work.  Group g of a part
//   covers head g / (hd/64) and RoPE pair indices [32 qq, 32 qq + 32), qq = g % (hd/64);
//   groups at or beyond d_kv / 64 are zero padding.  The first 32 rows of a group are the
//   first members of those pairs, the last 32 rows the second members (half-split: features
//   i and i + hd/2; interleaved: features 2i and 2i + 1; V rows use the same order);
//   inside a 32-row block (two 16-row matrix-op blocks), row i maps to pair offset
//   u = 8*((i/4)%4) + 4*(i/16) + i%4: register v of lane quarter q of v_mfma_f32_16x16x32
//   holds block row 4*q + v, so a lane's registers of the two blocks are the 8 consecutive
//   pair offsets 8*q .. 8*q + 7 (one 16-byte store).
// Value: bf16( float(W[logical row][c]) * float(gamma[c]) ), one rounding.
// Memory order: tiles of 256 physical rows x 32 channels, [row tile][channel tile][row][32],
// each tile 16 KiB and laid out exactly as the restoration kernel wants it in LDS (the four
// 16-byte chunks of a row XOR-swizzled by swz_w), so a tile is fetched with fully
// contiguous 1 KiB wave loads.
__device__ __forceinline__ int logical_row(int p, int d_kv, int d_kv_pad, int hd, int style) {
  const int part = (p >> 6) & 1;                          // K and V groups alternate
  const int grp = p >> 7;
  if (grp * kPairGroup >= d_kv) return -1;                // padding
  const int member = (p >> 5) & 1, i = p & 31;
  const int u = 8 * ((i >> 2) & 3) + 4 * (i >> 4) + (i & 3);
  const int gph = hd >> 6;
  const int head = grp / gph, qq = grp - head * gph;
  const int pair = 32 * qq + u;
  // style 2 (no rotation) shares the half-split order
  const int f = style != 1 ? head * hd + member * (hd >> 1) + pair : head * hd + 2 * pair + member;
  return part * d_kv + f;
}

// bf16( W * gamma ), round to nearest even: the value the matrix cores multiply with
__device__ __forceinline__ uint16_t fold_gain(uint16_t w_bits, uint16_t g_bits) {
  const float prod = __uint_as_float((uint32_t)w_bits << 16) * __uint_as_float((uint32_t)g_bits << 16);
  uint32_t u = __float_as_uint(prod);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;     // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t* __restrict__ wkv,
                                                           const uint16_t* __restrict__ gamma,
                                                           uint16_t* __restrict__ wpack, int d_model,
                                                           int d_kv, int d_kv_pad, int hd, int style) {
  const int p = blockIdx.x;                               // physical row
  const int src = logical_row(p, d_kv, d_kv_pad, hd, style);
  for (int c = threadIdx.x; c < d_model; c += blockDim.x) {
    const uint16_t out = src >= 0 ? fold_gain(wkv[(size_t)src * d_model + c], gamma[c]) : (uint16_t)0;
    const int tile_f = p >> 8, r = p & 255, kt = c >> 5, chunk = (c >> 3) & 3, e = c & 7;
    const size_t tile = (size_t)tile_f * (d_model >> 5) + kt;
    wpack[tile * (kWTileBytes / 2) + r * 32 + ((chunk ^ swz_w(r)) << 3) + e] = out;
  }
}

hipError_t launch_pack_weights(const uint16_t* wkv, const uint16_t* gamma, uint16_t* wpack,
                               int d_model, int d_kv, int head_dim, int rope_style,
                               hipStream_t stream) {
  const int d_kv_pad = round_up(d_kv, kPartAlign);
  hipLaunchKernelGGL(pack_weights_kernel, dim3(2 * d_kv_pad), dim3(256), 0, stream, wkv, gamma,
                     wpack, d_model, d_kv, d_kv_pad, head_dim, rope_style);
  return hipGetLastError();
}

// Row constants of the affine variants (LayerNorm shift, projection bias), in fp64 and rounded
// once: S[n] = sum_c W'[n,c] over exactly the rounded values the pack kernel stores (so that
// mean * S cancels the mean's share of the accumulator), C[n] = sum_c W[n,c] beta[c] + bias[n].
__global__ __launch_bounds__(256) void pack_affine_kernel(const uint16_t* __restrict__ wkv,
                                                          const uint16_t* __restrict__ gamma,
                                                          const uint16_t* __restrict__ beta,
                                                          const uint16_t* __restrict__ bias,
                                                          float2* __restrict__ affine, int d_model,
                                                          int d_kv, int d_kv_pad, int hd, int style) {
  __shared__ double red[2][256];
  const int p = blockIdx.x;
  const int src = logical_row(p, d_kv, d_kv_pad, hd, style);
  double s = 0.0, c0 = 0.0;
  if (src >= 0) {
    for (int c = threadIdx.x; c < d_model; c += 256) {
      const uint16_t w = wkv[(size_t)src * d_model + c];
      s += (double)__uint_as_float((uint32_t)fold_gain(w, gamma[c]) << 16);
      if (beta) c0 += (double)__uint_as_float((uint32_t)w << 16) * (double)__uint_as_float((uint32_t)beta[c] << 16);
    }
  }
  red[0][threadIdx.x] = s;
  red[1][threadIdx.x] = c0;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      red[0][threadIdx.x] += red[0][threadIdx.x + w];
      red[1][threadIdx.x] += red[1][threadIdx.x + w];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    double c = red[1][0];
    if (src >= 0 && bias) c += (double)__uint_as_float((uint32_t)bias[src] << 16);
    affine[p] = make_float2((float)red[0][0], (float)c);
  }
}

hipError_t launch_pack_affine(const uint16_t* wkv, const uint16_t* gamma, const uint16_t* beta,
                              const uint16_t* bias, float2* affine, int d_model, int d_kv,
                              int head_dim, int rope_style, hipStream_t stream) {
  const int d_kv_pad = round_up(d_kv, kPartAlign);
  hipLaunchKernelGGL(pack_affine_kernel, dim3(2 * d_kv_pad), dim3(256), 0, stream, wkv, gamma, beta,
                     bias, affine, d_model, d_kv, d_kv_pad, head_dim, rope_style);
  return hipGetLastError();
}

// ---- RoPE table -----------------------------------------------------------------------
// table[p][i] = (cos, sin)(p * theta^(-2i/hd)), evaluated in fp64 and rounded once to fp32:
// an fp32 product p * inv_freq would already be off by ~2e-3 rad at position 32768.
__global__ __launch_bounds__(256) void rope_table_kernel(float2* __restrict__ table,
                                                         int max_position, int half, double theta,
                                                         double inv_hd) {
  const long n = (long)max_position * half;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < n;
       e += (long)gridDim.x * blockDim.x) {
    const int p = (int)(e / half), i = (int)(e - (long)p * half);
    const double inv_freq = pow(theta, -2.0 * (double)i * inv_hd);
    double s, c;
    sincos((double)p * inv_freq, &s, &c);
    table[e] = make_float2((float)c, (float)s);
  }
}

hipError_t launch_rope_table(float2* table, int max_position, int head_dim, double theta,
                             hipStream_t stream) {
  const int half = head_dim / 2;
  const long n = (long)max_position * half;
  if (n == 0) return hipSuccess;
  const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  hipLaunchKernelGGL(rope_table_kernel, dim3(blocks), dim3(256), 0, stream, table, max_position,
                     half, theta, 1.0 / (double)head_dim);
  return hipGetLastError();
}

// ---- chunk gather ---------------------------------------------------------------------
// Host->HBM loader of the pipelined restore (paper Section 5, "Pipelined state
// transmission"): the chunks of one layer sit at arbitrary places of the pinned host arena.
// A few workgroups read them over the host link with 16-byte loads (several in flight per
// lane) and write the staging buffer; measured at the link's full rate, which a sequence of
// per-chunk hipMemcpyAsync calls does not reach.  Each segment is served by
// kGatherBlocksPerSegment workgroups, each taking an interleaved share of its 16-byte words.
typedef __attribute__((ext_vector_type(4))) uint32_t gather_vec;

__global__ __launch_bounds__(256) void gather_segments_kernel(const CopySegment* __restrict__ segs,
                                                              int n_seg) {
  const int seg = blockIdx.x / kGatherBlocksPerSegment;
  const int share = blockIdx.x - seg * kGatherBlocksPerSegment;
  if (seg >= n_seg) return;
  const gather_vec* src = static_cast<const gather_vec*>(segs[seg].src);
  gather_vec* dst = static_cast<gather_vec*>(segs[seg].dst);
  const long n = (long)(segs[seg].bytes >> 4);
  const long stride = (long)kGatherBlocksPerSegment * 256;
  for (long i = (long)share * 256 + threadIdx.x; i < n; i += 4 * stride) {
    gather_vec v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * stride < n) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * stride < n) dst[i + u * stride] = v[u];
  }
}

hipError_t launch_gather(const CopySegment* segs, int n_seg, hipStream_t stream) {
  if (n_seg <= 0) return hipSuccess;
  hipLaunchKernelGGL(gather_segments_kernel, dim3(n_seg * kGatherBlocksPerSegment), dim3(256), 0,
                     stream, segs, n_seg);
  return hipGetLastError();
}

// ---- KV rows <-> paged pool --------------------------------------------------------------
// The KV-offload complement of the bubble-free scheduler (paper Section 4.1.2): layers that
// are not restored from hidden states keep their KV cache on the host as token rows
// [n_tok][K row | V row] (2 * d_kv bf16, K already rotated).  TO_POOL copies such rows into
// the pages the block table names (restoration); otherwise pages are read out into rows
// (saving).  Pure byte movement, one 16-byte word per lane; a row with an invalid position
// or page is skipped and raises the same sticky flags as the fused kernel.
template <bool TO_POOL>
__global__ __launch_bounds__(256) void kv_rows_kernel(KvRowsArgs a) {
  const int vec_per_part = a.d_kv >> 3;                // 16-byte words per K (or V) row
  const int vec_per_row = 2 * vec_per_part;
  const long total = (long)a.n_tok * vec_per_row;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
    const int t = (int)(i / vec_per_row);
    const int j = (int)(i - (long)t * vec_per_row);
    const int part = j >= vec_per_part;                // 0 = K, 1 = V
    const int jj = j - part * vec_per_part;
    const int pos = a.positions ? a.positions[t] : a.pos_base + t;
    if (pos < 0 || pos >= a.max_position || (pos >> a.block_shift) >= a.n_blocks) {
      if (j == 0) atomicOr(a.err, HC_DEV_BAD_POSITION);
      continue;
    }
    const long page = a.block_table[pos >> a.block_shift];
    if (page < 0 || page >= a.num_pages) {
      if (j == 0) atomicOr(a.err, HC_DEV_BAD_PAGE);
      continue;
    }
    const int slot = pos & ((1 << a.block_shift) - 1);
    const long rows_per_page = 2L << a.block_shift;
    gather_vec* in_pool = reinterpret_cast<gather_vec*>(a.pool) +
        ((page * rows_per_page + ((long)part << a.block_shift) + slot) * vec_per_part + jj);
    gather_vec* in_rows = reinterpret_cast<gather_vec*>(a.rows) + i;
    if (TO_POOL) *in_pool = __builtin_nontemporal_load(in_rows);
    else *in_rows = *in_pool;
  }
}

hipError_t launch_kv_rows(const KvRowsArgs& a, bool to_pool, hipStream_t stream) {
  if (a.n_tok <= 0) return hipSuccess;
  const long total = (long)a.n_tok * (a.d_kv >> 2);
  long blocks = (total + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (to_pool)
    hipLaunchKernelGGL(kv_rows_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, a);
  else
    hipLaunchKernelGGL(kv_rows_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ---- matrix-pipe duty-cycle probe (measurement only) -----------------------------------------
// Every CU runs bursts of v_mfma_f32_32x32x16_bf16 or v_mfma_f32_16x16x32_bf16 (the restoration kernel's op)
// on register operands (eight waves, two per SIMD, 128 accumulator registers each) gated by the constant-rate wall clock: busy while
// (t mod period) < busy, asleep otherwise; with `half_phase` odd workgroups are busy in the
// other half of the period.  The matrix ops issued inside the busy windows are counted.
// If the chip's power management averaged over time, a 50 % duty cycle would let the busy
// windows run faster than a continuous run; if it follows the instantaneous activity of the
// whole chip, they run at the continuous rate -- and faster only when half the CUs are idle at
// any moment.
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t probe_u32x4;

typedef __attribute__((ext_vector_type(4))) float probe_f32x4;

// SHAPE 0: 32 ops 32x32x16 per batch (8 accumulator blocks of 16 registers);
// SHAPE 1: 64 ops 16x16x32 per batch (16 accumulator blocks of 4 registers): the same flop.
template <int SHAPE>
__global__ __launch_bounds__(512) void mfma_duty_kernel(const probe_u32x4* __restrict__ ops,
                                                        float* __restrict__ sink,
                                                        unsigned long long period_ticks,
                                                        unsigned long long busy_ticks,
                                                        unsigned long long total_ticks, int half_phase,
                                                        unsigned long long* __restrict__ batches_out) {
  probe_f32x16 acc[8];
  probe_f32x4 acc4[16];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc4[i][v] = 0.f;
  probe_bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(probe_bf16x8, ops[(threadIdx.x * 8 + i) & 2047]);
#pragma unroll
  for (int i = 0; i < 4; ++i) b[i] = __builtin_bit_cast(probe_bf16x8, ops[(threadIdx.x * 8 + 4 + i) & 2047]);
  const unsigned long long t_begin = wall_clock64();      // 100 MHz
  const unsigned long long phase = (half_phase && (blockIdx.x & 1)) ? period_ticks / 2 : 0;
  unsigned long long batches = 0;
  for (;;) {                                              // every wave leaves after total_ticks
    const unsigned long long t = wall_clock64();
    if (t - t_begin >= total_ticks) break;
    if (((t + phase) % period_ticks) < busy_ticks) {
      for (int it = 0; it < 4; ++it) {                    // one batch = 32 * 32768 flop per wave
        if constexpr (SHAPE == 0) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
              acc[i * 2 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i * 2 + j], 0, 0, 0);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
              acc4[i * 4 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc4[i * 4 + j], 0, 0, 0);
        }
      }
      ++batches;
    } else {
      __builtin_amdgcn_s_sleep(32);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) s += acc4[i][v];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if ((threadIdx.x & 63) == 0) batches_out[blockIdx.x * 8 + (threadIdx.x >> 6)] = batches;
}

hipError_t run_mfma_duty(double period_us, double duty, int half_phase, double total_us,
                         int zero_operands, int op_shape, double* out_tflops) {
  const int n_wg = 256, n_waves = n_wg * 8;
  probe_u32x4* ops = nullptr;
  float* sink = nullptr;
  unsigned long long* batches = nullptr;
  std::vector<uint32_t> h(2048 * 4);
  uint32_t x = 0x9E3779B9u;                               // xorshift: random signs and mantissas,
  for (uint32_t& w : h) {                                 // exponents of values near 1
    uint32_t halves[2];
    for (uint32_t& half : halves) {
      x ^= x << 13; x ^= x >> 17; x ^= x << 5;
      half = (x & 0x807Fu) | ((0x7Eu + (x >> 20) % 3u) << 7);
    }
    w = zero_operands ? 0u : (halves[1] << 16) | halves[0];
  }
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&ops), h.size() * 4);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&sink), (size_t)n_wg * 512 * 4);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&batches), (size_t)n_waves * 8);
  if (e == hipSuccess) e = hipMemcpy(ops, h.data(), h.size() * 4, hipMemcpyHostToDevice);
  std::vector<unsigned long long> hb(n_waves);
  if (e == hipSuccess) {
    const unsigned long long P = (unsigned long long)(period_us * 100.0);
    const unsigned long long B = (unsigned long long)(period_us * 100.0 * duty);
    const unsigned long long T = (unsigned long long)(total_us * 100.0);
    for (int rep = 0; rep < 2 && e == hipSuccess; ++rep) {   // the first run warms up
      if (op_shape == 0)
        hipLaunchKernelGGL(mfma_duty_kernel<0>, dim3(n_wg), dim3(512), 0, nullptr, ops, sink, P ? P : 1, B, T,
                           half_phase, batches);
      else
        hipLaunchKernelGGL(mfma_duty_kernel<1>, dim3(n_wg), dim3(512), 0, nullptr, ops, sink, P ? P : 1, B, T,
                           half_phase, batches);
      e = hipGetLastError();
      if (e == hipSuccess) e = hipDeviceSynchronize();
    }
    if (e == hipSuccess) e = hipMemcpy(hb.data(), batches, hb.size() * 8, hipMemcpyDeviceToHost);
  }
  if (e == hipSuccess) {
    double n = 0;
    for (unsigned long long v : hb) n += (double)v;
    // flop issued inside busy windows / time the windows were open (per CU: duty * total)
    *out_tflops = n * 32.0 * 32768.0 / (duty * total_us * 1e-6) / 1e12;
  }
  if (ops) (void)hipFree(ops);
  if (sink) (void)hipFree(sink);
  if (batches) (void)hipFree(batches);
  return e;
}

}  // namespace hc
