// Fused restoration kernel for gfx950 (MI355X): RMSNorm -> K|V projection -> RoPE(K) ->
// bf16 -> paged scatter, one launch per layer (paper Section 3.1 equations; Section 5:
// GEMM followed by the RoPE + copy-to-KV-cache step; Section 6: paged KV cache).
//
// Formulation.  With g the RMSNorm gain and r_t = 1/sqrt(mean_c x[t,c]^2 + eps),
//     y[t,n] = sum_c (x[t,c] r_t g[c]) W[n,c] = r_t * sum_c x[t,c] (g[c] W[n,c]).
// The gain is folded into the packed weights once per layer; the per-token scale r_t is
// a scalar that commutes with the contraction, so it is accumulated from the same
// activation fragments that feed the matrix cores and applied to the fp32 accumulators
// afterwards.  The normalised activations therefore never exist in memory.
//
// Operand roles.  The packed weights are the MFMA "A" operand (rows = output features),
// the hidden states are the "B" operand (columns = tokens).  With
// v_mfma_f32_32x32x16_bf16 a lane then owns ONE token (column lane%32) and 16 features
// of each 32x32 block, which makes everything per-token in the epilogue (r_t, position,
// page, slot) a per-lane scalar.  The packing order of the weight rows (pack kernel)
// makes those 16 features consecutive in the cache row and puts the two members of
// every RoPE pair into the same lane and register index of two neighbouring blocks.
//
// Tiling.  Workgroup = 256 threads = 4 waves in a 2x2 arrangement; workgroup tile =
// 256 features x 256 tokens, wave tile = 128 x 128 (4x4 MFMA blocks, 256 accumulator
// registers).  The d_model loop advances 32 channels per step through a ring of four LDS
// stages of 32 KiB (16 KiB weights + 16 KiB activations) filled by direct global->LDS
// loads issued four tiles ahead; rows are 64 bytes and their 16-byte chunks are
// XOR-swizzled (on the global address side, since a direct load fills LDS lane by lane)
// so that the ds_read_b128 fragment reads are bank-conflict free.
#include "hcache_internal.h"

namespace hc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kThreads = 256;
constexpr int kStages = 4;                               // LDS ring depth (tiles in flight)
constexpr int kRowBytes = kTileK * 2;                    // 64
constexpr int kOperandBytes = 256 * kRowBytes;           // 16 KiB per operand per stage
constexpr int kStageBytes = 2 * kOperandBytes;           // 32 KiB
constexpr int kLdsBytes = kStages * kStageBytes;         // 128 KiB
static_assert(kTileK == 32, "the waitcnt constants below assume 8 direct loads per thread per tile");

// 16-byte chunk `chunk` (0..3) of LDS row `row` lives at chunk position chunk ^ f(row); f is
// chosen so that the 16 (or 8) consecutive rows one ds_read_b128 pass touches fall into
// distinct banks whether the LDS serves 64 or 32 banks per clock.
__device__ __forceinline__ int swizzle_of_row(int row) { return ((row >> 1) ^ (row >> 3)) & 3; }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);         // round to nearest even
  return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ float sumsq8(bf16x8 v, float acc) {
  const bf16x2 p0 = {v[0], v[1]}, p1 = {v[2], v[3]}, p2 = {v[4], v[5]}, p3 = {v[6], v[7]};
  acc = __builtin_amdgcn_fdot2_f32_bf16(p0, p0, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(p1, p1, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(p2, p2, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(p3, p3, acc, false);
  return acc;
}

// 16 bytes per lane straight from global memory into LDS (no registers): the wave's 64
// lanes fill 1 KiB starting at the wave-uniform LDS address `lds_wave_base`, lane i at
// byte 16*i.  Completion is tracked by vmcnt.
__device__ __forceinline__ void load_to_lds_16(const void* gptr, unsigned char* lds_wave_base) {
  __builtin_amdgcn_global_load_lds(
      (const __attribute__((address_space(1))) void*)gptr,
      (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// Tile scheduling.  Workgroup ids are handed to the 8 XCDs round-robin and every XCD has
// its own L2, so the tiles one XCD works on at the same time should share weight rows
// and token rows.  The tile grid is cut into super tiles of GF x GT = 32 tiles; super
// tile k belongs to XCD k % 8.  Workgroups that fall outside the grid exit at once.
struct TileGrid {
  int nf, nt;        // tiles along features / tokens
  int gf_shift;      // log2(GF); GT = 32 >> gf_shift
  int nsf;           // super tiles along features
};

template <int STYLE>
__global__ __launch_bounds__(kThreads) void restore_kernel(const RestoreArgs a, const TileGrid g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  // ---- which tile
  const int wg = blockIdx.x;
  const int xcd = wg & 7, li = wg >> 3;
  const int super = (li >> 5) * 8 + xcd, r = li & 31;
  const int tile_f = (super % g.nsf) * (1 << g.gf_shift) + (r & ((1 << g.gf_shift) - 1));
  const int tile_t = (super / g.nsf) * (32 >> g.gf_shift) + (r >> g.gf_shift);
  if (tile_f >= g.nf || tile_t >= g.nt) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;               // wave position: features / tokens
  const int l32 = lane & 31, lh = lane >> 5;
  const int d = a.d_model;

  // ---- global -> LDS assignment.  One wave instruction fills 16 rows x 64 bytes; wave w
  // issues instructions q = 0..3 for rows (4w + q) * 16 .. + 15 of each operand.  Lane i
  // writes chunk position i & 3 of row i >> 2, so it fetches logical chunk (i & 3) ^ f(row).
  // Addresses are a wave-uniform base (advanced by 64 bytes per step with scalar adds) plus a
  // per-lane 32-bit offset that never changes.
  const unsigned char* wbase =
      reinterpret_cast<const unsigned char*>(a.wpack) + (size_t)tile_f * kTileF * d * 2;
  const unsigned char* xbase =
      reinterpret_cast<const unsigned char*>(a.hidden) + (size_t)tile_t * kTileT * d * 2;
  uint32_t woff[4], xoff[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int row = (wave * 4 + q) * 16 + (lane >> 2);
    const int chunk = (lane & 3) ^ swizzle_of_row(row);
    woff[q] = ((uint32_t)row * d + chunk * 8) * 2;
    const int last = a.n_tok - 1 - tile_t * kTileT;      // ragged tail: re-read the last row
    xoff[q] = ((uint32_t)(row < last ? row : last) * d + chunk * 8) * 2;
  }
  const int nk = d / kTileK;
  // One direct load (n = 0..7) of tile kt: even n -> weight rows, odd n -> token rows.
  // Tiles past the end re-read the last one: the load count per step stays uniform and
  // the data is never consumed.
  auto issue_load = [&](int kt, int n) {
    const int kk = kt < nk ? kt : nk - 1;
    unsigned char* stage = lds + (kt & (kStages - 1)) * kStageBytes + wave * 4096;
    const size_t koff = (size_t)kk * (kTileK * 2);
    const int q = n >> 1;
    if (n & 1) load_to_lds_16(xbase + koff + xoff[q], stage + kOperandBytes + q * 1024);
    else       load_to_lds_16(wbase + koff + woff[q], stage + q * 1024);
  };

  // ---- LDS -> fragment read offsets.  A fragment is 8 consecutive channels (one 16-byte
  // chunk) of row l32 of a 32-row block; lanes 32..63 take the next chunk.  f(row) is the
  // same for the four blocks of a wave (block stride 32 rows).
  const int fl = swizzle_of_row(l32);
  int a_off[2], b_off[2];                                // per k sub-step
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int pc = ((ks * 2 + lh) ^ fl) << 4;
    a_off[ks] = (wm * 128 + l32) * kRowBytes + pc;
    b_off[ks] = kOperandBytes + (wn * 128 + l32) * kRowBytes + pc;
  }
  // Fragment n = 0..7 of (tile kt, sub-step ks), in the order the matrix ops consume them:
  // A0 B0 B1 B2 B3 A1 A2 A3.
  auto read_frag = [&](int kt, int ks, int n, bf16x8 (&af)[4], bf16x8 (&bf)[4]) {
    const unsigned char* stage = lds + (kt & (kStages - 1)) * kStageBytes;
    if (n == 0)      af[0] = *reinterpret_cast<const bf16x8*>(stage + a_off[ks]);
    else if (n <= 4) bf[n - 1] = *reinterpret_cast<const bf16x8*>(stage + b_off[ks] + (n - 1) * 32 * kRowBytes);
    else             af[n - 4] = *reinterpret_cast<const bf16x8*>(stage + a_off[ks] + (n - 4) * 32 * kRowBytes);
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  float ss[4] = {0.f, 0.f, 0.f, 0.f};

  // ---- pipeline.  Stage kt % 4 holds tile kt.  Per step one barrier, placed after the
  // fragments of the tile's second half are in registers: past it, the tile's stage is
  // free (refilled with tile kt + 4) and tile kt + 1 is visible to every wave.
  // The issue order is written out by hand and pinned with scheduling fences: every
  // matrix op is followed by at most one LDS read or one global->LDS load plus the
  // sum-of-squares dot products, so the matrix pipe never waits for the other ports.
  bf16x8 af0[4], bf0[4], af1[4], bf1[4];
#pragma unroll
  for (int s = 0; s < kStages; ++s)
#pragma unroll
    for (int n = 0; n < 8; ++n) issue_load(s, n);
  asm volatile("s_waitcnt vmcnt(24)" ::: "memory");      // tile 0 landed (3 x 8 loads may be in flight)
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int n = 0; n < 8; ++n) read_frag(0, 0, n, af0, bf0);

  for (int kt = 0; kt < nk; ++kt) {
    // phase A: matrix ops on the first half (fragments already in registers) while the
    // second half's fragments stream in from LDS
#pragma unroll
    for (int n = 0; n < 16; ++n) {
      const int i = n >> 2, j = n & 3;
      if (n < 8) read_frag(kt, 1, n, af1, bf1);
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af0[i], bf0[j], acc[i][j], 0, 0, 0);
      if (n < 4) ss[n] = sumsq8(bf0[n], ss[n]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // tiles kt+2, kt+3 may still be in flight (2 x 8 loads); tile kt+1 must have landed
    asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // phase B: matrix ops on the second half while the first fragments of tile kt + 1
    // stream in and the stage just consumed is refilled with tile kt + 4
#pragma unroll
    for (int n = 0; n < 16; ++n) {
      const int i = n >> 2, j = n & 3;
      if (n < 8) read_frag(kt + 1, 0, n, af0, bf0);
      else       issue_load(kt + kStages, n - 8);
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af1[i], bf1[j], acc[i][j], 0, 0, 0);
      if (n < 4) ss[n] = sumsq8(bf1[n], ss[n]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");   // drain the look-ahead loads
  __syncthreads();

  // ---- epilogue: everything per token is per lane
  const int wave_f0 = tile_f * kTileF + wm * 128;         // first physical weight row of the wave
  const int part = wave_f0 >= a.d_kv_pad ? 1 : 0;         // 0 = K rows, 1 = V rows (wave-uniform)
  const int part_f0 = wave_f0 - part * a.d_kv_pad;
  const int hd = a.head_dim, half = hd >> 1, groups_per_head = hd >> 6;
  const int bmask = (1 << a.block_shift) - 1;

#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int t = tile_t * kTileT + wn * 128 + j * 32 + l32;
    const float s = ss[j] + __shfl_xor(ss[j], 32);        // the two lane halves hold different channels
    const float rstd = rsqrtf(s * a.inv_d + a.eps);
    if (t >= a.n_tok) continue;
    const int pos = a.positions ? a.positions[t] : a.pos_base + t;
    int seq = 0;
    if (a.cu_seqlens) {                                   // largest s with cu[s] <= t
      int lo = 0, hi = a.n_seq;                           // invariant: cu[lo] <= t < cu[hi]
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.cu_seqlens[mid] <= t) lo = mid; else hi = mid;
      }
      seq = lo;
    }
    const int blk = pos >> a.block_shift;
    if (pos < 0 || pos >= a.max_position || blk >= a.max_blocks) {
      atomicOr(a.err, HC_DEV_BAD_POSITION);
      continue;
    }
    const int page = a.block_tables[(size_t)seq * a.max_blocks + blk];
    if (page < 0 || page >= a.num_pages) {
      atomicOr(a.err, HC_DEV_BAD_PAGE);
      continue;
    }
    uint16_t* dst_row = a.pool +
        ((((size_t)page * 2 + part) << a.block_shift) + (size_t)(pos & bmask)) * a.d_kv;
    const float2* rope_row = a.rope + (size_t)pos * half;

#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int grp = (part_f0 >> 6) + q;                 // pair group inside the K or V part
      if (grp * kPairGroup >= a.d_kv) continue;           // padding rows (wave-uniform)
      const int head = grp / groups_per_head, qq = grp - head * groups_per_head;
      const int i0 = 32 * qq + 16 * lh;                   // first RoPE pair index of this lane
      float oa[16], ob[16];
      if (part == 0) {
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
          const float4 cs = *reinterpret_cast<const float4*>(rope_row + i0 + v);
          const float a0 = acc[2 * q][j][v] * rstd, b0 = acc[2 * q + 1][j][v] * rstd;
          const float a1 = acc[2 * q][j][v + 1] * rstd, b1 = acc[2 * q + 1][j][v + 1] * rstd;
          oa[v] = a0 * cs.x - b0 * cs.y;
          ob[v] = b0 * cs.x + a0 * cs.y;
          oa[v + 1] = a1 * cs.z - b1 * cs.w;
          ob[v + 1] = b1 * cs.z + a1 * cs.w;
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          oa[v] = acc[2 * q][j][v] * rstd;
          ob[v] = acc[2 * q + 1][j][v] * rstd;
        }
      }
      if (STYLE == 0) {
        // first member at head*hd + i, second at head*hd + hd/2 + i
        u32x4* da = reinterpret_cast<u32x4*>(dst_row + head * hd + i0);
        u32x4* db = reinterpret_cast<u32x4*>(dst_row + head * hd + half + i0);
        u32x4 w0, w1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          w0[e] = pack_bf16x2(oa[2 * e], oa[2 * e + 1]);
          w1[e] = pack_bf16x2(oa[8 + 2 * e], oa[8 + 2 * e + 1]);
        }
        da[0] = w0; da[1] = w1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          w0[e] = pack_bf16x2(ob[2 * e], ob[2 * e + 1]);
          w1[e] = pack_bf16x2(ob[8 + 2 * e], ob[8 + 2 * e + 1]);
        }
        db[0] = w0; db[1] = w1;
      } else {
        // members of pair i at head*hd + 2i and 2i + 1: interleave the two blocks
        u32x4* dq = reinterpret_cast<u32x4*>(dst_row + head * hd + 2 * i0);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          u32x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(oa[4 * c + e], ob[4 * c + e]);
          dq[c] = w;
        }
      }
    }
  }
}

hipError_t configure_kernels() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(restore_kernel<0>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(restore_kernel<1>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
}

hipError_t launch_restore(const RestoreArgs& a, hipStream_t stream) {
  if (a.n_tok <= 0) return hipSuccess;
  TileGrid g;
  g.nf = 2 * a.d_kv_pad / kTileF;
  g.nt = (a.n_tok + kTileT - 1) / kTileT;
  // super tile shape: as close to square as the feature extent allows (8x4, 4x8, 2x16, 1x32)
  g.gf_shift = g.nf >= 8 ? 3 : g.nf >= 4 ? 2 : g.nf >= 2 ? 1 : 0;
  const int gf = 1 << g.gf_shift, gt = 32 >> g.gf_shift;
  g.nsf = (g.nf + gf - 1) / gf;
  const int nst = (g.nt + gt - 1) / gt;
  const int n_super = g.nsf * nst;
  const int rounds = (n_super + 7) / 8;                   // super tiles per XCD
  const unsigned grid = (unsigned)rounds * 8u * 32u;
  if (a.rope_style == 0)
    hipLaunchKernelGGL(restore_kernel<0>, dim3(grid), dim3(kThreads), kLdsBytes, stream, a, g);
  else
    hipLaunchKernelGGL(restore_kernel<1>, dim3(grid), dim3(kThreads), kLdsBytes, stream, a, g);
  return hipGetLastError();
}

}  // namespace hc
