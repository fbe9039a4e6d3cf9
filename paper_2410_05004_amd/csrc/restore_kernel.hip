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
// registers).  The d_model loop advances 64 channels per step through two LDS stages of
// 64 KiB (32 KiB weights + 32 KiB activations); rows are 128 bytes and their 16-byte
// chunks are XOR-swizzled so that both the 16-byte LDS writes and the ds_read_b128
// fragment reads are bank-conflict free.
#include "hcache_internal.h"

namespace hc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kThreads = 256;
constexpr int kRowBytes = kTileK * 2;                    // 128
constexpr int kOperandBytes = 256 * kRowBytes;           // 32 KiB per operand per stage
constexpr int kStageBytes = 2 * kOperandBytes;           // 64 KiB
constexpr int kLdsBytes = 2 * kStageBytes;               // 128 KiB

// 16-byte chunk `chunk` (0..7) of LDS row `row` lives at chunk position chunk ^ f(row).
__device__ __forceinline__ int swizzle_of_row(int row) { return (row ^ (row >> 3)) & 7; }

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
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;               // wave position: features / tokens
  const int l32 = lane & 31, lh = lane >> 5;
  const int d = a.d_model;

  // ---- global -> LDS copy assignment: thread owns chunk lc of rows lr, lr+32, ...
  const int lr = tid >> 3, lc = tid & 7;
  const uint16_t* wsrc = a.wpack + (size_t)(tile_f * kTileF + lr) * d + lc * 8;
  const uint16_t* xsrc[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    int row = tile_t * kTileT + p * 32 + lr;
    row = row < a.n_tok ? row : a.n_tok - 1;             // ragged tail: re-read the last row
    xsrc[p] = a.hidden + (size_t)row * d + lc * 8;
  }
  int st_off[8];                                          // LDS byte offset inside an operand
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const int row = p * 32 + lr;
    st_off[p] = row * kRowBytes + ((lc ^ swizzle_of_row(row)) << 4);
  }

  // ---- LDS -> fragment read offsets (bytes inside an operand), per block and k sub-step
  // fragment: lane reads 8 consecutive channels (one 16-byte chunk) of row l32 of its block;
  // lanes 32..63 take the next chunk.
  int a_row_off[4], b_row_off[4], a_sw[4], b_sw[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ra = wm * 128 + i * 32 + l32, rb = wn * 128 + i * 32 + l32;
    a_row_off[i] = ra * kRowBytes; a_sw[i] = swizzle_of_row(ra);
    b_row_off[i] = rb * kRowBytes; b_sw[i] = swizzle_of_row(rb);
  }

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  float ss[4] = {0.f, 0.f, 0.f, 0.f};

  u32x4 wreg[8], xreg[8];
  const int nk = d / kTileK;

  // prologue: stage 0
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    wreg[p] = *reinterpret_cast<const u32x4*>(wsrc + (size_t)p * 32 * d);
    xreg[p] = *reinterpret_cast<const u32x4*>(xsrc[p]);
  }
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    *reinterpret_cast<u32x4*>(lds + st_off[p]) = wreg[p];
    *reinterpret_cast<u32x4*>(lds + kOperandBytes + st_off[p]) = xreg[p];
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const unsigned char* cur = lds + (kt & 1) * kStageBytes;
    unsigned char* nxt = lds + ((kt + 1) & 1) * kStageBytes;
    const bool more = kt + 1 < nk;
    if (more) {
      const int koff = (kt + 1) * kTileK;
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        wreg[p] = *reinterpret_cast<const u32x4*>(wsrc + (size_t)p * 32 * d + koff);
        xreg[p] = *reinterpret_cast<const u32x4*>(xsrc[p] + koff);
      }
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 af[4], bf[4];
      const int chunk = ks * 2 + lh;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        af[i] = *reinterpret_cast<const bf16x8*>(cur + a_row_off[i] + ((chunk ^ a_sw[i]) << 4));
        bf[i] = *reinterpret_cast<const bf16x8*>(cur + kOperandBytes + b_row_off[i] +
                                                 ((chunk ^ b_sw[i]) << 4));
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) ss[j] = sumsq8(bf[j], ss[j]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        *reinterpret_cast<u32x4*>(nxt + st_off[p]) = wreg[p];
        *reinterpret_cast<u32x4*>(nxt + kOperandBytes + st_off[p]) = xreg[p];
      }
    }
    __syncthreads();
  }

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
