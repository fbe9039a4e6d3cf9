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
// makes those 16 features consecutive in the cache row, puts the two members of every
// RoPE pair into the same lane and register index of two neighbouring blocks, and
// alternates K and V row groups so that every wave has one of each.
//
// Tiling.  Workgroup = 512 threads = 8 waves, two per SIMD, arranged 2 (features) x 4
// (tokens); workgroup tile = 256 features x 256 tokens, wave tile = 128 x 64 (4x2 MFMA
// blocks, 128 accumulator registers).  Two waves share a SIMD on purpose: a wave cannot
// issue anything else while one of its matrix ops occupies the pipe, so the LDS reads,
// global loads and vector ALU work of one wave run in the shadow of the other wave's
// matrix ops.  The d_model loop advances 32 channels per step.  Operands reach LDS by
// direct global->LDS loads (no registers) that are issued several steps ahead:
//   * weights: ring of four 16 KiB stages, one packed tile each (256 rows x 64 bytes); the
//     pack kernel stores tiles contiguously in LDS order, so a wave load is 1 KiB contiguous;
//   * activations: ring of three 32 KiB super-stages of 256 token rows x 128 bytes (two steps'
//     worth of channels), so that every row fetch is one full 128-byte line; a super-stage is
//     refilled in two halves over the two steps after it has been consumed.
// 96 + 64 = 160 KiB, the whole LDS of a CU.  The 16-byte chunks of every row are
// XOR-swizzled (for activations on the global-address side, since a direct load fills LDS
// lane by lane) so that the ds_read_b128 fragment reads are bank-conflict free.
#include <type_traits>

#include "hcache_internal.h"

namespace hc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kThreads = 512;
constexpr int kWStages = 4;                              // weight ring depth (steps)
constexpr int kXStages = 3;                              // activation ring depth (double steps)
constexpr int kWStageBytes = kWTileBytes;                // 16 KiB
constexpr int kXRowBytes = 4 * kTileK;                   // 128: two steps' worth of channels
constexpr int kXStageBytes = kTileT * kXRowBytes;        // 32 KiB
constexpr int kXRegion = kXStages * kXStageBytes;        // activations at LDS offset 0
constexpr int kLdsBytes = kXRegion + kWStages * kWStageBytes;   // 160 KiB
static_assert(kTileK == 32 && kTileF == 256 && kTileT == 256, "load counts below assume these");

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);         // round to nearest even
  return __builtin_bit_cast(uint32_t, b);
}

// acc + x0^2 + x1^2 for element pair `pair` (0..3) of a fragment, with ordinary fp32 ALU ops
// (a bf16 is the upper half of an fp32).  The packed-dot instruction is avoided on purpose:
// it competes with the matrix ops for their pipe, plain VALU ops run beside them.
__device__ __forceinline__ float sumsq2(bf16x8 v, int pair, float acc) {
  const uint32_t w = __builtin_bit_cast(u32x4, v)[pair];
  const float lo = __uint_as_float(w << 16), hi = __uint_as_float(w & 0xffff0000u);
  return __builtin_fmaf(hi, hi, __builtin_fmaf(lo, lo, acc));
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
// and token rows.  The tile grid is cut into super tiles of GF x GT tiles (powers of two,
// GF * GT <= 32 = the CUs of an XCD); super tile k belongs to XCD k % 8.  The host picks the
// shape that keeps the XCDs evenly loaded first and shares the most rows second.
// Workgroups that fall outside the grid exit at once.
struct TileGrid {
  int nf, nt;        // tiles along features / tokens
  int gf_shift;      // log2(GF)
  int g_shift;       // log2(GF * GT)
  int nsf;           // super tiles along features
};

template <int STYLE>
__global__ __launch_bounds__(kThreads) void restore_kernel(const RestoreArgs a, const TileGrid g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  // ---- which tile
  const int wg = blockIdx.x;
  const int xcd = wg & 7, li = wg >> 3;
  const int super = (li >> g.g_shift) * 8 + xcd, r = li & ((1 << g.g_shift) - 1);
  const int tile_f = (super % g.nsf) * (1 << g.gf_shift) + (r & ((1 << g.gf_shift) - 1));
  const int tile_t = ((super / g.nsf) << (g.g_shift - g.gf_shift)) + (r >> g.gf_shift);
  if (tile_f >= g.nf || tile_t >= g.nt) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;               // wave position: features (2) / tokens (4)
  const int l32 = lane & 31, lh = lane >> 5;
  const int d = a.d_model;

  const int nk = d / kTileK;                             // steps (even: d_model % 64 == 0)
  const int nm = nk >> 1;                                // activation super-tiles

  // ---- global -> LDS assignment.
  // Weights: tile (tile_f, kt) is 16 KiB contiguous; wave w copies KiB 2w, 2w+1 of it.
  const unsigned char* wtiles = reinterpret_cast<const unsigned char*>(a.wpack) +
                                (size_t)tile_f * nk * kWTileBytes + wave * 2048;
  const uint32_t wlane = lane * 16;
  // Activations: one wave load covers 8 token rows x 128 bytes.  Load g = 0..31 of a
  // super-tile covers rows 8g .. 8g+7; wave w issues g = 16*half + 2w + q.  Lane i fills
  // chunk position i & 7 of row i >> 3, so it fetches logical chunk (i & 7) ^ swz_x(row).
  const unsigned char* xbase =
      reinterpret_cast<const unsigned char*>(a.hidden) + (size_t)tile_t * kTileT * d * 2;
  uint32_t xoff[4];
  {
    const int last = a.n_tok - 1 - tile_t * kTileT;      // ragged tail: re-read the last row
#pragma unroll
    for (int hq = 0; hq < 4; ++hq) {
      const int g = (hq >> 1) * 16 + wave * 2 + (hq & 1);
      const int row = g * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ swz_x(row);
      xoff[hq] = (uint32_t)(row < last ? row : last) * d * 2 + chunk * 16;
    }
  }
  // Loads past the end of d_model re-read the last tile: the load count per step stays
  // uniform (the vmcnt waits below count loads) and that data is never consumed.
  auto load_w = [&](int kt, int q) {                     // half q of this wave's share of tile kt
    const int kk = kt < nk ? kt : nk - 1;
    load_to_lds_16(wtiles + (size_t)kk * kWTileBytes + q * 1024 + wlane,
                   lds + kXRegion + (kt & (kWStages - 1)) * kWStageBytes + wave * 2048 + q * 1024);
  };
  auto load_x = [&](int m, int stage, int half, int q) { // super-tile m -> super-stage `stage`
    const int mm = m < nm ? m : nm - 1;
    load_to_lds_16(xbase + (size_t)mm * kXRowBytes + xoff[half * 2 + q],
                   lds + stage * kXStageBytes + (half * 16 + wave * 2 + q) * 1024);
  };

  // ---- LDS -> fragment reads.  A fragment is 8 consecutive channels (one 16-byte chunk) of
  // row l32 of a 32-row block; lanes 32..63 take the next chunk.  The swizzle term is the
  // same for all blocks of a wave (block stride 32 rows).
  int a_off[2], b_off[2][2];                             // [k sub-step], [step parity][k sub-step]
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    a_off[ks] = kXRegion + (wm * 128 + l32) * (kTileK * 2) + (((ks * 2 + lh) ^ swz_w(l32)) << 4);
#pragma unroll
    for (int par = 0; par < 2; ++par)
      b_off[par][ks] = (wn * 64 + l32) * kXRowBytes + (((par * 4 + ks * 2 + lh) ^ swz_x(l32)) << 4);
  }
  // Fragment n = 0..5 of (step kt, sub-step ks), in the order the matrix ops consume them:
  // A0 B0 B1 A1 A2 A3.  `xs` is the super-stage holding step kt's activations.
  auto read_frag = [&](int kt, int xs, int par, int ks, int n, bf16x8 (&af)[4], bf16x8 (&bf)[2]) {
    const unsigned char* wst = lds + (kt & (kWStages - 1)) * kWStageBytes + a_off[ks];
    const unsigned char* xst = lds + xs * kXStageBytes + b_off[par][ks];
    if (n == 0)      af[0] = *reinterpret_cast<const bf16x8*>(wst);
    else if (n <= 2) bf[n - 1] = *reinterpret_cast<const bf16x8*>(xst + (n - 1) * 32 * kXRowBytes);
    else             af[n - 2] = *reinterpret_cast<const bf16x8*>(wst + (n - 2) * 32 * (kTileK * 2));
  };

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // sum of squares of the token column this wave is responsible for: the two waves that
  // share a token range (wm = 0, 1) split its two 32-token blocks between them
  float ssum = 0.f;

  bf16x8 af0[4], bf0[2], af1[4], bf1[2];

  // ---- prologue (18 loads per thread): W0 X0 | W1 X1 | W2 W3 X2(first half), with the
  // per-token lookups slotted in so that their memory latency hides behind the tile loads.
  // Lane l32 owns token column l32 of each of its two 32-token blocks: position, (ragged)
  // context and page are fetched here; the pool row is worked out after the main loop.
#pragma unroll
  for (int q = 0; q < 2; ++q) load_w(0, q);
#pragma unroll
  for (int hq = 0; hq < 4; ++hq) load_x(0, 0, hq >> 1, hq & 1);
  __builtin_amdgcn_sched_barrier(0);
  int pos[2], seq[2], page[2];
  bool valid[2];                                          // token exists and is mapped so far
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int t = tile_t * kTileT + wn * 64 + j * 32 + l32;
    pos[j] = 0;
    seq[j] = 0;
    valid[j] = t < a.n_tok;
    if (valid[j]) {
      pos[j] = a.positions ? a.positions[t] : a.pos_base + t;
      if (a.cu_seqlens) {                                 // largest s with cu[s] <= t
        int lo = 0, hi = a.n_seq;                         // invariant: cu[lo] <= t < cu[hi]
        while (hi - lo > 1) {
          const int mid = (lo + hi) >> 1;
          if (a.cu_seqlens[mid] <= t) lo = mid; else hi = mid;
        }
        seq[j] = lo;
      }
    }
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int q = 0; q < 2; ++q) load_w(1, q);
#pragma unroll
  for (int hq = 0; hq < 4; ++hq) load_x(1, 1, hq >> 1, hq & 1);
#pragma unroll
  for (int q = 0; q < 2; ++q) load_w(2, q);
#pragma unroll
  for (int q = 0; q < 2; ++q) load_w(3, q);
#pragma unroll
  for (int q = 0; q < 2; ++q) load_x(2, 2, 0, q);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    page[j] = -1;
    if (valid[j]) {
      const int blk = pos[j] >> a.block_shift;
      if (pos[j] < 0 || pos[j] >= a.max_position || blk >= a.max_blocks) {
        atomicOr(a.err, HC_DEV_BAD_POSITION);
        valid[j] = false;
      } else {
        page[j] = a.block_tables[(size_t)seq[j] * a.max_blocks + blk];
      }
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_waitcnt vmcnt(12)" ::: "memory");      // the first 6 (W0, X0) have landed
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int n = 0; n < 6; ++n) read_frag(0, 0, 0, 0, n, af0, bf0);

  // ---- pipeline.  Weight stage kt % 4 holds step kt; activation super-stage (kt/2) % 3
  // holds steps kt, kt^1.  Per step there is one barrier, placed after the fragments of the
  // step's second half are in registers.  Past it the step's weight stage is free (refilled
  // with step kt + 4), after an odd step so is the activation super-stage (refilled in two
  // halves, in this step and the next, with super-tile kt/2 + 3), and step kt + 1 is
  // visible to every wave.  Every step issues exactly 4 loads per thread, in program order
  // [2 weight, 2 activation]; "vmcnt(8)" therefore means "everything issued up to three
  // steps ago has landed", which covers step kt + 1's operands.
  // The issue order is written out by hand and pinned with scheduling fences: every matrix
  // op is followed by at most one LDS read or one global->LDS load plus a few ALU ops.
  //
  // one step; PAR = kt & 1 and WM = wm are compile-time constants.
  //   xs      super-stage of step kt
  //   xs_next super-stage of step kt + 1 (= xs for even kt)
  //   xl      super-stage refilled in this step, with super-tile ml
  auto step = [&](int kt, auto par_c, auto wm_c, int xs, int xs_next, int xl, int ml) {
    constexpr int PAR = decltype(par_c)::value;
    constexpr int WM = decltype(wm_c)::value;
    // phase A: matrix ops on the first half (fragments already in registers) while the
    // second half's fragments stream in from LDS
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const int i = n >> 1, j = n & 1;
      if (n < 6) read_frag(kt, xs, PAR, 1, n, af1, bf1);
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af0[i], bf0[j], acc[i][j], 0, 0, 0);
      if (n < 4) ssum = sumsq2(bf0[WM], n, ssum);
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // phase B: matrix ops on the second half while the first fragments of step kt + 1 stream
    // in and the stages just consumed are refilled
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const int i = n >> 1, j = n & 1;
      if (n < 6) read_frag(kt + 1, xs_next, PAR ^ 1, 0, n, af0, bf0);
      if (n >= 4) {
        if (n < 6) load_w(kt + kWStages, n - 4);
        else       load_x(ml, xl, PAR ^ 1, n - 6);
      }
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af1[i], bf1[j], acc[i][j], 0, 0, 0);
      if (n < 4) ssum = sumsq2(bf1[WM], n, ssum);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto run = [&](auto wm_c) {
    int xr = 0;                                          // (kt / 2) % 3 for the even step kt
    for (int kt = 0; kt < nk; kt += 2) {
      const int xr1 = xr == 2 ? 0 : xr + 1, xr2 = xr == 0 ? 2 : xr - 1;   // +1, +2 mod 3
      // even step: completes super-tile kt/2 + 2 (second half) in super-stage xr + 2
      step(kt, std::integral_constant<int, 0>{}, wm_c, xr, xr, xr2, (kt >> 1) + 2);
      // odd step: super-stage xr is consumed; starts super-tile kt/2 + 3 (first half) in it
      step(kt + 1, std::integral_constant<int, 1>{}, wm_c, xr, xr1, xr, (kt >> 1) + 3);
      xr = xr1;
    }
  };
  if (wm == 0) run(std::integral_constant<int, 0>{});
  else         run(std::integral_constant<int, 1>{});
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");   // drain the look-ahead loads
  __syncthreads();

  // ---- epilogue: everything per token is per lane.  fp32 accumulators are scaled by the
  // token's 1/rms, K is rotated with the (cos, sin) table row of the token's position, and
  // one round-to-nearest-even conversion to bf16 precedes the 16-byte stores into the
  // token's cache row.  The table reads of token block j + 1 are issued before block j is
  // processed, so their latency overlaps the arithmetic and the stores.
  int tok_row[2];                                         // row of the token's K in the pool, or -1
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    tok_row[j] = -1;
    if (valid[j]) {
      if (page[j] < 0 || page[j] >= a.num_pages) atomicOr(a.err, HC_DEV_BAD_PAGE);
      else tok_row[j] = ((page[j] * 2) << a.block_shift) + (pos[j] & ((1 << a.block_shift) - 1));
    }
  }
  float rstd[2];
  {
    // exchange the sums of squares between the two waves of a token range through LDS
    float* sums = reinterpret_cast<float*>(lds);          // [wn][block][32]
    const float s = ssum + __shfl_xor(ssum, 32);          // the two lane halves hold different channels
    if (lh == 0) sums[(wn * 2 + wm) * 32 + l32] = s;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j) rstd[j] = rsqrtf(sums[(wn * 2 + j) * 32 + l32] * a.inv_d + a.eps);
  }
  // The wave's 128 weight rows are one K pair group (blocks 0, 1) and the V pair group of the
  // same index (blocks 2, 3).
  const int grp = (tile_f * kTileF + wm * 128) >> 7;
  if (grp * kPairGroup >= a.d_kv) return;                 // padding rows only (wave-uniform)
  const int hd = a.head_dim, half = hd >> 1, groups_per_head = hd >> 6;
  const int head = grp / groups_per_head;
  const int i0 = 32 * (grp - head * groups_per_head) + 16 * lh;   // first RoPE pair index of this lane
  // batches b = 2 j + q: token block j, q = 0 -> K (rotated), q = 1 -> V
  float4 cs[2][8];                                        // [token block][v / 2]: two (cos, sin) pairs each
  auto load_cs = [&](int j) {
    if (tok_row[j] < 0) return;
    const float2* rope_row = a.rope + (size_t)pos[j] * half + i0;
#pragma unroll
    for (int v = 0; v < 16; v += 2) cs[j][v >> 1] = *reinterpret_cast<const float4*>(rope_row + v);
  };
  load_cs(0);
  load_cs(1);
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const int j = b >> 1, q = b & 1;
    if (tok_row[j] < 0) continue;
    // V rows of a page follow its K rows: + block_size token rows
    uint16_t* dst = a.pool + ((size_t)tok_row[j] + ((size_t)q << a.block_shift)) * a.d_kv + head * hd;
    uint32_t pa[8], pb[8];                                // bf16 pairs of the first / second members
    if (q == 0) {
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const float4 c4 = cs[j][v >> 1];
        const float a0 = acc[0][j][v] * rstd[j], b0 = acc[1][j][v] * rstd[j];
        const float a1 = acc[0][j][v + 1] * rstd[j], b1 = acc[1][j][v + 1] * rstd[j];
        const float ra0 = a0 * c4.x - b0 * c4.y, rb0 = b0 * c4.x + a0 * c4.y;
        const float ra1 = a1 * c4.z - b1 * c4.w, rb1 = b1 * c4.z + a1 * c4.w;
        if (STYLE == 0) { pa[v >> 1] = pack_bf16x2(ra0, ra1); pb[v >> 1] = pack_bf16x2(rb0, rb1); }
        else            { pa[v >> 1] = pack_bf16x2(ra0, rb0); pb[v >> 1] = pack_bf16x2(ra1, rb1); }
      }
    } else {
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const float a0 = acc[2][j][v] * rstd[j], b0 = acc[3][j][v] * rstd[j];
        const float a1 = acc[2][j][v + 1] * rstd[j], b1 = acc[3][j][v + 1] * rstd[j];
        if (STYLE == 0) { pa[v >> 1] = pack_bf16x2(a0, a1); pb[v >> 1] = pack_bf16x2(b0, b1); }
        else            { pa[v >> 1] = pack_bf16x2(a0, b0); pb[v >> 1] = pack_bf16x2(a1, b1); }
      }
    }
    if (STYLE == 0) {
      // first members at head*hd + i, second members at head*hd + hd/2 + i
      u32x4* da = reinterpret_cast<u32x4*>(dst + i0);
      u32x4* db = reinterpret_cast<u32x4*>(dst + half + i0);
      da[0] = u32x4{pa[0], pa[1], pa[2], pa[3]};
      da[1] = u32x4{pa[4], pa[5], pa[6], pa[7]};
      db[0] = u32x4{pb[0], pb[1], pb[2], pb[3]};
      db[1] = u32x4{pb[4], pb[5], pb[6], pb[7]};
    } else {
      // members of pair i at head*hd + 2i and 2i + 1: pa/pb hold (first, second) of even/odd v
      u32x4* dq = reinterpret_cast<u32x4*>(dst + 2 * i0);
      dq[0] = u32x4{pa[0], pb[0], pa[1], pb[1]};
      dq[1] = u32x4{pa[2], pb[2], pa[3], pb[3]};
      dq[2] = u32x4{pa[4], pb[4], pa[5], pb[5]};
      dq[3] = u32x4{pa[6], pb[6], pa[7], pb[7]};
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
  // Super-tile shape: fewest rounds on the busiest XCD (an XCD runs 32 workgroups at a
  // time, one per CU), then the most row sharing (smallest 1/GF + 1/GT), then fewest slots.
  int best_rounds = 1 << 30, best_slots = 1 << 30, best_share = 1 << 30;
  g.gf_shift = g.g_shift = 0;
  for (int fs = 0; fs <= 5; ++fs) {
    for (int ts = 0; fs + ts <= 5; ++ts) {
      const int gf = 1 << fs, gt = 1 << ts;
      const int n_super = ((g.nf + gf - 1) / gf) * ((g.nt + gt - 1) / gt);
      const int slots = (n_super + 7) / 8 * gf * gt;      // workgroup slots per XCD
      const int rounds = (slots + 31) / 32;
      const int share = (32 >> fs) + (32 >> ts);          // 32 * (1/GF + 1/GT)
      if (rounds < best_rounds || (rounds == best_rounds && share < best_share) ||
          (rounds == best_rounds && share == best_share && slots < best_slots)) {
        best_rounds = rounds; best_share = share; best_slots = slots;
        g.gf_shift = fs; g.g_shift = fs + ts;
      }
    }
  }
  g.nsf = (g.nf + (1 << g.gf_shift) - 1) >> g.gf_shift;
  const unsigned grid = (unsigned)best_slots * 8u;
  if (a.rope_style == 0)
    hipLaunchKernelGGL(restore_kernel<0>, dim3(grid), dim3(kThreads), kLdsBytes, stream, a, g);
  else
    hipLaunchKernelGGL(restore_kernel<1>, dim3(grid), dim3(kThreads), kLdsBytes, stream, a, g);
  return hipGetLastError();
}

}  // namespace hc
