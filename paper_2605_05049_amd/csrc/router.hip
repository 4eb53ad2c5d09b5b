// The gating function's linear map, logits = x W_r^T (Section II-A), as a skinny MFMA kernel of its own.
//
// The problem is T x E x d with E small (8 .. a few hundred): its FLOPs are negligible and its time is the time to
// read x once, so the kernel is built for HBM streaming, not for the matrix cores' peak.  A wavefront owns TB blocks
// of 16 tokens and all (up to 128) experts of its expert tile and walks one eighth of K = d_model: every x fragment
// goes from global memory straight into the MFMA operand registers (16 bytes per lane, 64 contiguous bytes per token
// row and instruction, two k-groups kept in flight), every W_r fragment comes from the L2 (W_r is at most a few MB
// and is re-read 8/TB times the bytes of x at E = 128), no LDS, no barrier in the loop.  The 8 wavefronts of a block
// are the 8 parts of K of the SAME tokens; their partial sums meet in LDS at the end and are added in part order, so
// the result never depends on timing and the whole call is a single launch.  TB is chosen from T so that the grid
// has at least one block per CU.  (Many experts and many tokens take the second forward kernel below, which stages both
// operands through LDS; the backward's kernels follow it.)
//
// MFMA 16x16x32 bf16: A = 16 experts x 32 k (lane l: expert l%16, k = 8 (l/16) .. +7), B = 16 tokens x 32 k (same
// pattern), D[expert][token]: lane l holds token l%16 and experts 4 (l/16) .. +3, i.e. 4 consecutive logits of a row.
#include "common.h"

#include <type_traits>

namespace moe {

typedef __bf16 r_bf16x8 __attribute__((ext_vector_type(8)));
typedef float r_f32x4 __attribute__((ext_vector_type(4)));

constexpr int kRouterWaves = 8;          // parts of K per block
constexpr int kRouterExpertTile = 128;   // experts per block (grid.y walks the tiles)

template <int TB, int NEB>
__global__ __launch_bounds__(kRouterWaves * kWave) void router_fwd_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_router,
                                                                         float* __restrict__ logits, int T, int E, int d) {
  constexpr int NBLK = (NEB * TB < 16) ? NEB * TB : 16;   // 16 x 16 blocks of partial logits that meet in LDS at a time
  __shared__ float part_sum[kRouterWaves][NBLK][16 * 16];   // (up to 128 KB)
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int n = lane & 15, kg = lane >> 4;            // token (or expert) inside a block of 16, group of 8 k
  const int t0 = blockIdx.x * (TB * 16);
  const int e0 = blockIdx.y * kRouterExpertTile;
  // this wavefront's part of K, in groups of 32
  const int n_groups = d / 32;
  const int per = (n_groups + kRouterWaves - 1) / kRouterWaves;
  const int g_begin = min(wave * per, n_groups), g_end = min(n_groups, g_begin + per);

  // rows past the end are clamped onto the last valid one (never stored); a row is addressed by the block's base
  // (wave-uniform) plus a 32-bit element offset per lane
  const uint16_t* xbase = x + (size_t)t0 * d;
  const uint16_t* wbase = w_router + (size_t)e0 * d;
  unsigned xoff[TB], woff[NEB];
#pragma unroll
  for (int b = 0; b < TB; b++) xoff[b] = (unsigned)min(16 * b + n, T - 1 - t0) * (unsigned)d + 8 * kg;
#pragma unroll
  for (int m = 0; m < NEB; m++) woff[m] = (unsigned)min(16 * m + n, E - 1 - e0) * (unsigned)d + 8 * kg;

  r_f32x4 acc[NEB][TB];
#pragma unroll
  for (int m = 0; m < NEB; m++)
#pragma unroll
    for (int b = 0; b < TB; b++) acc[m][b] = r_f32x4{0.f, 0.f, 0.f, 0.f};

  // DEPTH k-groups in flight (as many as the registers of this TB x NEB allow): while one is multiplied the loads of
  // the next DEPTH - 1 are already out.  x from HBM (touched once: non-temporal), W_r from the L2.
  constexpr int DEPTH = (TB + NEB) <= 2 ? 8 : ((TB + NEB) <= 6 ? 4 : 2);
  r_bf16x8 xf[DEPTH][TB], wf[DEPTH][NEB];
  auto load = [&](auto slot_c, int g) __attribute__((always_inline)) {
    constexpr int SL = decltype(slot_c)::value;
#pragma unroll
    for (int b = 0; b < TB; b++) xf[SL][b] = __builtin_nontemporal_load(reinterpret_cast<const r_bf16x8*>(xbase + xoff[b] + (size_t)g * 32));
#pragma unroll
    for (int m = 0; m < NEB; m++) wf[SL][m] = *reinterpret_cast<const r_bf16x8*>(wbase + woff[m] + (size_t)g * 32);
  };
  auto multiply = [&](auto slot_c) __attribute__((always_inline)) {
    constexpr int SL = decltype(slot_c)::value;
#pragma unroll
    for (int m = 0; m < NEB; m++)
#pragma unroll
      for (int b = 0; b < TB; b++) acc[m][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[SL][m], xf[SL][b], acc[m][b], 0, 0, 0);
  };
  auto for_each_slot = [&](auto&& f) __attribute__((always_inline)) {
    f(std::integral_constant<int, 0>{});
    if constexpr (DEPTH > 1) f(std::integral_constant<int, 1>{});
    if constexpr (DEPTH > 2) { f(std::integral_constant<int, 2>{}); f(std::integral_constant<int, 3>{}); }
    if constexpr (DEPTH > 4) { f(std::integral_constant<int, 4>{}); f(std::integral_constant<int, 5>{}); f(std::integral_constant<int, 6>{}); f(std::integral_constant<int, 7>{}); }
  };
  // prologue: slots 0 .. DEPTH-2 take k-groups g_begin .. g_begin + DEPTH - 2
  for_each_slot([&](auto sc) __attribute__((always_inline)) {
    constexpr int SL = decltype(sc)::value;
    if (SL < DEPTH - 1 && g_begin + SL < g_end) load(sc, g_begin + SL);
  });
  for (int g = g_begin; g < g_end; g += DEPTH) {
    for_each_slot([&](auto sc) __attribute__((always_inline)) {
      constexpr int SL = decltype(sc)::value;
      if (g + SL < g_end) {
        if (g + SL + DEPTH - 1 < g_end) load(std::integral_constant<int, (SL + DEPTH - 1) % DEPTH>{}, g + SL + DEPTH - 1);
        multiply(sc);
      }
    });
  }

  // the 8 parts of K meet in LDS, NBLK blocks of 16 x 16 at a time (block q = m TB + b), and are added in part order;
  // item i of a pass is logit (token (i % 256) / 16, expert i % 16) of block i / 256: 16 consecutive experts of a row
  // per 16 threads
  constexpr int NPASS = (NEB * TB + NBLK - 1) / NBLK;
#pragma unroll
  for (int pass = 0; pass < NPASS; pass++) {
    if (pass > 0) __syncthreads();   // the previous pass has been read
#pragma unroll
    for (int j = 0; j < NBLK; j++) {
      const int q = pass * NBLK + j;
      if (q < NEB * TB) *reinterpret_cast<r_f32x4*>(&part_sum[wave][j][n * 16 + 4 * kg]) = acc[q / TB][q % TB];   // [token][expert]
    }
    __syncthreads();
    for (int i = threadIdx.x; i < NBLK * 256; i += kRouterWaves * kWave) {
      const int j = i >> 8, idx = i & 255, q = pass * NBLK + j;
      if (q >= NEB * TB) break;
      float sum = 0.f;
#pragma unroll
      for (int p = 0; p < kRouterWaves; p++) sum += part_sum[p][j][idx];
      const int t = t0 + 16 * (q % TB) + (idx >> 4), e = e0 + 16 * (q / TB) + (idx & 15);
      if (t < T && e < E) logits[(size_t)t * E + e] = sum;
    }
  }
}

// The same map for many experts and many tokens (E > 32, T >= 8192).  There every block of the kernel above also
// streams its expert tile's whole W_r (1 MB at E = 128) for 64 tokens, twice the bytes of its x rows, and the MFMA
// operand layout makes every load fetch 64 bytes of 16 different lines.  Here both operands go through LDS instead:
// a block of 8 wavefronts owns 64 tokens x 32 NEBH experts and walks all of K in steps of 64 (whole 128-byte lines,
// direct global->LDS loads, one instruction = 8 rows, chunks XOR-swizzled with the row so that the fragment reads are
// conflict-free), through a ring of four stages of (64 + 32 NEBH) x 128 bytes, three steps ahead; wavefront w
// multiplies token block w % 4 with expert half w / 4.  Every wavefront issues three loads per stage (one of x, two of
// W_r), so "all but the two youngest stages" is vmcnt(6).  No K split: each logit is one wavefront's sum.
template <int NEBH>
__global__ __launch_bounds__(kRouterWaves * kWave) void router_fwd_wide_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_router,
                                                                               float* __restrict__ logits, int T, int E, int d) {
  constexpr int XROWS = 64, WROWS = 32 * NEBH;
  constexpr int STAGE = (XROWS + WROWS) * 128;   // bytes
  __shared__ __attribute__((aligned(1024))) char ring[4][STAGE];
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 15, kg = lane >> 4;
  const int t0 = blockIdx.x * XROWS, e0 = blockIdx.y * WROWS;
  const int tb = wave & 3, eh = wave >> 2;
  const int n_steps = d / 64;

  // direct loads: instruction i of an operand = rows 8 i .. 8 i + 7, lane L = row 8 i + L / 8, the 16-byte chunk
  // (L % 8) ^ ((row >> 1) & 7) of the row's 128 bytes of this step; rows past the end are clamped (never stored)
  auto src_off = [&](int row_in_tile, int limit_rows) -> unsigned {
    const int r = min(row_in_tile, limit_rows - 1);
    const int c = (lane & 7) ^ ((row_in_tile >> 1) & 7);
    return (unsigned)(((size_t)r * d + c * 8) * 2);
  };
  const uint16_t* xbase = x + (size_t)t0 * d;
  const uint16_t* wbase = w_router + (size_t)e0 * d;
  const unsigned xo = src_off(8 * wave + (lane >> 3), T - t0);
  unsigned wo[NEBH / 2 > 0 ? NEBH / 2 : 1];   // W_r instructions of this wavefront: WROWS / 8 / 8 = NEBH / 2
#pragma unroll
  for (int i = 0; i < NEBH / 2; i++) wo[i] = src_off(8 * (wave * (NEBH / 2) + i) + (lane >> 3), E - e0);
  constexpr int LOADS = 1 + NEBH / 2;   // per wavefront and stage
  static_assert(LOADS == 3 || LOADS == 2, "the wait counts below are written for NEBH = 4 or 2");
  auto issue = [&](int step, char* stage) __attribute__((always_inline)) {
    direct_load16(xbase + (size_t)step * 64, xo, stage + wave * 1024);
#pragma unroll
    for (int i = 0; i < NEBH / 2; i++) direct_load16(wbase + (size_t)step * 64, wo[i], stage + XROWS * 128 + (wave * (NEBH / 2) + i) * 1024);
  };
  // fragment of 16 rows x 32 k: lane (n, kg) reads chunk 4 g + kg of row r0 + n
  auto frag = [&](const char* rows, int r0, int g) __attribute__((always_inline)) -> r_bf16x8 {
    const int r = r0 + n;
    return *reinterpret_cast<const r_bf16x8*>(rows + r * 128 + (((4 * g + kg) ^ ((r >> 1) & 7)) << 4));
  };

  r_f32x4 acc[NEBH];
#pragma unroll
  for (int m = 0; m < NEBH; m++) acc[m] = r_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s0 = 0; s0 < 3; s0++)
    if (s0 < n_steps) issue(s0, ring[s0]);
  for (int step = 0; step < n_steps; step++) {
    // loads of steps step + 1 and step + 2 may still be in flight
    const int younger = min(2, n_steps - 1 - step);
    if (younger == 2) {
      if (LOADS == 3) __builtin_amdgcn_s_waitcnt(0x0F76); else __builtin_amdgcn_s_waitcnt(0x0F74);   // vmcnt(6) / vmcnt(4)
    } else if (younger == 1) {
      if (LOADS == 3) __builtin_amdgcn_s_waitcnt(0x0F73); else __builtin_amdgcn_s_waitcnt(0x0F72);   // vmcnt(3) / vmcnt(2)
    } else {
      __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    __syncthreads();   // this step's stage has landed for everyone; everyone is done with the stage of step - 1
    if (step + 3 < n_steps) issue(step + 3, ring[(step + 3) & 3]);
    const char* xs = ring[step & 3];
    const char* ws = xs + XROWS * 128;
#pragma unroll
    for (int g = 0; g < 2; g++) {
      const r_bf16x8 xf = frag(xs, 16 * tb, g);
#pragma unroll
      for (int m = 0; m < NEBH; m++) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag(ws, 16 * (eh * NEBH + m), g), xf, acc[m], 0, 0, 0);
    }
  }
  // acc[m][i] = logit (token t0 + 16 tb + n, expert e0 + 16 (eh NEBH + m) + 4 kg + i)
  const int t = t0 + 16 * tb + n;
  if (t < T) {
#pragma unroll
    for (int m = 0; m < NEBH; m++) {
      const int e = e0 + 16 * (eh * NEBH + m) + 4 * kg;
      float* dst = logits + (size_t)t * E + e;
      if ((E & 3) == 0 && e + 4 <= E) {
        *reinterpret_cast<r_f32x4*>(dst) = acc[m];
      } else {
#pragma unroll
        for (int i = 0; i < 4; i++)
          if (e + i < E) dst[i] = acc[m][i];
      }
    }
  }
}

template <int TB>
static void launch_router_fwd(hipStream_t st, dim3 grid, int neb, const uint16_t* x, const uint16_t* w_router, float* logits, int T, int E, int d) {
  const dim3 block(kRouterWaves * kWave);
  if (neb <= 1) MOE_LAUNCH("router_fwd", st, (router_fwd_kernel<TB, 1>), grid, block, 0, st, x, w_router, logits, T, E, d);
  else if (neb <= 2) MOE_LAUNCH("router_fwd", st, (router_fwd_kernel<TB, 2>), grid, block, 0, st, x, w_router, logits, T, E, d);
  else if (neb <= 4) MOE_LAUNCH("router_fwd", st, (router_fwd_kernel<TB, 4>), grid, block, 0, st, x, w_router, logits, T, E, d);
  else MOE_LAUNCH("router_fwd", st, (router_fwd_kernel<TB, 8>), grid, block, 0, st, x, w_router, logits, T, E, d);
}


// ---------------------------------------------------------------------------------------------------------
// Backward of the linear map: helpers for dx_router = dlogits W_r and dW_r = dlogits^T x.
// ---------------------------------------------------------------------------------------------------------

// Splits dlogits into a bf16 head and a bf16 remainder (hi = bf16(v), lo = bf16(v - hi): hi + lo carries 16
// significand bits of v), zero-padded to Epad columns; writes W_r^T [d, Ek] bf16 (Ek = E rounded up to 32, zero
// padded), so that the expert index is the contiguous one for the dx kernel's fragments; writes the offset arrays of
// the GEMM-path problems: {0, T} at [0..1], {0, E} at [4..5], and at [8 .. 8 + S] the S + 1 bounds of the S equal
// parts of the token range that the dW_r contraction is cut into; and what the weight-gradient kernel reads of a
// schedule: the order of its segments (the parts in turn: they are equally long but for the last), the zero page and
// its zeroed tile queue.
__global__ __launch_bounds__(256) void router_prepare_kernel(const float* __restrict__ dlogits, const uint16_t* __restrict__ w_router,
                                                             uint16_t* __restrict__ hi, uint16_t* __restrict__ lo,
                                                             uint16_t* __restrict__ w_t, int32_t* __restrict__ offsets2,
                                                             int32_t* __restrict__ part_order, int32_t* __restrict__ tile_queue,
                                                             uint32_t* __restrict__ zero_page, int T, int E, int Epad, int Ek, int d, int S,
                                                             int part_rows) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i == 0) {
    offsets2[0] = 0; offsets2[1] = T;
    offsets2[4] = 0; offsets2[5] = E;
  }
  if (i <= S) offsets2[8 + i] = (int)min((long long)T, i * part_rows);
  if (i < S) part_order[i] = (int)i;
  if (i < 64) zero_page[i] = 0u;
  if (i < 8) tile_queue[i] = 0;
  if (w_t != nullptr && i < (long long)d * (Ek / 8)) {
    const int dcol = (int)(i % d), ec = (int)(i / d);
    uint32_t v[4];
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int e0 = 8 * ec + 2 * j;
      const uint32_t a = e0 < E ? w_router[(size_t)e0 * d + dcol] : 0u;
      const uint32_t b = e0 + 1 < E ? w_router[(size_t)(e0 + 1) * d + dcol] : 0u;
      v[j] = a | (b << 16);
    }
    *reinterpret_cast<uint4*>(w_t + (size_t)dcol * Ek + 8 * ec) = make_uint4(v[0], v[1], v[2], v[3]);
  }
  // 8 consecutive experts of a token per thread (Epad is a multiple of 64): 16 bytes of each of the two copies
  if (i >= (long long)T * (Epad / 8)) return;
  const int t = (int)(i / (Epad / 8)), e0 = (int)(i % (Epad / 8)) * 8;
  float v[8];
  const float* src = dlogits + (size_t)t * E + e0;
  if ((E & 3) == 0 && e0 + 8 <= E) {
    const r_f32x4 a = *reinterpret_cast<const r_f32x4*>(src), b = *reinterpret_cast<const r_f32x4*>(src + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  } else {
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = (e0 + j < E) ? src[j] : 0.f;
  }
  uint32_t h[4], l[4];
#pragma unroll
  for (int j = 0; j < 4; j++) {
    h[j] = pack_bf16(v[2 * j], v[2 * j + 1]);
    l[j] = pack_bf16(v[2 * j] - bf16lo(h[j]), v[2 * j + 1] - bf16hi(h[j]));
  }
  *reinterpret_cast<uint4*>(hi + (size_t)t * Epad + e0) = make_uint4(h[0], h[1], h[2], h[3]);
  *reinterpret_cast<uint4*>(lo + (size_t)t * Epad + e0) = make_uint4(l[0], l[1], l[2], l[3]);
}

// dx_router[t, c] = sum_e dlogits[t, e] W_r[e, c] for E <= 128: T x d x E with E small, so its time is the time to
// write dx once.  A block of 16 wavefronts owns `tokens_per_block` tokens and 1024 columns (2 KB of a token's row:
// narrower blocks measured slower); a wavefront keeps the W_r^T fragments of its 64 columns (4 blocks of 16 columns x
// KG groups of 32 experts) in registers for the whole block.  Per 64 tokens the block stages the head and the
// remainder of dlogits in LDS once (16-byte loads, the next 64 tokens' pieces in flight in registers, chunk positions
// XOR-swizzled with the token so that the fragment reads are conflict-free); between two such barriers every
// wavefront works through four tiles of 16 tokens at its own pace: multiply (MFMA 16x16x32, columns as rows of the
// result so that a lane ends up with 4 consecutive columns of a token), bounce the 16 x 64 bf16 results through its
// own LDS patch, store 128 contiguous bytes per token, so that one wavefront's stores overlap another's multiplies.
constexpr int kDxWaves = 16;
constexpr int kDxColsPerWave = 64;
constexpr int kDxTokensPerStage = 64;
constexpr int kDxBouncePitch = kDxColsPerWave * 2 + 16;   // bytes per staged token row (the +16 spreads the banks)

template <int KG>
__global__ __launch_bounds__(kDxWaves * kWave) void router_bwd_dx_kernel(const uint16_t* __restrict__ dl_hi, const uint16_t* __restrict__ dl_lo,
                                                                         const uint16_t* __restrict__ w_t, uint16_t* __restrict__ dx,
                                                                         int T, int d, int Epad, int tokens_per_block) {
  constexpr int Ek = 32 * KG;                  // experts padded to whole k-groups
  constexpr int CH = 4 * KG;                   // 16-byte chunks per staged row
  constexpr int ROWB = Ek * 2;                 // bytes per staged row
  constexpr int TS = kDxTokensPerStage;
  constexpr int NTHR = kDxWaves * kWave;
  constexpr int ITEMS = 2 * TS * CH;           // 16-byte pieces of a stage (head and remainder)
  constexpr int PER = (ITEMS + NTHR - 1) / NTHR;   // ... per thread
  __shared__ __attribute__((aligned(16))) char dl_tile[2][2 * TS * ROWB];       // [buffer][hi | lo][token][expert]
  __shared__ __attribute__((aligned(16))) char bounce[kDxWaves][16 * kDxBouncePitch];
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int n = lane & 15, kg = lane >> 4;
  const int t_begin = blockIdx.x * tokens_per_block;
  const int t_end = min(T, t_begin + tokens_per_block);
  const int c0 = blockIdx.y * (kDxWaves * kDxColsPerWave) + wave * kDxColsPerWave;   // first column of this wavefront
  constexpr int MB = kDxColsPerWave / 16;                                              // blocks of 16 columns per wavefront
  const int n_cb = max(0, min(MB, (d - c0) / 16));                                     // ... that exist

  // W_r^T fragments: rows = columns of dx (clamped onto the last valid one where the wavefront has fewer)
  r_bf16x8 wf[MB][KG];
#pragma unroll
  for (int m = 0; m < MB; m++) {
    const int c = min(c0 + 16 * m + n, d - 1);
#pragma unroll
    for (int g = 0; g < KG; g++) wf[m][g] = *reinterpret_cast<const r_bf16x8*>(w_t + (size_t)c * Ek + 32 * g + 8 * kg);
  }

  // staging: piece i of a stage = tensor i / (TS CH), token row (i / CH) % TS, chunk i % CH; thread t takes pieces
  // t, t + NTHR, ...
  uint4 staged[PER];
  auto fetch = [&](int t0) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < PER; k++) {
      const int i = threadIdx.x + k * NTHR;
      const int part = i / (TS * CH), row = (i / CH) % TS, ch = i % CH;
      const int t = min(t0 + row, T - 1);   // rows past the end are clamped (never stored)
      staged[k] = (i < ITEMS) ? *reinterpret_cast<const uint4*>((part == 0 ? dl_hi : dl_lo) + (size_t)t * Epad + 8 * ch) : make_uint4(0u, 0u, 0u, 0u);
    }
  };
  auto publish = [&](int b) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < PER; k++) {
      const int i = threadIdx.x + k * NTHR;
      const int part = i / (TS * CH), row = (i / CH) % TS, ch = i % CH;
      if (i < ITEMS) *reinterpret_cast<uint4*>(&dl_tile[b][(part * TS + row) * ROWB + ((ch ^ (((row & 15) * KG) >> 2)) & (CH - 1)) * 16]) = staged[k];
    }
  };
  r_f32x4 acc[MB];
  auto multiply = [&](int b, int j) __attribute__((always_inline)) {   // tile j of stage b
#pragma unroll
    for (int m = 0; m < MB; m++) acc[m] = r_f32x4{0.f, 0.f, 0.f, 0.f};
    // 2 KG fragment reads (remainder first, then the head), each one group ahead of the MFMAs that use it
    auto frag = [&](int sidx) __attribute__((always_inline)) -> r_bf16x8 {
      const int part = 1 - sidx / KG, g = sidx % KG;
      const int ch = ((4 * g + kg) ^ ((n * KG) >> 2)) & (CH - 1);
      return *reinterpret_cast<const r_bf16x8*>(&dl_tile[b][(part * TS + 16 * j + n) * ROWB + ch * 16]);
    };
    r_bf16x8 df = frag(0);
#pragma unroll
    for (int sidx = 0; sidx < 2 * KG; sidx++) {
      const r_bf16x8 nxt = frag(min(sidx + 1, 2 * KG - 1));
      __builtin_amdgcn_sched_barrier(0);   // (keeps the read above the MFMAs it is meant to overlap)
#pragma unroll
      for (int m = 0; m < MB; m++) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[m][sidx % KG], df, acc[m], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      df = nxt;
    }
  };
  // acc[m][i] = dx[t0 + n][c0 + 16 m + 4 kg + i]: to LDS as bf16, back as 16 bytes per lane along a token's row
  auto store_tile = [&](int t0) __attribute__((always_inline)) {
    char* mine = bounce[wave];
#pragma unroll
    for (int m = 0; m < MB; m++)
      *reinterpret_cast<uint2*>(mine + n * kDxBouncePitch + (16 * m + 4 * kg) * 2) =
          make_uint2(pack_bf16(acc[m][0], acc[m][1]), pack_bf16(acc[m][2], acc[m][3]));
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wavefront's LDS writes are done
    __builtin_amdgcn_wave_barrier();
    constexpr int CPR = kDxColsPerWave / 8;   // 16-byte chunks per token row
    constexpr int RPI = kWave / CPR;          // token rows per store instruction
#pragma unroll
    for (int it = 0; it < 16 / RPI; it++) {
      const int r = RPI * it + lane / CPR, cc = lane % CPR;   // token row of the tile, chunk of 8 columns
      if (t0 + r < t_end && cc < 2 * n_cb)
        *reinterpret_cast<uint4*>(dx + (size_t)(t0 + r) * d + c0 + 8 * cc) = *reinterpret_cast<const uint4*>(mine + r * kDxBouncePitch + 16 * cc);
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);   // the read-back is complete before the next tile overwrites the patch
    __builtin_amdgcn_wave_barrier();
  };
  fetch(t_begin);
  int buf = 0;
  for (int ts = t_begin; ts < t_end; ts += TS, buf ^= 1) {
    publish(buf);
    __syncthreads();   // (a stage is overwritten two barriers after it was published: everyone has finished with it)
    if (ts + TS < t_end) fetch(ts + TS);
#pragma unroll
    for (int j = 0; j < TS / 16; j++) {
      if (ts + 16 * j < t_end) {
        multiply(buf, j);
        store_tile(ts + 16 * j);
      }
    }
  }
}

// dW_r[e, c] (+)= sum over the S parts of partial[s][c][e]: the parts are the weight-gradient kernel's outputs for the
// S pieces of the token range (columns of dx as rows, experts as columns, row pitch ldp, a multiple of 4); added in
// part order.  A block sums 32 columns x up to 128 experts with 16-byte loads along the experts (all parts of an
// element requested before the first add) and transposes through LDS, so that dW_r is written 128 bytes at a time.
constexpr int kDwReduceCols = 32, kDwReduceExperts = 128;
__global__ __launch_bounds__(256) void router_dw_reduce_kernel(const float* __restrict__ partial, float* __restrict__ dw, int S, int E, int d,
                                                               int ldp, int accumulate) {
  __shared__ float tile[kDwReduceCols][kDwReduceExperts + 1];
  const int c0 = blockIdx.x * kDwReduceCols, e0 = blockIdx.y * kDwReduceExperts;
  const int ew = min(kDwReduceExperts, ldp - e0);   // experts (padded to 4) of this tile
  const int quads = ew / 4;
  const size_t part_stride = (size_t)d * ldp;
  for (int i = threadIdx.x; i < kDwReduceCols * quads; i += 256) {
    const int c = i / quads, q = i % quads;   // consecutive threads: consecutive 16 bytes of a column's row
    r_f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (c0 + c < d) {
      const float* src = partial + (size_t)(c0 + c) * ldp + e0 + 4 * q;
      for (int p = 0; p < S; p += 8) {
        r_f32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = (p + j < S) ? *reinterpret_cast<const r_f32x4*>(src + (size_t)(p + j) * part_stride) : r_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 8; j++) s += v[j];
      }
    }
    tile[c][4 * q] = s.x; tile[c][4 * q + 1] = s.y; tile[c][4 * q + 2] = s.z; tile[c][4 * q + 3] = s.w;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kDwReduceCols * ew; i += 256) {
    const int e = i / kDwReduceCols, c = i % kDwReduceCols;   // consecutive threads: consecutive columns of an expert's row
    if (c0 + c < d && e0 + e < E) {
      float* dst = dw + (size_t)(e0 + e) * d + c0 + c;
      *dst = accumulate ? *dst + tile[c][e] : tile[c][e];
    }
  }
}

void launch_router_prepare(hipStream_t st, const float* dlogits, const uint16_t* w_router, uint16_t* hi, uint16_t* lo, uint16_t* w_t,
                           int32_t* offsets2, int32_t* part_order, int32_t* tile_queue, uint32_t* zero_page, int T, int E, int Epad, int Ek,
                           int d, int S, int part_rows) {
  const long long n = max((long long)T * (Epad / 8), max((long long)d * (Ek / 8), 64LL));
  MOE_LAUNCH("router_prepare", st, router_prepare_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dlogits, w_router, hi, lo, w_t,
             offsets2, part_order, tile_queue, zero_page, T, E, Epad, Ek, d, S, part_rows);
}

void launch_router_bwd_dx(hipStream_t st, const uint16_t* dl_hi, const uint16_t* dl_lo, const uint16_t* w_t, uint16_t* dx, int T, int d,
                          int E, int Epad) {
  // tokens per block: a multiple of a stage's 64, as large as still gives every CU a block
  const unsigned col_groups = (unsigned)((d + kDxWaves * kDxColsPerWave - 1) / (kDxWaves * kDxColsPerWave));
  int tpb = 1024;
  while (tpb > kDxTokensPerStage && (long long)((T + tpb - 1) / tpb) * col_groups < 256) tpb >>= 1;
  const dim3 grid((unsigned)((T + tpb - 1) / tpb), col_groups), block(kDxWaves * kWave);
  const int kgroups = (E + 31) / 32;
  if (kgroups <= 1) MOE_LAUNCH("router_bwd_dx", st, (router_bwd_dx_kernel<1>), grid, block, 0, st, dl_hi, dl_lo, w_t, dx, T, d, Epad, tpb);
  else if (kgroups <= 2) MOE_LAUNCH("router_bwd_dx", st, (router_bwd_dx_kernel<2>), grid, block, 0, st, dl_hi, dl_lo, w_t, dx, T, d, Epad, tpb);
  else MOE_LAUNCH("router_bwd_dx", st, (router_bwd_dx_kernel<4>), grid, block, 0, st, dl_hi, dl_lo, w_t, dx, T, d, Epad, tpb);
}

void launch_router_dw_reduce(hipStream_t st, const float* partial, float* dw, int S, int E, int d, int ldp, int accumulate) {
  const dim3 grid((unsigned)((d + kDwReduceCols - 1) / kDwReduceCols), (unsigned)((ldp + kDwReduceExperts - 1) / kDwReduceExperts));
  MOE_LAUNCH("router_dw_reduce", st, router_dw_reduce_kernel, grid, dim3(256), 0, st, partial, dw, S, E, d, ldp, accumulate);
}

}  // namespace moe

extern "C" int moe_router_fwd(const moe_shape* shape, const uint16_t* x, const uint16_t* w_router, float* logits,
                              void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  Dims D;
  int rc = check_shape(shape, &D);
  if (rc != MOE_OK) return rc;
  if (!ws) return MOE_ERR_NULL;
  if (!aligned(ws, 256)) return MOE_ERR_ALIGN;
  if (ws_bytes < ws_layout(D).total) return MOE_ERR_WORKSPACE;   // (kept in the signature; this kernel needs no scratch)
  MOE_REQUIRE_PTR(x); MOE_REQUIRE_PTR(w_router); MOE_REQUIRE_PTR(logits);
  MOE_REQUIRE_ALIGNED(x); MOE_REQUIRE_ALIGNED(w_router); MOE_REQUIRE_ALIGNED(logits);
  if (D.T == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)stream;
  if (D.E > 32 && D.T >= 8192) {   // many experts, many tokens: both operands through LDS
    const dim3 block(kRouterWaves * kWave);
    if (D.E <= 64) {
      MOE_LAUNCH("router_fwd", st, (router_fwd_wide_kernel<2>), dim3((unsigned)((D.T + 63) / 64), (unsigned)((D.E + 63) / 64)), block, 0, st, x, w_router,
                 logits, (int)D.T, (int)D.E, (int)D.d);
    } else {
      MOE_LAUNCH("router_fwd", st, (router_fwd_wide_kernel<4>), dim3((unsigned)((D.T + 63) / 64), (unsigned)((D.E + 127) / 128)), block, 0, st, x,
                 w_router, logits, (int)D.T, (int)D.E, (int)D.d);
    }
    return launch_status();
  }
  const unsigned e_tiles = (unsigned)((D.E + kRouterExpertTile - 1) / kRouterExpertTile);
  // tokens per block: 64 when that still gives every CU a block, else 32 or 16
  const int tb = (D.T >= 64 * 256) ? 4 : (D.T >= 32 * 256 ? 2 : 1);
  const dim3 grid((unsigned)((D.T + tb * 16 - 1) / (tb * 16)), e_tiles);
  const int neb = (min(D.E, kRouterExpertTile) + 15) / 16;   // expert blocks per tile (the last tile may hold fewer)
  if (tb == 4) launch_router_fwd<4>(st, grid, neb, x, w_router, logits, D.T, D.E, D.d);
  else if (tb == 2) launch_router_fwd<2>(st, grid, neb, x, w_router, logits, D.T, D.E, D.d);
  else launch_router_fwd<1>(st, grid, neb, x, w_router, logits, D.T, D.E, D.d);
  return launch_status();
}
