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
// has at least one block per CU.
//
// MFMA 16x16x32 bf16: A = 16 experts x 32 k (lane l: expert l%16, k = 8 (l/16) .. +7), B = 16 tokens x 32 k (same
// pattern), D[expert][token]: lane l holds token l%16 and experts 4 (l/16) .. +3, i.e. 4 consecutive logits of a row.
#include "common.h"

namespace moe {

typedef __bf16 r_bf16x8 __attribute__((ext_vector_type(8)));
typedef float r_f32x4 __attribute__((ext_vector_type(4)));

constexpr int kRouterWaves = 8;          // parts of K per block
constexpr int kRouterExpertTile = 128;   // experts per block (grid.y walks the tiles)

template <int TB, int NEB>
__global__ __launch_bounds__(kRouterWaves * kWave) void router_fwd_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_router,
                                                                         float* __restrict__ logits, int T, int E, int d) {
  __shared__ float part_sum[kRouterWaves][16 * 16];   // one 16 x 16 block of partial logits per wavefront
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int n = lane & 15, kg = lane >> 4;            // token (or expert) inside a block of 16, group of 8 k
  const int t0 = blockIdx.x * (TB * 16);
  const int e0 = blockIdx.y * kRouterExpertTile;
  // this wavefront's part of K, in groups of 32
  const int n_groups = d / 32;
  const int per = (n_groups + kRouterWaves - 1) / kRouterWaves;
  const int g_begin = min(wave * per, n_groups), g_end = min(n_groups, g_begin + per);

  // rows past the end are clamped onto the last valid one (never stored)
  const uint16_t* xrow[TB];
#pragma unroll
  for (int b = 0; b < TB; b++) xrow[b] = x + (size_t)min(t0 + 16 * b + n, T - 1) * d + 8 * kg;
  const uint16_t* wrow[NEB];
#pragma unroll
  for (int m = 0; m < NEB; m++) wrow[m] = w_router + (size_t)min(e0 + 16 * m + n, E - 1) * d + 8 * kg;

  r_f32x4 acc[NEB][TB];
#pragma unroll
  for (int m = 0; m < NEB; m++)
#pragma unroll
    for (int b = 0; b < TB; b++) acc[m][b] = r_f32x4{0.f, 0.f, 0.f, 0.f};

  // fragments of k-group g: x from HBM (touched once: non-temporal), W_r from the L2
  auto load = [&](r_bf16x8 (&xf)[TB], r_bf16x8 (&wf)[NEB], int g) __attribute__((always_inline)) {
#pragma unroll
    for (int b = 0; b < TB; b++) xf[b] = __builtin_nontemporal_load(reinterpret_cast<const r_bf16x8*>(xrow[b] + (size_t)g * 32));
#pragma unroll
    for (int m = 0; m < NEB; m++) wf[m] = *reinterpret_cast<const r_bf16x8*>(wrow[m] + (size_t)g * 32);
  };
  auto multiply = [&](const r_bf16x8 (&xf)[TB], const r_bf16x8 (&wf)[NEB]) __attribute__((always_inline)) {
#pragma unroll
    for (int m = 0; m < NEB; m++)
#pragma unroll
      for (int b = 0; b < TB; b++) acc[m][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[m], xf[b], acc[m][b], 0, 0, 0);
  };
  // two k-groups in flight: while one is multiplied the next one's loads are already out
  r_bf16x8 x0[TB], x1[TB], w0[NEB], w1[NEB];
  if (g_begin < g_end) load(x0, w0, g_begin);
  for (int g = g_begin; g < g_end; g += 2) {
    if (g + 1 < g_end) load(x1, w1, g + 1);
    multiply(x0, w0);
    if (g + 1 < g_end) {
      if (g + 2 < g_end) load(x0, w0, g + 2);
      multiply(x1, w1);
    }
  }

  // the 8 parts of K meet in LDS, one 16 x 16 block at a time, and are added in part order; thread i of the block
  // then owns logit (token i / 16, expert i % 16) of the block: 16 consecutive experts of a row per 16 threads
  const int rt = threadIdx.x >> 4, re = threadIdx.x & 15;
#pragma unroll
  for (int m = 0; m < NEB; m++) {
    if (e0 + 16 * m >= E) break;   // (uniform over the block)
#pragma unroll
    for (int b = 0; b < TB; b++) {
      *reinterpret_cast<r_f32x4*>(&part_sum[wave][n * 16 + 4 * kg]) = acc[m][b];   // [token][expert]
      __syncthreads();
      if (threadIdx.x < 256) {
        float s = 0.f;
#pragma unroll
        for (int p = 0; p < kRouterWaves; p++) s += part_sum[p][threadIdx.x];
        const int t = t0 + 16 * b + rt, e = e0 + 16 * m + re;
        if (t < T && e < E) logits[(size_t)t * E + e] = s;
      }
      __syncthreads();
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
