// Top-k softmax gating and its derivative (Section II-A: learned gating function; Section III-A: E, E_s, k).
//
// One group of W lanes (W = 8..64, a power of two) owns one token; lane g holds logits g, g+W, g+2W, ...
// Max, sum-of-exp and each of the k arg-max rounds are butterfly reductions inside the group, so a 64-wide
// wavefront serves 64/W tokens at once when E is small.  HBM traffic is T*E*4 bytes in, T*K'*8 out: trivial.
#include "common.h"

namespace moe {

template <int W>
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int o = W / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, W));
  return v;
}
template <int W>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = W / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, W);
  return v;
}

// (value, index) ordering of the selection: larger logit first, equal logits -> lower expert id first.
__device__ __forceinline__ bool better(float v, int i, float v2, int i2) { return v > v2 || (v == v2 && i < i2); }

template <int W, int PER>
__global__ __launch_bounds__(256) void route_topk_kernel(const float* __restrict__ logits, int32_t* __restrict__ topk_idx,
                                                         float* __restrict__ topk_w, float* __restrict__ probs_save,
                                                         int T, int E, int k, int Es, int renorm) {
  const int Kp = k + Es;
  const int g = threadIdx.x % W;
  const int t = (blockIdx.x * 256 + threadIdx.x) / W;
  if (t >= T) return;  // whole groups leave together (256 % W == 0), shuffles below stay inside a group
  const float NEG_INF = -__builtin_inff();
  float val[PER];
  bool taken[PER];
#pragma unroll
  for (int p = 0; p < PER; p++) {
    int e = g + p * W;
    float v = (e < E) ? logits[(size_t)t * E + e] : NEG_INF;
    val[p] = (v != v) ? NEG_INF : v;  // NaN -> -inf keeps every selected index in range
    taken[p] = (e >= E);
  }
  float m = NEG_INF;
#pragma unroll
  for (int p = 0; p < PER; p++) m = fmaxf(m, val[p]);
  m = group_max<W>(m);
  float ex[PER];
  float z = 0.f;
#pragma unroll
  for (int p = 0; p < PER; p++) {
    ex[p] = (g + p * W < E) ? expf(val[p] - m) : 0.f;
    z += ex[p];
  }
  z = group_sum<W>(z);
  const float inv_z = 1.0f / z;
  if (probs_save) {
#pragma unroll
    for (int p = 0; p < PER; p++)
      if (g + p * W < E) probs_save[(size_t)t * E + g + p * W] = ex[p] * inv_z;
  }

  float held[PER];  // selection j is parked on lane j % W, slot j / W, until the sum over the k is known
#pragma unroll
  for (int p = 0; p < PER; p++) held[p] = 0.f;
  float sel_sum = 0.f;
  for (int j = 0; j < k; j++) {
    float bv = NEG_INF;
    int bi = 0x7fffffff;
    float bp = 0.f;
#pragma unroll
    for (int p = 0; p < PER; p++) {
      int e = g + p * W;
      if (!taken[p] && better(val[p], e, bv, bi)) { bv = val[p]; bi = e; bp = ex[p]; }
    }
#pragma unroll
    for (int o = W / 2; o > 0; o >>= 1) {
      float ov = __shfl_xor(bv, o, W);
      int oi = __shfl_xor(bi, o, W);
      float op = __shfl_xor(bp, o, W);
      if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; bp = op; }
    }
    // bi is now the same on every lane of the group
#pragma unroll
    for (int p = 0; p < PER; p++)
      if (g + p * W == bi) taken[p] = true;
    float pj = bp * inv_z;
    sel_sum += pj;
    if (g == 0) topk_idx[(size_t)t * Kp + j] = bi;
#pragma unroll
    for (int p = 0; p < PER; p++)
      if (g == j % W && p == j / W) held[p] = pj;
  }
  const float scale = renorm ? 1.0f / sel_sum : 1.0f;
#pragma unroll
  for (int p = 0; p < PER; p++) {
    int j = g + p * W;
    if (j < k) topk_w[(size_t)t * Kp + j] = held[p] * scale;
  }
  for (int j = g; j < Es; j += W) {
    topk_idx[(size_t)t * Kp + k + j] = E + j;
    topk_w[(size_t)t * Kp + k + j] = 1.0f;
  }
}

template <int W>
__global__ __launch_bounds__(256) void route_topk_bwd_kernel(const float* __restrict__ dtopk_w, const int32_t* __restrict__ topk_idx,
                                                             const float* __restrict__ topk_w, const float* __restrict__ probs,
                                                             float* __restrict__ dlogits, int T, int E, int k, int Es, int renorm) {
  const int Kp = k + Es;
  const int g = threadIdx.x % W;
  const int t = (blockIdx.x * 256 + threadIdx.x) / W;
  if (t >= T) return;
  const float* dw = dtopk_w + (size_t)t * Kp;
  const float* w = topk_w + (size_t)t * Kp;
  const int32_t* idx = topk_idx + (size_t)t * Kp;
  float inner = 0.f;  // sum_j w_j dw_j (w_j is the selected probability itself when renorm is off)
  for (int j = g; j < k; j += W) inner += w[j] * dw[j];
  inner = group_sum<W>(inner);
  for (int mcol = g; mcol < E; mcol += W) {
    float pm = renorm ? 0.f : probs[(size_t)t * E + mcol];
    float out = renorm ? 0.f : -pm * inner;
    for (int j = 0; j < k; j++) {
      if (idx[j] == mcol) out += renorm ? w[j] * (dw[j] - inner) : pm * dw[j];
    }
    dlogits[(size_t)t * E + mcol] = out;
  }
}

template <int W, int PER>
static void launch_route(const Dims& D, const float* logits, int32_t* idx, float* w, float* probs, hipStream_t st) {
  int groups_per_block = 256 / W;
  int blocks = (D.T + groups_per_block - 1) / groups_per_block;
  MOE_LAUNCH("route_topk", st, (route_topk_kernel<W, PER>), dim3(blocks), dim3(256), 0, st, logits, idx, w, probs, D.T, D.E, D.k, D.Es,
                     D.renorm);
}

}  // namespace moe

extern "C" int moe_route_topk(const moe_shape* shape, const float* logits, int32_t* topk_idx, float* topk_w,
                              float* probs_save, void* stream) {
  using namespace moe;
  Dims D;
  int rc = check_shape(shape, &D);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(logits); MOE_REQUIRE_PTR(topk_idx); MOE_REQUIRE_PTR(topk_w);
  MOE_REQUIRE_ALIGNED(logits); MOE_REQUIRE_ALIGNED(topk_idx); MOE_REQUIRE_ALIGNED(topk_w); MOE_REQUIRE_ALIGNED(probs_save);
  if (D.T == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)stream;
  if (D.E <= 8) launch_route<8, 1>(D, logits, topk_idx, topk_w, probs_save, st);
  else if (D.E <= 16) launch_route<16, 1>(D, logits, topk_idx, topk_w, probs_save, st);
  else if (D.E <= 32) launch_route<32, 1>(D, logits, topk_idx, topk_w, probs_save, st);
  else if (D.E <= 64) launch_route<64, 1>(D, logits, topk_idx, topk_w, probs_save, st);
  else if (D.E <= 128) launch_route<64, 2>(D, logits, topk_idx, topk_w, probs_save, st);
  else if (D.E <= 256) launch_route<64, 4>(D, logits, topk_idx, topk_w, probs_save, st);
  else if (D.E <= 512) launch_route<64, 8>(D, logits, topk_idx, topk_w, probs_save, st);
  else launch_route<64, 16>(D, logits, topk_idx, topk_w, probs_save, st);
  return launch_status();
}

extern "C" int moe_route_topk_bwd(const moe_shape* shape, const float* dtopk_w, const int32_t* topk_idx,
                                  const float* topk_w, const float* probs_save, float* dlogits, void* stream) {
  using namespace moe;
  Dims D;
  int rc = check_shape(shape, &D);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(dtopk_w); MOE_REQUIRE_PTR(topk_idx); MOE_REQUIRE_PTR(topk_w); MOE_REQUIRE_PTR(dlogits);
  if (!D.renorm) MOE_REQUIRE_PTR(probs_save);
  MOE_REQUIRE_ALIGNED(dtopk_w); MOE_REQUIRE_ALIGNED(topk_idx); MOE_REQUIRE_ALIGNED(topk_w); MOE_REQUIRE_ALIGNED(probs_save);
  MOE_REQUIRE_ALIGNED(dlogits);
  if (D.T == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)stream;
#define MOE_LAUNCH_RBWD(W_)                                                                                              \
  MOE_LAUNCH("route_topk_bwd", st, (route_topk_bwd_kernel<W_>), dim3((D.T + 256 / W_ - 1) / (256 / W_)), dim3(256), 0, st, dtopk_w,   \
                     topk_idx, topk_w, probs_save, dlogits, D.T, D.E, D.k, D.Es, D.renorm)
  if (D.E <= 8) MOE_LAUNCH_RBWD(8);
  else if (D.E <= 16) MOE_LAUNCH_RBWD(16);
  else if (D.E <= 32) MOE_LAUNCH_RBWD(32);
  else MOE_LAUNCH_RBWD(64);
#undef MOE_LAUNCH_RBWD
  return launch_status();
}
