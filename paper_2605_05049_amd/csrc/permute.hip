// Local pack / unpack around the expert FFNs (the per-GPU halves of the dispatch and combine of Section III-B):
// a deterministic stable counting sort of the T*K' slots by expert id, the row gather it defines, the weighted
// combine that undoes it, and the derivatives of both.
//
// Counting sort = three launches, no atomics (so the order never depends on scheduling):
//   1. rank    : each block ranks 1024 consecutive slots among the same-expert slots of the block
//                (wave ballots give the rank inside 64 slots, an LDS table chains the 16 sub-groups) and
//                emits its expert histogram;
//   2. scan    : one block turns the per-block histograms into per-block bases, counts and offsets;
//   3. scatter : one wavefront per token finishes row = base + rank, writes both maps and copies the token's
//                row to its K' destinations (each source row is read from HBM once).
// The copy kernels are pure HBM streaming with 16-byte accesses per lane.
#include "common.h"

namespace moe {

constexpr int kSub = kPermSlotsPerBlock / kWave;  // 16 sub-groups of 64 slots per block

__device__ __forceinline__ int clamp_expert(int e, int Et) { return e < 0 ? 0 : (e >= Et ? Et - 1 : e); }

// ---------------------------------------------------------------------------------------------------------
// 1. rank
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void perm_rank_kernel(const int32_t* __restrict__ topk_idx, int32_t* __restrict__ lrank,
                                                        int32_t* __restrict__ block_hist, int N, int Et, int nbits) {
  extern __shared__ uint16_t sub_hist[];  // [kSub][Et]: count, then exclusive prefix over the sub-groups
  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = tid / kWave;
  const long long base = (long long)blockIdx.x * kPermSlotsPerBlock;
  for (int i = tid; i < kSub * Et; i += 256) sub_hist[i] = 0;
  __syncthreads();

  int key[4], rank_in_sub[4];
#pragma unroll
  for (int r = 0; r < 4; r++) {
    const int sub = r * 4 + wave;
    const long long s = base + sub * kWave + lane;
    const bool valid = s < N;
    const int e = valid ? clamp_expert(topk_idx[s], Et) : 0;
    unsigned long long peers = __ballot(valid);
    for (int b = 0; b < nbits; b++) {
      const bool bit = (e >> b) & 1;
      const unsigned long long bal = __ballot(bit);
      peers &= bit ? bal : ~bal;
    }
    const unsigned long long lower = peers & ((1ull << lane) - 1ull);
    key[r] = e;
    rank_in_sub[r] = __popcll(lower);
    if (valid && lower == 0) sub_hist[sub * Et + e] = (uint16_t)__popcll(peers);
  }
  __syncthreads();
  for (int e = tid; e < Et; e += 256) {
    int run = 0;
#pragma unroll
    for (int sub = 0; sub < kSub; sub++) {
      int c = sub_hist[sub * Et + e];
      sub_hist[sub * Et + e] = (uint16_t)run;
      run += c;
    }
    block_hist[(size_t)blockIdx.x * Et + e] = run;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 4; r++) {
    const int sub = r * 4 + wave;
    const long long s = base + sub * kWave + lane;
    if (s < N) lrank[s] = sub_hist[sub * Et + key[r]] + rank_in_sub[r];
  }
}

// ---------------------------------------------------------------------------------------------------------
// 2. scan: block_hist[b][e] -> offsets[e] + sum_{b'<b} block_hist[b'][e]; counts; offsets
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void perm_scan_kernel(int32_t* __restrict__ block_hist, int32_t* __restrict__ counts,
                                                         int32_t* __restrict__ offsets, int nblk, int Et) {
  __shared__ int32_t tot[kMaxExperts];
  __shared__ int32_t scan[kMaxExperts];
  const int e = threadIdx.x;
  int total = 0;
  if (e < Et) {
    for (int b = 0; b < nblk; b++) total += block_hist[(size_t)b * Et + e];
  }
  tot[e] = (e < Et) ? total : 0;
  scan[e] = tot[e];
  __syncthreads();
  // Hillis-Steele inclusive scan over the (at most 1024) experts
  for (int o = 1; o < kMaxExperts; o <<= 1) {
    int v = (e >= o) ? scan[e - o] : 0;
    __syncthreads();
    scan[e] += v;
    __syncthreads();
  }
  if (e < Et) {
    const int off = scan[e] - tot[e];
    counts[e] = tot[e];
    offsets[e] = off;
    if (e == Et - 1) offsets[Et] = scan[e];
    int run = off;
    for (int b = 0; b < nblk; b++) {
      int c = block_hist[(size_t)b * Et + e];
      block_hist[(size_t)b * Et + e] = run;
      run += c;
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// 3. scatter the maps and gather the rows: one wavefront per token
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void perm_scatter_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ topk_idx,
                                                           const int32_t* __restrict__ lrank, const int32_t* __restrict__ block_base,
                                                           uint4* __restrict__ x_perm, int32_t* __restrict__ row_of_slot,
                                                           int32_t* __restrict__ slot_of_row, int T, int Kp, int Et, int dvec) {
  const int lane = threadIdx.x % kWave;
  const int t = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + threadIdx.x / kWave);
  if (t >= T) return;
  const uint4* src = x ? x + (size_t)t * dvec : nullptr;
  for (int j = 0; j < Kp; j++) {
    const int s = t * Kp + j;
    const int e = clamp_expert(topk_idx[s], Et);
    const int row = block_base[(size_t)(s / kPermSlotsPerBlock) * Et + e] + lrank[s];
    if (lane == 0) {
      row_of_slot[s] = row;
      slot_of_row[row] = s;
    }
    if (src) {
      uint4* dst = x_perm + (size_t)row * dvec;
      for (int v = lane; v < dvec; v += kWave) dst[v] = src[v];
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// combine: out[t] = sum_j w[t,j] * y[row_of_slot[t*K'+j]]   (UNIT = true: all weights 1 -> permute_bwd)
// ---------------------------------------------------------------------------------------------------------
__device__ __forceinline__ void fma_bf16x8(float (&acc)[8], const uint4& v, float w) {
  acc[0] += w * bf16lo(v.x); acc[1] += w * bf16hi(v.x);
  acc[2] += w * bf16lo(v.y); acc[3] += w * bf16hi(v.y);
  acc[4] += w * bf16lo(v.z); acc[5] += w * bf16hi(v.z);
  acc[6] += w * bf16lo(v.w); acc[7] += w * bf16hi(v.w);
}

template <bool UNIT>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ y, const int32_t* __restrict__ row_of_slot,
                                                      const float* __restrict__ topk_w, uint4* __restrict__ out, int T, int Kp,
                                                      int dvec) {
  const int lane = threadIdx.x % kWave;
  const int t = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + threadIdx.x / kWave);
  if (t >= T) return;
  const int32_t* rows = row_of_slot + (size_t)t * Kp;
  const float* w = UNIT ? nullptr : topk_w + (size_t)t * Kp;
  for (int v = lane; v < dvec; v += kWave) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < Kp; j++) {
      const uint4 val = y[(size_t)rows[j] * dvec + v];
      fma_bf16x8(acc, val, UNIT ? 1.0f : w[j]);
    }
    uint4 o;
    o.x = pack_bf16(acc[0], acc[1]); o.y = pack_bf16(acc[2], acc[3]);
    o.z = pack_bf16(acc[4], acc[5]); o.w = pack_bf16(acc[6], acc[7]);
    out[(size_t)t * dvec + v] = o;
  }
}

// combine_bwd: dy[row] = bf16(w * dout[t]);  dw[t,j] = <dout[t], y[row]>
__global__ __launch_bounds__(256) void combine_bwd_kernel(const uint4* __restrict__ dout, const uint4* __restrict__ y,
                                                          const int32_t* __restrict__ row_of_slot, const float* __restrict__ topk_w,
                                                          uint4* __restrict__ dy, float* __restrict__ dtopk_w, int T, int Kp, int dvec) {
  const int lane = threadIdx.x % kWave;
  const int t = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + threadIdx.x / kWave);
  if (t >= T) return;
  const uint4* g = dout + (size_t)t * dvec;
  for (int j = 0; j < Kp; j++) {
    const int s = t * Kp + j;
    const int row = row_of_slot[s];
    const float w = topk_w[s];
    const uint4* yr = y + (size_t)row * dvec;
    uint4* dyr = dy + (size_t)row * dvec;
    float dot = 0.f;
    for (int v = lane; v < dvec; v += kWave) {
      const uint4 gv = g[v];
      const uint4 yv = yr[v];
      float a[8] = {bf16lo(gv.x), bf16hi(gv.x), bf16lo(gv.y), bf16hi(gv.y), bf16lo(gv.z), bf16hi(gv.z), bf16lo(gv.w), bf16hi(gv.w)};
      float b[8] = {bf16lo(yv.x), bf16hi(yv.x), bf16lo(yv.y), bf16hi(yv.y), bf16lo(yv.z), bf16hi(yv.z), bf16lo(yv.w), bf16hi(yv.w)};
      uint4 o;
      o.x = pack_bf16(w * a[0], w * a[1]); o.y = pack_bf16(w * a[2], w * a[3]);
      o.z = pack_bf16(w * a[4], w * a[5]); o.w = pack_bf16(w * a[6], w * a[7]);
      dyr[v] = o;
#pragma unroll
      for (int q = 0; q < 8; q++) dot += a[q] * b[q];
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, kWave);
    if (lane == 0) dtopk_w[s] = dot;
  }
}

}  // namespace moe

extern "C" int moe_permute(const moe_shape* shape, const uint16_t* x, const int32_t* topk_idx, uint16_t* x_perm,
                           int32_t* counts, int32_t* offsets, int32_t* row_of_slot, int32_t* slot_of_row,
                           void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  Dims D;
  int rc = check_shape(shape, &D);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(topk_idx); MOE_REQUIRE_PTR(counts); MOE_REQUIRE_PTR(offsets); MOE_REQUIRE_PTR(row_of_slot);
  MOE_REQUIRE_PTR(slot_of_row); MOE_REQUIRE_PTR(ws);
  if ((x == nullptr) != (x_perm == nullptr)) return MOE_ERR_NULL;
  MOE_REQUIRE_ALIGNED(x); MOE_REQUIRE_ALIGNED(topk_idx); MOE_REQUIRE_ALIGNED(x_perm); MOE_REQUIRE_ALIGNED(counts);
  MOE_REQUIRE_ALIGNED(offsets); MOE_REQUIRE_ALIGNED(row_of_slot); MOE_REQUIRE_ALIGNED(slot_of_row);
  if (!aligned(ws, 256)) return MOE_ERR_ALIGN;
  const WsLayout L = ws_layout(D);
  if (ws_bytes < L.total) return MOE_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  int32_t* block_hist = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.perm_hist);
  int32_t* lrank = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.perm_rank);
  const int nblk = perm_num_blocks(D.N);
  int nbits = 0;
  while ((1 << nbits) < D.Et) nbits++;
  if (nblk > 0) {
    MOE_LAUNCH("perm_rank", st, perm_rank_kernel, dim3(nblk), dim3(256), (size_t)kSub * D.Et * sizeof(uint16_t), st, topk_idx, lrank,
                       block_hist, (int)D.N, D.Et, nbits);
  }
  // with no slots the scan still defines counts = 0 and offsets = 0
  MOE_LAUNCH("perm_scan", st, perm_scan_kernel, dim3(1), dim3(1024), 0, st, block_hist, counts, offsets, nblk, D.Et);
  if (D.T > 0) {
    MOE_LAUNCH("perm_scatter_gather", st, perm_scatter_kernel, dim3((D.T + 3) / 4), dim3(256), 0, st, reinterpret_cast<const uint4*>(x), topk_idx,
                       lrank, block_hist, reinterpret_cast<uint4*>(x_perm), row_of_slot, slot_of_row, D.T, D.Kp, D.Et, D.d / 8);
  }
  return launch_status();
}

extern "C" int moe_permute_bwd(const moe_shape* shape, const uint16_t* dx_perm, const int32_t* row_of_slot,
                               uint16_t* dx, void* stream) {
  using namespace moe;
  Dims D;
  int rc = check_shape(shape, &D);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(dx_perm); MOE_REQUIRE_PTR(row_of_slot); MOE_REQUIRE_PTR(dx);
  MOE_REQUIRE_ALIGNED(dx_perm); MOE_REQUIRE_ALIGNED(row_of_slot); MOE_REQUIRE_ALIGNED(dx);
  if (D.T == 0) return MOE_OK;
  MOE_LAUNCH("permute_bwd", (hipStream_t)stream, (combine_kernel<true>), dim3((D.T + 3) / 4), dim3(256), 0, (hipStream_t)stream,
                     reinterpret_cast<const uint4*>(dx_perm), row_of_slot, (const float*)nullptr, reinterpret_cast<uint4*>(dx),
                     D.T, D.Kp, D.d / 8);
  return launch_status();
}

extern "C" int moe_unpermute_combine(const moe_shape* shape, const uint16_t* y_perm, const int32_t* row_of_slot,
                                     const float* topk_w, uint16_t* out, void* stream) {
  using namespace moe;
  Dims D;
  int rc = check_shape(shape, &D);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(y_perm); MOE_REQUIRE_PTR(row_of_slot); MOE_REQUIRE_PTR(topk_w); MOE_REQUIRE_PTR(out);
  MOE_REQUIRE_ALIGNED(y_perm); MOE_REQUIRE_ALIGNED(row_of_slot); MOE_REQUIRE_ALIGNED(topk_w); MOE_REQUIRE_ALIGNED(out);
  if (D.T == 0) return MOE_OK;
  MOE_LAUNCH("unpermute_combine", (hipStream_t)stream, (combine_kernel<false>), dim3((D.T + 3) / 4), dim3(256), 0, (hipStream_t)stream,
                     reinterpret_cast<const uint4*>(y_perm), row_of_slot, topk_w, reinterpret_cast<uint4*>(out), D.T, D.Kp,
                     D.d / 8);
  return launch_status();
}

extern "C" int moe_unpermute_combine_bwd(const moe_shape* shape, const uint16_t* dout, const uint16_t* y_perm,
                                         const int32_t* row_of_slot, const float* topk_w, uint16_t* dy_perm,
                                         float* dtopk_w, void* stream) {
  using namespace moe;
  Dims D;
  int rc = check_shape(shape, &D);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(dout); MOE_REQUIRE_PTR(y_perm); MOE_REQUIRE_PTR(row_of_slot); MOE_REQUIRE_PTR(topk_w);
  MOE_REQUIRE_PTR(dy_perm); MOE_REQUIRE_PTR(dtopk_w);
  MOE_REQUIRE_ALIGNED(dout); MOE_REQUIRE_ALIGNED(y_perm); MOE_REQUIRE_ALIGNED(row_of_slot); MOE_REQUIRE_ALIGNED(topk_w);
  MOE_REQUIRE_ALIGNED(dy_perm); MOE_REQUIRE_ALIGNED(dtopk_w);
  if (D.T == 0) return MOE_OK;
  MOE_LAUNCH("unpermute_combine_bwd", (hipStream_t)stream, combine_bwd_kernel, dim3((D.T + 3) / 4), dim3(256), 0, (hipStream_t)stream,
                     reinterpret_cast<const uint4*>(dout), reinterpret_cast<const uint4*>(y_perm), row_of_slot, topk_w,
                     reinterpret_cast<uint4*>(dy_perm), dtopk_w, D.T, D.Kp, D.d / 8);
  return launch_status();
}
