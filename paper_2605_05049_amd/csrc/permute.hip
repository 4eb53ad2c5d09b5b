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

#include <mutex>

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
  // Thread (g, e): expert e, blocks [g*chunk, (g+1)*chunk).  G = 1024 / E' groups share the walk over the blocks.
  __shared__ int32_t part[kMaxExperts];   // [G][Et] chunk totals, then exclusive prefixes over g
  __shared__ int32_t tot[kMaxExperts];
  __shared__ int32_t scan[kMaxExperts];
  const int tid = threadIdx.x;
  const int G = kMaxExperts / Et;
  const int g = tid / Et, e = tid % Et;
  const int chunk = (nblk + G - 1) / G;
  const int b0 = g * chunk, b1 = min(nblk, b0 + chunk);
  const bool active = g < G;
  int sum = 0;
  if (active)
    for (int b = b0; b < b1; b += 8) {   // 8 loads in flight
      int c[8];
#pragma unroll
      for (int j = 0; j < 8; j++) c[j] = (b + j < b1) ? block_hist[(size_t)(b + j) * Et + e] : 0;
#pragma unroll
      for (int j = 0; j < 8; j++) sum += c[j];
    }
  if (active) part[g * Et + e] = sum;
  __syncthreads();
  if (tid < Et) {
    int run = 0;
    for (int gg = 0; gg < G; gg++) {
      const int c = part[gg * Et + tid];
      part[gg * Et + tid] = run;
      run += c;
    }
    tot[tid] = run;
  } else {
    tot[tid] = 0;
  }
  // inclusive scan over the (at most 1024) experts: inside each wavefront with lane shuffles, then over the 16
  // wavefront totals
  __shared__ int32_t wave_total[kMaxExperts / kWave];
  __syncthreads();
  {
    const int lane = tid % kWave, wv = tid / kWave;
    int v = (tid < Et) ? tot[tid] : 0;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(v, o, kWave);
      if (lane >= o) v += up;
    }
    if (lane == kWave - 1) wave_total[wv] = v;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wv; w++) before += wave_total[w];
    scan[tid] = v + before;
  }
  __syncthreads();
  if (tid < Et) {
    counts[tid] = tot[tid];
    offsets[tid] = scan[tid] - tot[tid];
    if (tid == Et - 1) offsets[Et] = scan[tid];
  }
  if (active) {
    int run = scan[e] - tot[e] + part[g * Et + e];
    for (int b = b0; b < b1; b += 8) {   // 8 loads in flight
      int c[8];
#pragma unroll
      for (int j = 0; j < 8; j++) c[j] = (b + j < b1) ? block_hist[(size_t)(b + j) * Et + e] : 0;
#pragma unroll
      for (int j = 0; j < 8; j++) {
        if (b + j < b1) block_hist[(size_t)(b + j) * Et + e] = run;
        run += c[j];
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// The streaming kernels below give a token to `parts` (1, 2 or 4) wavefronts of one block, each of which takes a
// contiguous part of the row: with rows of 256 vectors or more a block of four wavefronts then works on ONE token,
// i.e. on 1 + K' rows of 8 KB at a time instead of on 4 (1 + K'), which keeps its accesses inside few DRAM pages
// (measured on the imbalance shape: combine 66 -> 74 % of the HBM peak).  KP is the number of slots per token K' when
// it is small (1..8: the slot loop is unrolled, all K' row indices are fetched up front and the K' row accesses of a
// vector are in flight together); KP = 0 is the general loop for any K'.  Rows move as 16-byte vectors per lane, a
// few vectors per lane at a time, with non-temporal hints where they measured faster (each byte is touched once).
// ---------------------------------------------------------------------------------------------------------
constexpr int CHUNK = 4;  // 16-byte vectors per lane held in registers at once (4 x 64 x 16 B = 4 KB of a row)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Cache policy per kernel, chosen by measurement on the imbalance shape (671 MB per launch, cold caches, one block
// per token): the scatter runs 2 % faster with ordinary accesses, the combine 7 % and the combine backward 4 % faster
// with non-temporal loads and stores.
constexpr bool kGatherNT = false, kCombineNT = true, kCombineBwdNT = true;
// Wavefronts per token: 4 for rows of at least 256 vectors (d_model >= 2048), else 2 or 1 (at least 64 vectors each).
static int row_parts(int dvec) { return dvec >= 256 ? 4 : (dvec >= 128 ? 2 : 1); }
static unsigned token_blocks(int T, int parts) { return (unsigned)(((long long)T * parts + 3) / 4); }
template <bool NT> __device__ __forceinline__ u32x4 ld_row(const u32x4* p) { return NT ? __builtin_nontemporal_load(p) : *p; }
template <bool NT> __device__ __forceinline__ void st_row(u32x4* p, u32x4 v) {
  if (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// ---------------------------------------------------------------------------------------------------------
// 3. scatter the maps and gather the rows
// ---------------------------------------------------------------------------------------------------------
template <int KP>
__global__ __launch_bounds__(256) void perm_scatter_kernel(const u32x4* __restrict__ x, const int32_t* __restrict__ topk_idx,
                                                           const int32_t* __restrict__ lrank, const int32_t* __restrict__ block_base,
                                                           u32x4* __restrict__ x_perm, int32_t* __restrict__ row_of_slot,
                                                           int32_t* __restrict__ slot_of_row, int T, int Kp, int Et, int dvec, int parts) {
  const int lane = threadIdx.x % kWave;
  const int wid = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + threadIdx.x / kWave);
  const int t = wid / parts, part = wid % parts;
  if (t >= T) return;
  const int part_len = (dvec + parts - 1) / parts;
  const int v_begin = part * part_len, v_end = min(dvec, v_begin + part_len);
  const u32x4* src = x ? x + (size_t)t * dvec : nullptr;
  if (KP > 0) {
    int rows[KP > 0 ? KP : 1];
#pragma unroll
    for (int j = 0; j < KP; j++) {
      const int s = t * KP + j;
      const int e = clamp_expert(topk_idx[s], Et);
      rows[j] = block_base[(size_t)(s / kPermSlotsPerBlock) * Et + e] + lrank[s];
    }
    if (part == 0 && lane < KP) {
      int row = rows[0];
#pragma unroll
      for (int j = 1; j < KP; j++) row = (lane == j) ? rows[j] : row;
      row_of_slot[t * KP + lane] = row;
      slot_of_row[row] = t * KP + lane;
    }
    if (src) {
      for (int v0 = v_begin; v0 < v_end; v0 += CHUNK * kWave) {
        u32x4 r[CHUNK];
#pragma unroll
        for (int i = 0; i < CHUNK; i++) {
          const int v = v0 + i * kWave + lane;
          if (v < v_end) r[i] = ld_row<kGatherNT>(src + v);
        }
#pragma unroll
        for (int j = 0; j < KP; j++) {
          u32x4* dst = x_perm + (size_t)rows[j] * dvec;
#pragma unroll
          for (int i = 0; i < CHUNK; i++) {
            const int v = v0 + i * kWave + lane;
            if (v < v_end) st_row<kGatherNT>(dst + v, r[i]);
          }
        }
      }
    }
  } else {
    for (int j = 0; j < Kp; j++) {
      const int s = t * Kp + j;
      const int e = clamp_expert(topk_idx[s], Et);
      const int row = block_base[(size_t)(s / kPermSlotsPerBlock) * Et + e] + lrank[s];
      if (part == 0 && lane == 0) {
        row_of_slot[s] = row;
        slot_of_row[row] = s;
      }
      if (src) {
        u32x4* dst = x_perm + (size_t)row * dvec;
        for (int v = v_begin + lane; v < v_end; v += kWave) st_row<kGatherNT>(dst + v, src[v]);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// combine: out[t] = sum_j w[t,j] * y[row_of_slot[t*K'+j]]   (UNIT = true: all weights 1 -> permute_bwd)
// ---------------------------------------------------------------------------------------------------------
__device__ __forceinline__ void fma_bf16x8(float (&acc)[8], const u32x4& v, float w) {
  acc[0] += w * bf16lo(v.x); acc[1] += w * bf16hi(v.x);
  acc[2] += w * bf16lo(v.y); acc[3] += w * bf16hi(v.y);
  acc[4] += w * bf16lo(v.z); acc[5] += w * bf16hi(v.z);
  acc[6] += w * bf16lo(v.w); acc[7] += w * bf16hi(v.w);
}
__device__ __forceinline__ u32x4 pack8(const float (&a)[8]) {
  u32x4 o;
  o.x = pack_bf16(a[0], a[1]); o.y = pack_bf16(a[2], a[3]); o.z = pack_bf16(a[4], a[5]); o.w = pack_bf16(a[6], a[7]);
  return o;
}

template <int KP, bool UNIT>
__global__ __launch_bounds__(256) void combine_kernel(const u32x4* __restrict__ y, const int32_t* __restrict__ row_of_slot,
                                                      const float* __restrict__ topk_w, const u32x4* __restrict__ addend,
                                                      u32x4* __restrict__ out, int T, int Kp, int dvec, int parts) {
  const int lane = threadIdx.x % kWave;
  const int wid = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + threadIdx.x / kWave);
  const int t = wid / parts;
  if (t >= T) return;
  const int part_len = (dvec + parts - 1) / parts;
  const int v_begin = (wid % parts) * part_len, v_end = min(dvec, v_begin + part_len);
  u32x4* dst = out + (size_t)t * dvec;
  if (KP > 0) {
    const u32x4* rowp[KP > 0 ? KP : 1];
    float w[KP > 0 ? KP : 1];
#pragma unroll
    for (int j = 0; j < KP; j++) {
      rowp[j] = y + (size_t)row_of_slot[(size_t)t * KP + j] * dvec;
      w[j] = UNIT ? 1.0f : topk_w[(size_t)t * KP + j];
    }
    constexpr int VU = (KP <= 4) ? 2 : 1;  // vectors per lane per iteration: keep KP*VU row loads in flight
    for (int v0 = v_begin; v0 < v_end; v0 += VU * kWave) {
      u32x4 val[VU][KP > 0 ? KP : 1];
#pragma unroll
      for (int i = 0; i < VU; i++) {
        const int v = v0 + i * kWave + lane;
        if (v < v_end) {
#pragma unroll
          for (int j = 0; j < KP; j++) val[i][j] = ld_row<kCombineNT>(rowp[j] + v);
        }
      }
#pragma unroll
      for (int i = 0; i < VU; i++) {
        const int v = v0 + i * kWave + lane;
        if (v < v_end) {
          float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int j = 0; j < KP; j++) fma_bf16x8(acc, val[i][j], w[j]);  // slot order, fp32
          if (addend) fma_bf16x8(acc, addend[(size_t)t * dvec + v], 1.0f);
          st_row<kCombineNT>(dst + v, pack8(acc));
        }
      }
    }
  } else {
    const int32_t* rows = row_of_slot + (size_t)t * Kp;
    const float* w = UNIT ? nullptr : topk_w + (size_t)t * Kp;
    for (int v = v_begin + lane; v < v_end; v += kWave) {
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int j = 0; j < Kp; j++) fma_bf16x8(acc, y[(size_t)rows[j] * dvec + v], UNIT ? 1.0f : w[j]);
      if (addend) fma_bf16x8(acc, addend[(size_t)t * dvec + v], 1.0f);
      st_row<kCombineNT>(dst + v, pack8(acc));
    }
  }
}

// combine_bwd: dy[row] = bf16(w * dout[t]);  dw[t,j] = <dout[t], y[row]>
template <int KP>
__global__ __launch_bounds__(256) void combine_bwd_kernel(const u32x4* __restrict__ dout, const u32x4* __restrict__ y,
                                                          const int32_t* __restrict__ row_of_slot, const float* __restrict__ topk_w,
                                                          u32x4* __restrict__ dy, float* __restrict__ dtopk_w, int T, int Kp, int dvec,
                                                          int parts) {
  // dot products of the parts of a row meet in LDS and are added in part order (the result never depends on timing)
  extern __shared__ float part_dot[];   // [4 wavefronts][K']
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int wid = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + wave);
  const int t = wid / parts, part = wid % parts;
  const bool active = t < T;   // (no early return: the block meets at a barrier below)
  const int part_len = (dvec + parts - 1) / parts;
  const int v_begin = active ? part * part_len : 0, v_end = active ? min(dvec, v_begin + part_len) : 0;
  const u32x4* g = dout + (size_t)(active ? t : 0) * dvec;
  if (KP > 0) {
    size_t rowoff[KP > 0 ? KP : 1];
    float w[KP > 0 ? KP : 1], dot[KP > 0 ? KP : 1];
#pragma unroll
    for (int j = 0; j < KP; j++) {
      rowoff[j] = active ? (size_t)row_of_slot[(size_t)t * KP + j] * dvec : 0;
      w[j] = active ? topk_w[(size_t)t * KP + j] : 0.f;
      dot[j] = 0.f;
    }
    constexpr int VU = (KP <= 4) ? 2 : 1;  // vectors per lane per iteration: (1 + KP) * VU row loads in flight
    for (int v0 = v_begin; v0 < v_end; v0 += VU * kWave) {
      u32x4 gv[VU], yv[VU][KP > 0 ? KP : 1];
#pragma unroll
      for (int i = 0; i < VU; i++) {
        const int v = v0 + i * kWave + lane;
        if (v < v_end) {
          gv[i] = ld_row<kCombineBwdNT>(g + v);
#pragma unroll
          for (int j = 0; j < KP; j++) yv[i][j] = ld_row<kCombineBwdNT>(y + rowoff[j] + v);
        }
      }
#pragma unroll
      for (int i = 0; i < VU; i++) {
        const int v = v0 + i * kWave + lane;
        if (v < v_end) {
          const u32x4 gg = gv[i];
          const float a[8] = {bf16lo(gg.x), bf16hi(gg.x), bf16lo(gg.y), bf16hi(gg.y), bf16lo(gg.z), bf16hi(gg.z), bf16lo(gg.w), bf16hi(gg.w)};
#pragma unroll
          for (int j = 0; j < KP; j++) {
            float sc[8];
#pragma unroll
            for (int q = 0; q < 8; q++) sc[q] = w[j] * a[q];
            st_row<kCombineBwdNT>(dy + rowoff[j] + v, pack8(sc));
            const u32x4 yy = yv[i][j];
            const float b[8] = {bf16lo(yy.x), bf16hi(yy.x), bf16lo(yy.y), bf16hi(yy.y), bf16lo(yy.z), bf16hi(yy.z), bf16lo(yy.w), bf16hi(yy.w)};
#pragma unroll
            for (int q = 0; q < 8; q++) dot[j] += a[q] * b[q];
          }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < KP; j++) {
      float dsum = dot[j];
#pragma unroll
      for (int o = kWave / 2; o > 0; o >>= 1) dsum += __shfl_xor(dsum, o, kWave);
      if (lane == 0) part_dot[wave * KP + j] = dsum;
    }
    __syncthreads();
    if (active && part == 0 && lane < KP) {
      float dsum = 0.f;
      for (int p2 = 0; p2 < parts; p2++) dsum += part_dot[(wave + p2) * KP + lane];
      dtopk_w[(size_t)t * KP + lane] = dsum;
    }
  } else {
    for (int j = 0; j < Kp; j++) {
      const int s = (active ? t : 0) * Kp + j;
      const size_t ro = (size_t)row_of_slot[s] * dvec;
      const float w = topk_w[s];
      float dot = 0.f;
      for (int v = v_begin + lane; v < v_end; v += kWave) {
        const u32x4 gv = g[v];
        const u32x4 yy = y[ro + v];
        const float a[8] = {bf16lo(gv.x), bf16hi(gv.x), bf16lo(gv.y), bf16hi(gv.y), bf16lo(gv.z), bf16hi(gv.z), bf16lo(gv.w), bf16hi(gv.w)};
        const float b[8] = {bf16lo(yy.x), bf16hi(yy.x), bf16lo(yy.y), bf16hi(yy.y), bf16lo(yy.z), bf16hi(yy.z), bf16lo(yy.w), bf16hi(yy.w)};
        float sc[8];
#pragma unroll
        for (int q = 0; q < 8; q++) { sc[q] = w * a[q]; dot += a[q] * b[q]; }
        st_row<kCombineBwdNT>(dy + ro + v, pack8(sc));
      }
#pragma unroll
      for (int o = kWave / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, kWave);
      if (lane == 0) part_dot[wave * Kp + j] = dot;
    }
    __syncthreads();
    if (active && part == 0)
      for (int j = lane; j < Kp; j += kWave) {
        float dsum = 0.f;
        for (int p2 = 0; p2 < parts; p2++) dsum += part_dot[(wave + p2) * Kp + j];
        dtopk_w[(size_t)t * Kp + j] = dsum;
      }
  }
}

// Picks the unrolled instantiation for K' = 1..8 and the general one otherwise.
#define MOE_DISPATCH_KP(Kp_, CALL)                                                     \
  switch (Kp_) {                                                                       \
    case 1: { constexpr int KP = 1; CALL; } break;                                     \
    case 2: { constexpr int KP = 2; CALL; } break;                                     \
    case 3: { constexpr int KP = 3; CALL; } break;                                     \
    case 4: { constexpr int KP = 4; CALL; } break;                                     \
    case 5: { constexpr int KP = 5; CALL; } break;                                     \
    case 6: { constexpr int KP = 6; CALL; } break;                                     \
    case 7: { constexpr int KP = 7; CALL; } break;                                     \
    case 8: { constexpr int KP = 8; CALL; } break;                                     \
    default: { constexpr int KP = 0; CALL; } break;                                    \
  }

}  // namespace moe

namespace moe {

// Host-side argument checks shared by the two entry points of the permutation.
static int permute_checks(const moe_shape* shape, Dims* D, const uint16_t* x, const int32_t* topk_idx, uint16_t* x_perm,
                          int32_t* counts, int32_t* offsets, int32_t* row_of_slot, int32_t* slot_of_row) {
  int rc = check_shape(shape, D);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(topk_idx); MOE_REQUIRE_PTR(counts); MOE_REQUIRE_PTR(offsets); MOE_REQUIRE_PTR(row_of_slot);
  MOE_REQUIRE_PTR(slot_of_row);
  if ((x == nullptr) != (x_perm == nullptr)) return MOE_ERR_NULL;
  MOE_REQUIRE_ALIGNED(x); MOE_REQUIRE_ALIGNED(topk_idx); MOE_REQUIRE_ALIGNED(x_perm); MOE_REQUIRE_ALIGNED(counts);
  MOE_REQUIRE_ALIGNED(offsets); MOE_REQUIRE_ALIGNED(row_of_slot); MOE_REQUIRE_ALIGNED(slot_of_row);
  return MOE_OK;
}

// The three launches of the counting sort.  block_hist: perm_num_blocks(N) * E' int32; lrank: N int32.  Every entry of
// both that a later kernel reads is written by an earlier one of the same call, so neither has to start at zero.
static int permute_launch(const Dims& D, const uint16_t* x, const int32_t* topk_idx, uint16_t* x_perm, int32_t* counts,
                          int32_t* offsets, int32_t* row_of_slot, int32_t* slot_of_row, int32_t* block_hist, int32_t* lrank,
                          hipStream_t st) {
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
    const int parts = x ? row_parts(D.d / 8) : 1;
    MOE_DISPATCH_KP(D.Kp, MOE_LAUNCH("perm_scatter_gather", st, (perm_scatter_kernel<KP>), dim3(token_blocks(D.T, parts)), dim3(256), 0, st,
                                     reinterpret_cast<const u32x4*>(x), topk_idx, lrank, block_hist, reinterpret_cast<u32x4*>(x_perm),
                                     row_of_slot, slot_of_row, D.T, D.Kp, D.Et, D.d / 8, parts));
  }
  return launch_status();
}

// Scratch of moe_permute_noalloc: the per-slot ranks (kNoAllocMaxSlots int32) followed by the per-block histograms
// (kNoAllocMaxHist int32), 8 MiB in all, resident on every GPU the library runs on until the process ends.
constexpr long long kNoAllocMaxSlots = 1ll << 20;   // T*K' limit
constexpr long long kNoAllocMaxHist = 1ll << 20;    // ceil(T*K'/1024) * E' limit
static __device__ __align__(256) int32_t scratch[kNoAllocMaxSlots + kNoAllocMaxHist];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static int32_t* scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up on first use

// The array's name is only a host-side handle: its device address (one per GPU) comes from the runtime.
static int scratch_on_current_device(int32_t** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_ERR_RUNTIME;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return MOE_ERR_RUNTIME;
    scratch_ptr[dev] = static_cast<int32_t*>(p);
  }
  *out = scratch_ptr[dev];
  return MOE_OK;
}

}  // namespace moe

extern "C" int moe_permute(const moe_shape* shape, const uint16_t* x, const int32_t* topk_idx, uint16_t* x_perm,
                           int32_t* counts, int32_t* offsets, int32_t* row_of_slot, int32_t* slot_of_row,
                           void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  Dims D;
  int rc = permute_checks(shape, &D, x, topk_idx, x_perm, counts, offsets, row_of_slot, slot_of_row);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(ws);
  if (!aligned(ws, 256)) return MOE_ERR_ALIGN;
  const WsLayout L = ws_layout(D);
  if (ws_bytes < L.total) return MOE_ERR_WORKSPACE;
  return permute_launch(D, x, topk_idx, x_perm, counts, offsets, row_of_slot, slot_of_row,
                        reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.perm_hist),
                        reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.perm_rank), (hipStream_t)stream);
}

extern "C" int moe_permute_noalloc(const moe_shape* shape, const uint16_t* x, const int32_t* topk_idx, uint16_t* x_perm,
                                   int32_t* counts, int32_t* offsets, int32_t* row_of_slot, int32_t* slot_of_row,
                                   void* stream) {
  using namespace moe;
  Dims D;
  int rc = permute_checks(shape, &D, x, topk_idx, x_perm, counts, offsets, row_of_slot, slot_of_row);
  if (rc != MOE_OK) return rc;
  if (D.N > kNoAllocMaxSlots || (long long)perm_num_blocks(D.N) * D.Et > kNoAllocMaxHist) return MOE_ERR_WORKSPACE;
  int32_t* base = nullptr;
  rc = scratch_on_current_device(&base);
  if (rc != MOE_OK) return rc;
  return permute_launch(D, x, topk_idx, x_perm, counts, offsets, row_of_slot, slot_of_row, base + kNoAllocMaxSlots, base,
                        (hipStream_t)stream);
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
  hipStream_t st = (hipStream_t)stream;
  MOE_DISPATCH_KP(D.Kp, MOE_LAUNCH("permute_bwd", st, (combine_kernel<KP, true>), dim3(token_blocks(D.T, row_parts(D.d / 8))), dim3(256), 0, st,
                                   reinterpret_cast<const u32x4*>(dx_perm), row_of_slot, (const float*)nullptr,
                                   (const u32x4*)nullptr, reinterpret_cast<u32x4*>(dx), D.T, D.Kp, D.d / 8, row_parts(D.d / 8)));
  return launch_status();
}

extern "C" int moe_permute_bwd_add(const moe_shape* shape, const uint16_t* dx_perm, const int32_t* row_of_slot,
                                   const uint16_t* dx_addend, uint16_t* dx, void* stream) {
  using namespace moe;
  Dims D;
  int rc = check_shape(shape, &D);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(dx_perm); MOE_REQUIRE_PTR(row_of_slot); MOE_REQUIRE_PTR(dx_addend); MOE_REQUIRE_PTR(dx);
  MOE_REQUIRE_ALIGNED(dx_perm); MOE_REQUIRE_ALIGNED(row_of_slot); MOE_REQUIRE_ALIGNED(dx_addend); MOE_REQUIRE_ALIGNED(dx);
  if (D.T == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)stream;
  MOE_DISPATCH_KP(D.Kp, MOE_LAUNCH("permute_bwd_add", st, (combine_kernel<KP, true>), dim3(token_blocks(D.T, row_parts(D.d / 8))), dim3(256), 0, st,
                                   reinterpret_cast<const u32x4*>(dx_perm), row_of_slot, (const float*)nullptr,
                                   reinterpret_cast<const u32x4*>(dx_addend), reinterpret_cast<u32x4*>(dx), D.T, D.Kp, D.d / 8, row_parts(D.d / 8)));
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
  hipStream_t st = (hipStream_t)stream;
  MOE_DISPATCH_KP(D.Kp, MOE_LAUNCH("unpermute_combine", st, (combine_kernel<KP, false>), dim3(token_blocks(D.T, row_parts(D.d / 8))), dim3(256), 0, st,
                                   reinterpret_cast<const u32x4*>(y_perm), row_of_slot, topk_w, (const u32x4*)nullptr,
                                   reinterpret_cast<u32x4*>(out), D.T, D.Kp, D.d / 8, row_parts(D.d / 8)));
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
  hipStream_t st = (hipStream_t)stream;
  const int parts = row_parts(D.d / 8);
  MOE_DISPATCH_KP(D.Kp, MOE_LAUNCH("unpermute_combine_bwd", st, (combine_bwd_kernel<KP>), dim3(token_blocks(D.T, parts)), dim3(256),
                                   4 * (size_t)D.Kp * sizeof(float), st,
                                   reinterpret_cast<const u32x4*>(dout), reinterpret_cast<const u32x4*>(y_perm), row_of_slot,
                                   topk_w, reinterpret_cast<u32x4*>(dy_perm), dtopk_w, D.T, D.Kp, D.d / 8, parts));
  return launch_status();
}
