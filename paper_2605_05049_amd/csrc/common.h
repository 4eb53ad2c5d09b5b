// Shared host/device helpers of the gfx950 MoE library: argument checks, workspace layout, bf16 conversion.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/moe.h"

namespace moe {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kMaxExperts = 1024;    // E' limit of the ABI
constexpr int kPermSlotsPerBlock = 1024;  // slots ranked by one block of the counting sort
constexpr int kSplitParts = 256;     // K-split parts in flight at most: 32 per XCD (one per CU)
constexpr int kSplitCounters = 128;  // split tiles at most: 16 per XCD
constexpr int kMaxWidth = 1 << 22;   // d_model, d_ffn limit: 256 rows x 2^22 elements x 2 bytes < 2^32
constexpr int kMinTileRows = 32;     // smallest row-tile height any GEMM schedule may use

struct Dims {
  int T, d, f, E, k, Es, Et, Kp, renorm;
  long long N;
};

// Validates a shape against the ABI limits and fills the derived sizes.
inline int check_shape(const moe_shape* s, Dims* out) {
  if (!s) return MOE_ERR_NULL;
  if (s->T < 0 || s->E < 1 || s->k < 1 || s->k > s->E || s->E_shared < 0) return MOE_ERR_SHAPE;
  if (s->E > kMaxExperts || (long long)s->E + s->E_shared > kMaxExperts) return MOE_ERR_SHAPE;
  if (s->d_model <= 0 || s->d_ffn <= 0 || (s->d_model % 64) || (s->d_ffn % 64)) return MOE_ERR_SHAPE;
  if (s->d_model > kMaxWidth || s->d_ffn > kMaxWidth) return MOE_ERR_SHAPE;  // 32-bit per-lane byte offsets in the GEMM loads
  long long Kp = (long long)s->k + s->E_shared;
  long long N = (long long)s->T * Kp;
  if (N >= (1ll << 31)) return MOE_ERR_SHAPE;
  out->T = s->T; out->d = s->d_model; out->f = s->d_ffn; out->E = s->E; out->k = s->k; out->Es = s->E_shared;
  out->Et = s->E + s->E_shared; out->Kp = (int)Kp; out->N = N; out->renorm = s->renorm ? 1 : 0;
  return MOE_OK;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Workspace carve-up.  Every region starts 256-byte aligned.
//   perm_hist : per-block expert histograms of the counting sort, then turned into per-block bases
//   perm_rank : rank of every slot among the same-expert slots of its block
//   sched     : tile schedule of the grouped GEMMs (header + two int arrays)
//   zero_page : 256 zero bytes, the source of k-rows past the end of a ragged contraction
//   h, dg, du : bf16 [N,f] intermediates of the expert FFN (H in forward; H, dG, dU in backward): with x_perm these are
//               the 3 d_ffn + d_model values per row of the activation-memory model of Section III-A
struct WsLayout {
  size_t perm_hist, perm_hist_bytes;
  size_t perm_rank, perm_rank_bytes;
  size_t sched, sched_bytes;
  size_t zero_page;
  size_t splitk_counters;   // kSplitCounters int32: arrivals per split tile
  size_t splitk_partial;    // kSplitParts fp32 tiles of up to 320 x 256: partial sums of the tiles whose K range is split
  size_t h, dg, du, nf_bytes;
  size_t g_re, u_re;        // G, U when the caller does not keep them (checkpointed forward, recomputing backward): = dg, du
  size_t router_offsets;    // 64 int32: {0, T}, {0, E} (one-segment "offsets" of the router's GEMMs) and the bounds of the parts of T
  size_t dl_hi, dl_lo;      // [T, Epad] bf16: head and remainder of the fp32 dlogits (Epad = E rounded up to 64)
  size_t w_router_t;        // [d, 128] bf16 at most: W_r transposed and zero-padded (router backward, E <= 128)
  size_t router_dw_partial; // router_dw_parts() fp32 partial results [d, ldp] of dW_r^T
  size_t total;
};

inline int perm_num_blocks(long long N) { return (int)((N + kPermSlotsPerBlock - 1) / kPermSlotsPerBlock); }
inline long long sched_max_tiles(const Dims& D) { return D.N / kMinTileRows + D.Et; }

// The router's dW_r contraction over the T tokens is cut into S parts whose fp32 results [d, ldp] (ldp = E rounded up to
// 4) are added afterwards: as many parts as give every CU a 256 x 128 tile, at most 32, at least 64 tokens each, and no
// more than fit 128 MB (always at least one).
inline size_t router_dw_part_bytes(const Dims& D) { return (size_t)D.d * round_up((size_t)D.E, 4) * sizeof(float); }
inline int router_dw_parts(const Dims& D) {
  const long long tiles = (long long)((D.d + 255) / 256) * ((D.E + 127) / 128);
  long long S = (256 + tiles - 1) / tiles;
  S = S < 32 ? S : 32;
  const long long by_tokens = (D.T + 63) / 64, by_bytes = (long long)(((size_t)128 << 20) / router_dw_part_bytes(D));
  S = S < by_tokens ? S : by_tokens;
  S = S < by_bytes ? S : by_bytes;
  return (int)(S < 1 ? 1 : S);
}

inline WsLayout ws_layout(const Dims& D) {
  WsLayout L;
  size_t off = 0;
  L.perm_hist = off;
  L.perm_hist_bytes = round_up((size_t)perm_num_blocks(D.N) * D.Et * sizeof(int32_t) + 256, 256);
  off += L.perm_hist_bytes;
  L.perm_rank = off;
  L.perm_rank_bytes = round_up((size_t)D.N * sizeof(int32_t) + 256, 256);
  off += L.perm_rank_bytes;
  L.sched = off;
  L.sched_bytes = round_up((size_t)(64 + 2 * sched_max_tiles(D) + kMaxExperts) * sizeof(int32_t), 256);
  off += L.sched_bytes;
  L.zero_page = off;
  off += 256;
  L.splitk_counters = off;
  off += round_up((size_t)kSplitCounters * sizeof(int32_t), 256);
  L.splitk_partial = off;
  off += (size_t)kSplitParts * 320 * 256 * sizeof(float);
  L.nf_bytes = round_up((size_t)D.N * D.f * sizeof(uint16_t), 256);
  L.h = off; off += L.nf_bytes;
  L.dg = off; off += L.nf_bytes;
  L.du = off; off += L.nf_bytes;
  // G, U that the caller does not keep share the memory of dG, dU: the kernel that consumes them (dH with the
  // d(SwiGLU) epilogue) reads G, U and writes dG, dU at the same element from the same lane, i.e. in place
  L.g_re = L.dg;
  L.u_re = L.du;
  L.router_offsets = off; off += 256;
  const size_t dl_bytes = round_up((size_t)D.T * round_up((size_t)D.E, 64) * sizeof(uint16_t) + 256, 256);
  L.dl_hi = off; off += dl_bytes;
  L.dl_lo = off; off += dl_bytes;
  L.w_router_t = off; off += D.E <= 128 ? round_up((size_t)D.d * 128 * sizeof(uint16_t), 256) : 0;
  L.router_dw_partial = off; off += round_up((size_t)router_dw_parts(D) * router_dw_part_bytes(D), 256);
  L.total = off;
  return L;
}

#define MOE_REQUIRE_PTR(p) do { if ((p) == nullptr) return MOE_ERR_NULL; } while (0)
#define MOE_REQUIRE_ALIGNED(p) do { if (!::moe::aligned((p), 16)) return MOE_ERR_ALIGN; } while (0)

inline int launch_status() { return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_RUNTIME; }

// Router backward pieces that live beside the router's forward kernel (router.hip) and are launched from the entry
// point that also launches the grouped GEMM kernel (grouped_gemm.hip).
void launch_router_prepare(hipStream_t st, const float* dlogits, const uint16_t* w_router, uint16_t* hi, uint16_t* lo, uint16_t* w_t,
                           int32_t* offsets2, int32_t* part_order, int32_t* tile_queue, uint32_t* zero_page, int T, int E, int Epad, int Ek,
                           int d, int S, int part_rows);
void launch_router_bwd_dx(hipStream_t st, const uint16_t* dl_hi, const uint16_t* dl_lo, const uint16_t* w_t, uint16_t* dx, int T, int d,
                          int E, int Epad);
void launch_router_dw_reduce(hipStream_t st, const float* partial, float* dw, int S, int E, int d, int ldp, int accumulate);

// Optional per-launch timing (moe_profile_* in the ABI).  While enabled, every kernel launch of the library is
// bracketed by two HIP events on the launch stream; disabled (the default) it costs one branch.
void prof_begin(const char* name, hipStream_t st);
void prof_end(hipStream_t st);
struct ProfScope {
  hipStream_t st;
  ProfScope(const char* name, hipStream_t s) : st(s) { prof_begin(name, s); }
  ~ProfScope() { prof_end(st); }
};
// hipLaunchKernelGGL with a label for the optional per-launch timing.
#define MOE_LAUNCH(label, st, ...)            \
  do {                                        \
    ::moe::ProfScope moe_prof_scope_(label, st); \
    hipLaunchKernelGGL(__VA_ARGS__);          \
  } while (0)

// ---------------------------------------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------------------------------------

// bf16 <-> fp32 on raw bit patterns.  fp32 -> bf16 is the hardware conversion (v_cvt_pk_bf16_f32: two values per
// instruction, round-to-nearest-even, NaN stays NaN).
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ float bf16lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16_pair __attribute__((ext_vector_type(2)));
  typedef float f32_pair __attribute__((ext_vector_type(2)));
  const f32_pair v = {lo, hi};
  const bf16_pair b = __builtin_convertvector(v, bf16_pair);
  return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float v) { return (uint16_t)(pack_bf16(v, 0.f) & 0xffffu); }

typedef __attribute__((address_space(3))) void* lptr_t;

// One direct global->LDS load: 16 bytes per lane, lane L lands at lds_base + 16 L (lds_base is wave-uniform).
// Written as inline assembly on purpose: the compiler does not track it, so it never makes the (transposing)
// fragment reads of the OTHER stage wait for loads still in flight.  A kernel that uses them orders them itself: an
// explicit s_waitcnt vmcnt(0) precedes the barrier that publishes a stage, and no compiler-tracked vector-memory
// load is in flight while these are (the epilogue starts after the last such wait).  m0 receives the LDS base: the
// backend reserves m0 (it is never allocated, and the compiler writes it only directly before an instruction of its
// own that reads it; the kernels here have none: no LDS-direct or GDS access, no register-indexed moves, no messages).  Two
// address forms: a 64-bit address per lane, or a scalar base plus a 32-bit byte offset per lane.
__device__ __forceinline__ void direct_load16(const void* g, const char* lds_dst) {
  const unsigned lds = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lptr_t)lds_dst);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds), "v"(g) : "memory");
}
__device__ __forceinline__ void direct_load16(const void* sbase, unsigned voff, const char* lds_dst) {
  const unsigned lds = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lptr_t)lds_dst);
  const unsigned long long b = (unsigned long long)sbase;  // wave-uniform by construction; tell the compiler so
  const unsigned long long sb = ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
                                (unsigned)__builtin_amdgcn_readfirstlane((int)b);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds), "v"(voff), "s"(sb) : "memory");
}

}  // namespace moe
