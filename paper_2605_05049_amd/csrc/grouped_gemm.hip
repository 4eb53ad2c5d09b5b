// Grouped bf16 MFMA GEMMs of the SwiGLU expert FFNs over ragged per-expert row segments, forward and backward
// (Section III-A: W_up, W_gate in R^{d x f}, W_down in R^{f x d}, per-expert token counts s_e; the "imbalanced
// tall-and-skinny GEMMs" of the abstract and Section II-A).
//
// One kernel template serves all seven contractions.  Every output tile is
//     C[p, q] = sum_k  P[p, k] * Q[q, k]          (p: 128 values, q: 128 values, k in steps of 64)
// where P is the operand whose index becomes the lane-column of the MFMA accumulator and Q the operand whose
// index becomes the accumulator register (so that each lane owns 4 consecutive q = 4 consecutive output
// elements of a row-major C).  An operand is "K-contiguous" (KC: element (r,k) at base[r*ld + k]) or
// "R-contiguous" (RC: element (r,k) at base[k*ld + r]).  KC tiles are read from LDS with 16-byte loads, RC tiles
// with the gfx950 transposing LDS read (ds_read_b64_tr_b16), so no operand is ever transposed in HBM.
//
//   forward   G,U = X Wg, X Wu     P = X (KC)        Q = Wg, Wu (RC)   two accumulators, SwiGLU epilogue
//             Y   = H Wd           P = H (KC)        Q = Wd (RC)
//   backward  dH  = dY Wd^T        P = dY (KC)       Q = Wd (KC)       d(SwiGLU) epilogue -> dG, dU, H
//             dX  = dG Wg^T+dU Wu^T P = dG then dU (KC) Q = Wg then Wu (KC)  one accumulator, two K passes
//             dWd = H^T dY         P = H (RC)        Q = dY (RC)       ragged K = rows of the expert, fp32 out
//             dWg,dWu = X^T dG, X^T dU   P = X (RC)  Q = dG, dU (RC)   two accumulators, ragged K, fp32 out
//
// Tiling: 256 threads = 4 wavefronts in a 2x2 grid, each owning 64x64 of the 128x128 tile as 2x2 MFMA
// 32x32x16 blocks (fp32 accumulators).  Global loads for step k+1 are issued into registers before the MFMAs of
// step k, then stored to the single LDS stage; two blocks per CU overlap each other's load and math phases.
// Row tiles of the ragged dimension come from a device-built schedule (no host sync on the counts); the
// block-id -> tile map hands each XCD a contiguous run of tiles so that tiles sharing a weight panel meet in
// one L2.
#include "common.h"

namespace moe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;          // k step
constexpr int TP = 128;         // p extent of a tile
constexpr int TQ = 128;         // q extent of a tile
constexpr int KC_LD = BK + 8;   // LDS row pitch of a K-contiguous tile [128][72]: 16-byte reads hit distinct banks
constexpr int RC_LD = 128 + 32; // LDS row pitch of an R-contiguous tile [64][160]: 4 k-rows of a transposing read
                                // land in 4 disjoint bank groups
constexpr int KC_TILE = 128 * KC_LD;  // elements
constexpr int RC_TILE = BK * RC_LD;   // elements
constexpr int kNumXcd = 8;

enum Epilogue { EPI_BF16 = 0, EPI_SWIGLU = 1, EPI_DSWIGLU = 2, EPI_F32 = 3 };

// One operand of one tile.
struct Operand {
  const uint16_t* base;  // element (r=0, k=0) of the tile
  size_t ld;             // elements between consecutive r (KC) or consecutive k (RC)
  int r_valid;           // r in [0, r_valid) exists (1..128); loads beyond are clamped and never stored
};

template <bool RC>
__device__ __forceinline__ void load_tile_regs(u32x4 (&reg)[4], const Operand& op, int k0, int k_end, int tid) {
  if (!RC) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int v = tid + 256 * i;
      int r = v >> 3;
      const int kc = v & 7;
      r = r < op.r_valid ? r : op.r_valid - 1;
      reg[i] = *reinterpret_cast<const u32x4*>(op.base + (size_t)r * op.ld + k0 + kc * 8);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int v = tid + 256 * i;
      const int kr = v >> 4;
      int c = (v & 15) * 8;
      c = c < op.r_valid ? c : op.r_valid - 8;
      const int k = k0 + kr;
      u32x4 z = {0u, 0u, 0u, 0u};
      reg[i] = (k < k_end) ? *reinterpret_cast<const u32x4*>(op.base + (size_t)k * op.ld + c) : z;
    }
  }
}

template <bool RC>
__device__ __forceinline__ void store_tile_lds(const u32x4 (&reg)[4], uint16_t* tile, int tid) {
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int v = tid + 256 * i;
    if (!RC) *reinterpret_cast<u32x4*>(tile + (v >> 3) * KC_LD + (v & 7) * 8) = reg[i];
    else *reinterpret_cast<u32x4*>(tile + (v >> 4) * RC_LD + (v & 15) * 8) = reg[i];
  }
}

// MFMA operand fragment: 32 r-values x 16 k-values; lane l gets r = r0 + l%32, k = kk + 8*(l/32) .. +7.
template <bool RC>
__device__ __forceinline__ bf16x8 read_frag(const uint16_t* tile, int r0, int kk, int lane) {
  if (!RC) {
    return *reinterpret_cast<const bf16x8*>(tile + (r0 + (lane & 31)) * KC_LD + kk + 8 * (lane >> 5));
  } else {
    // Transposing read: inside each group of 16 lanes, lane p supplies the address of 4 consecutive r at k-row
    // p/4, r-chunk p%4, and receives the 4 k-rows of r = (group base) + p.
    const int p = lane & 15;
    const uint16_t* a = tile + (kk + 8 * (lane >> 5) + (p >> 2)) * RC_LD + r0 + 16 * ((lane >> 4) & 1) + 4 * (p & 3);
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(a));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(a + 4 * RC_LD));
    union { struct { s16x4 lo, hi; } s; bf16x8 v; } u;
    u.s.lo = lo;
    u.s.hi = hi;
    return u.v;
  }
}

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

struct GemmArgs {
  // row-tile problems (forward / dgrad): schedule built on the device
  const int32_t* sched;    // [0] = number of row tiles; then tile_expert[max_tiles], tile_row0[max_tiles]
  int max_tiles;
  const int32_t* offsets;  // [E'+1]
  int n_q_tiles;           // tiles along q
  int q_dim;               // extent of q (output columns)
  int k_dim;               // contraction length per pass (row-tile problems); unused for wgrad
  // operands: p side (activations) and up to two q sides (weights), and a second pass for the dX contraction
  const uint16_t* p0; size_t p_ld;
  const uint16_t* p1;
  const uint16_t* q0; const uint16_t* q1; size_t q_ld; size_t q_expert_stride;
  // wgrad only
  int p_dim;               // extent of p (rows of dW)
  int n_p_tiles;
  int Et;
  int accumulate;
  // outputs
  uint16_t* c0; uint16_t* c1; uint16_t* c2; size_t c_ld;   // bf16 outputs (row-major, ld = q_dim)
  const uint16_t* g_in; const uint16_t* u_in;              // saved G, U for the d(SwiGLU) epilogue
  float* f0; float* f1; size_t f_expert_stride;            // fp32 outputs of the wgrads
};

// KIND 0: row-tile problem (p = ragged rows of an expert, k = k_dim);  KIND 1: wgrad (k = ragged rows).
template <int KIND, bool P_RC, bool Q_RC, int NQ, int NPASS, int EPI>
__global__ __launch_bounds__(256, 2) void grouped_gemm_kernel(const GemmArgs A) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int P_TILE = P_RC ? RC_TILE : KC_TILE;
  constexpr int Q_TILE = Q_RC ? RC_TILE : KC_TILE;
  uint16_t* p_lds = smem;
  uint16_t* q_lds = smem + P_TILE;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wp = (wave & 1) * 64;
  const int wq = (wave >> 1) * 64;

  // ---- block id -> tile (each XCD takes a contiguous run of the logical tile order) ----
  int expert, p_row0 = 0, p_valid, q0_col, k_len;
  size_t krow0 = 0;
  if (KIND == 0) {
    const int n_row_tiles = A.sched[0];
    const long long total = (long long)n_row_tiles * A.n_q_tiles;
    const long long chunk = (total + kNumXcd - 1) / kNumXcd;
    const long long within = blockIdx.x / kNumXcd;
    const long long lid = (long long)(blockIdx.x % kNumXcd) * chunk + within;
    if (within >= chunk || lid >= total) return;
    const int u = (int)(lid / A.n_q_tiles);  // some row tile of the expert this block works for
    expert = A.sched[64 + u];
    const int e_lo = A.offsets[expert], e_hi = A.offsets[expert + 1];
    const int e_tiles = (e_hi - e_lo + TP - 1) / TP;
    const int first = A.sched[64 + A.max_tiles + u];  // index of the expert's first row tile
    const long long local = lid - (long long)first * A.n_q_tiles;
    const int qt = (int)(local / e_tiles);
    const int mt = (int)(local % e_tiles);
    p_row0 = e_lo + mt * TP;
    p_valid = min(TP, e_hi - p_row0);
    q0_col = qt * TQ;
    k_len = A.k_dim;
  } else {
    const long long per_e = (long long)A.n_p_tiles * A.n_q_tiles;
    const long long total = per_e * A.Et;
    const long long chunk = (total + kNumXcd - 1) / kNumXcd;
    const long long within = blockIdx.x / kNumXcd;
    const long long lid = (long long)(blockIdx.x % kNumXcd) * chunk + within;
    if (within >= chunk || lid >= total) return;
    expert = (int)(lid / per_e);
    const int local = (int)(lid % per_e);
    const int qt = local / A.n_p_tiles;
    const int pt = local % A.n_p_tiles;
    const int e_lo = A.offsets[expert], e_hi = A.offsets[expert + 1];
    k_len = e_hi - e_lo;
    krow0 = (size_t)e_lo;
    p_row0 = pt * TP;
    p_valid = min(TP, A.p_dim - p_row0);
    q0_col = qt * TQ;
    if (k_len == 0 && A.accumulate) return;  // nothing to add
  }
  const int q_valid = min(TQ, A.q_dim - q0_col);

  f32x16 acc[NQ][2][2];
#pragma unroll
  for (int n = 0; n < NQ; n++)
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
      for (int b = 0; b < 2; b++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc[n][a][b][v] = 0.f;

#pragma unroll
  for (int pass = 0; pass < NPASS; pass++) {
    Operand P, Q[NQ];
    if (KIND == 0) {
      const uint16_t* pb = (pass == 0) ? A.p0 : A.p1;
      P.base = pb + (size_t)p_row0 * A.p_ld;
      P.ld = A.p_ld;
      P.r_valid = p_valid;
#pragma unroll
      for (int n = 0; n < NQ; n++) {
        // one accumulator, two passes: pass selects the weight; two accumulators: n selects it
        const uint16_t* qb = ((NPASS == 2 ? pass : n) == 0) ? A.q0 : A.q1;
        qb += (size_t)expert * A.q_expert_stride;
        Q[n].base = Q_RC ? qb + q0_col : qb + (size_t)q0_col * A.q_ld;
        Q[n].ld = A.q_ld;
        Q[n].r_valid = q_valid;
      }
    } else {
      P.base = A.p0 + krow0 * A.p_ld + p_row0;
      P.ld = A.p_ld;
      P.r_valid = p_valid;
#pragma unroll
      for (int n = 0; n < NQ; n++) {
        const uint16_t* qb = (n == 0) ? A.q0 : A.q1;
        Q[n].base = qb + krow0 * A.q_ld + q0_col;
        Q[n].ld = A.q_ld;
        Q[n].r_valid = q_valid;
      }
    }

    const int nk = (k_len + BK - 1) / BK;
    u32x4 preg[4], qreg[NQ][4];
    if (nk > 0) {
      load_tile_regs<P_RC>(preg, P, 0, k_len, tid);
#pragma unroll
      for (int n = 0; n < NQ; n++) load_tile_regs<Q_RC>(qreg[n], Q[n], 0, k_len, tid);
    }
    for (int kt = 0; kt < nk; kt++) {
      __syncthreads();  // everyone has finished reading the previous stage
      store_tile_lds<P_RC>(preg, p_lds, tid);
#pragma unroll
      for (int n = 0; n < NQ; n++) store_tile_lds<Q_RC>(qreg[n], q_lds + n * Q_TILE, tid);
      __syncthreads();
      if (kt + 1 < nk) {
        load_tile_regs<P_RC>(preg, P, (kt + 1) * BK, k_len, tid);
#pragma unroll
        for (int n = 0; n < NQ; n++) load_tile_regs<Q_RC>(qreg[n], Q[n], (kt + 1) * BK, k_len, tid);
      }
#pragma unroll
      for (int kk = 0; kk < BK; kk += 16) {
        bf16x8 pf[2], qf[NQ][2];
#pragma unroll
        for (int b = 0; b < 2; b++) pf[b] = read_frag<P_RC>(p_lds, wp + 32 * b, kk, lane);
#pragma unroll
        for (int n = 0; n < NQ; n++)
#pragma unroll
          for (int a = 0; a < 2; a++) qf[n][a] = read_frag<Q_RC>(q_lds + n * Q_TILE, wq + 32 * a, kk, lane);
#pragma unroll
        for (int n = 0; n < NQ; n++)
#pragma unroll
          for (int a = 0; a < 2; a++)
#pragma unroll
            for (int b = 0; b < 2; b++)
              acc[n][a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[n][a], pf[b], acc[n][a][b], 0, 0, 0);
      }
    }
  }

  // ---- epilogue.  acc[n][a][b][v]: q = wq + 32a + 8(v/4) + 4(lane/32) + v%4,  p = wp + 32b + lane%32 ----
#pragma unroll
  for (int a = 0; a < 2; a++)
#pragma unroll
    for (int b = 0; b < 2; b++) {
      const int p = wp + 32 * b + (lane & 31);
      if (p >= p_valid) continue;
#pragma unroll
      for (int v4 = 0; v4 < 4; v4++) {
        const int q = wq + 32 * a + 8 * v4 + 4 * (lane >> 5);
        if (q >= q_valid) continue;
        if (EPI == EPI_F32) {
          const size_t o = (size_t)expert * A.f_expert_stride + (size_t)(p_row0 + p) * A.c_ld + q0_col + q;
#pragma unroll
          for (int n = 0; n < NQ; n++) {
            float* dst = (n == 0 ? A.f0 : A.f1) + o;
            float4 r = make_float4(acc[n][a][b][4 * v4], acc[n][a][b][4 * v4 + 1], acc[n][a][b][4 * v4 + 2],
                                   acc[n][a][b][4 * v4 + 3]);
            if (A.accumulate) {
              const float4 old = *reinterpret_cast<const float4*>(dst);
              r.x += old.x; r.y += old.y; r.z += old.z; r.w += old.w;
            }
            *reinterpret_cast<float4*>(dst) = r;
          }
        } else {
          const size_t o = (size_t)(p_row0 + p) * A.c_ld + q0_col + q;
          if (EPI == EPI_BF16) {
            uint2 r;
            r.x = pack_bf16(acc[0][a][b][4 * v4], acc[0][a][b][4 * v4 + 1]);
            r.y = pack_bf16(acc[0][a][b][4 * v4 + 2], acc[0][a][b][4 * v4 + 3]);
            *reinterpret_cast<uint2*>(A.c0 + o) = r;
          } else if (EPI == EPI_SWIGLU) {
            float g[4], u[4], h[4];
#pragma unroll
            for (int i = 0; i < 4; i++) {
              g[i] = acc[0][a][b][4 * v4 + i];
              u[i] = acc[NQ - 1][a][b][4 * v4 + i];
              h[i] = silu_f(g[i]) * u[i];
            }
            *reinterpret_cast<uint2*>(A.c0 + o) = make_uint2(pack_bf16(g[0], g[1]), pack_bf16(g[2], g[3]));
            *reinterpret_cast<uint2*>(A.c1 + o) = make_uint2(pack_bf16(u[0], u[1]), pack_bf16(u[2], u[3]));
            *reinterpret_cast<uint2*>(A.c2 + o) = make_uint2(pack_bf16(h[0], h[1]), pack_bf16(h[2], h[3]));
          } else {  // EPI_DSWIGLU: acc = dH; read saved G, U; write dG, dU, H
            const uint2 gi = *reinterpret_cast<const uint2*>(A.g_in + o);
            const uint2 ui = *reinterpret_cast<const uint2*>(A.u_in + o);
            const float g[4] = {bf16lo(gi.x), bf16hi(gi.x), bf16lo(gi.y), bf16hi(gi.y)};
            const float u[4] = {bf16lo(ui.x), bf16hi(ui.x), bf16lo(ui.y), bf16hi(ui.y)};
            float dg[4], du[4], h[4];
#pragma unroll
            for (int i = 0; i < 4; i++) {
              const float dh = acc[0][a][b][4 * v4 + i];
              const float s = 1.0f / (1.0f + __expf(-g[i]));
              const float sl = g[i] * s;
              h[i] = sl * u[i];
              du[i] = dh * sl;
              dg[i] = dh * u[i] * (s * (1.0f + g[i] * (1.0f - s)));
            }
            *reinterpret_cast<uint2*>(A.c0 + o) = make_uint2(pack_bf16(dg[0], dg[1]), pack_bf16(dg[2], dg[3]));
            *reinterpret_cast<uint2*>(A.c1 + o) = make_uint2(pack_bf16(du[0], du[1]), pack_bf16(du[2], du[3]));
            *reinterpret_cast<uint2*>(A.c2 + o) = make_uint2(pack_bf16(h[0], h[1]), pack_bf16(h[2], h[3]));
          }
        }
      }
    }
}

// Row-tile schedule: one thread per expert.  sched[0] = number of 128-row tiles; sched[64 + u] = expert of tile u;
// sched[64 + max_tiles + u] = index of that expert's first tile.
__global__ __launch_bounds__(1024) void build_schedule_kernel(const int32_t* __restrict__ offsets, int32_t* __restrict__ sched,
                                                              int Et, int max_tiles) {
  __shared__ int32_t scan[kMaxExperts];
  const int e = threadIdx.x;
  const int n = (e < Et) ? offsets[e + 1] - offsets[e] : 0;
  const int nt = (n + TP - 1) / TP;
  scan[e] = nt;
  __syncthreads();
  for (int o = 1; o < kMaxExperts; o <<= 1) {
    int v = (e >= o) ? scan[e - o] : 0;
    __syncthreads();
    scan[e] += v;
    __syncthreads();
  }
  const int first = scan[e] - nt;
  if (e == kMaxExperts - 1) sched[0] = scan[e];
  for (int i = 0; i < nt; i++) {
    if (first + i < max_tiles) {
      sched[64 + first + i] = e;
      sched[64 + max_tiles + first + i] = first;
    }
  }
}

template <int KIND, bool P_RC, bool Q_RC, int NQ, int NPASS, int EPI>
static void launch_gemm(const char* label, const GemmArgs& A, long long max_blocks, hipStream_t st) {
  constexpr size_t lds = ((P_RC ? RC_TILE : KC_TILE) + NQ * (Q_RC ? RC_TILE : KC_TILE)) * sizeof(uint16_t);
  const long long grid = (max_blocks + kNumXcd - 1) / kNumXcd * kNumXcd;
  if (grid <= 0) return;
  MOE_LAUNCH(label, st, (grouped_gemm_kernel<KIND, P_RC, Q_RC, NQ, NPASS, EPI>), dim3((unsigned)grid), dim3(256), lds, st, A);
}

static int common_checks(const moe_shape* shape, Dims* D, void* ws, size_t ws_bytes, WsLayout* L) {
  int rc = check_shape(shape, D);
  if (rc != MOE_OK) return rc;
  if (!ws) return MOE_ERR_NULL;
  if (!aligned(ws, 256)) return MOE_ERR_ALIGN;
  *L = ws_layout(*D);
  if (ws_bytes < L->total) return MOE_ERR_WORKSPACE;
  return MOE_OK;
}

}  // namespace moe

extern "C" int moe_grouped_ffn_fwd(const moe_shape* shape, const uint16_t* x_perm, const int32_t* offsets,
                                   const uint16_t* w_gate, const uint16_t* w_up, const uint16_t* w_down,
                                   uint16_t* y_perm, uint16_t* save_g, uint16_t* save_u,
                                   void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  Dims D;
  WsLayout L;
  int rc = common_checks(shape, &D, ws, ws_bytes, &L);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(x_perm); MOE_REQUIRE_PTR(offsets); MOE_REQUIRE_PTR(w_gate); MOE_REQUIRE_PTR(w_up); MOE_REQUIRE_PTR(w_down);
  MOE_REQUIRE_PTR(y_perm); MOE_REQUIRE_PTR(save_g); MOE_REQUIRE_PTR(save_u);
  MOE_REQUIRE_ALIGNED(x_perm); MOE_REQUIRE_ALIGNED(offsets); MOE_REQUIRE_ALIGNED(w_gate); MOE_REQUIRE_ALIGNED(w_up);
  MOE_REQUIRE_ALIGNED(w_down); MOE_REQUIRE_ALIGNED(y_perm); MOE_REQUIRE_ALIGNED(save_g); MOE_REQUIRE_ALIGNED(save_u);
  if (D.N == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)stream;
  char* wsb = static_cast<char*>(ws);
  int32_t* sched = reinterpret_cast<int32_t*>(wsb + L.sched);
  uint16_t* h = reinterpret_cast<uint16_t*>(wsb + L.h);
  const int max_tiles = (int)sched_max_tiles(D);
  const long long ub_tiles = D.N / TP + D.Et;  // sum_e ceil(n_e/128) <= N/128 + E'
  MOE_LAUNCH("ffn_schedule", st, build_schedule_kernel, dim3(1), dim3(1024), 0, st, offsets, sched, D.Et, max_tiles);

  GemmArgs A = {};
  A.sched = sched; A.max_tiles = max_tiles; A.offsets = offsets; A.Et = D.Et;
  // G, U = X Wg, X Wu ; H = silu(G) * U
  A.n_q_tiles = (D.f + TQ - 1) / TQ; A.q_dim = D.f; A.k_dim = D.d;
  A.p0 = x_perm; A.p_ld = D.d;
  A.q0 = w_gate; A.q1 = w_up; A.q_ld = D.f; A.q_expert_stride = (size_t)D.d * D.f;
  A.c0 = save_g; A.c1 = save_u; A.c2 = h; A.c_ld = D.f;
  launch_gemm<0, false, true, 2, 1, EPI_SWIGLU>("ffn_fwd_gate_up_swiglu", A, ub_tiles * A.n_q_tiles, st);
  // Y = H Wd
  A.n_q_tiles = (D.d + TQ - 1) / TQ; A.q_dim = D.d; A.k_dim = D.f;
  A.p0 = h; A.p_ld = D.f;
  A.q0 = w_down; A.q1 = nullptr; A.q_ld = D.d; A.q_expert_stride = (size_t)D.f * D.d;
  A.c0 = y_perm; A.c1 = nullptr; A.c2 = nullptr; A.c_ld = D.d;
  launch_gemm<0, false, true, 1, 1, EPI_BF16>("ffn_fwd_down", A, ub_tiles * A.n_q_tiles, st);
  return launch_status();
}

extern "C" int moe_grouped_ffn_bwd(const moe_shape* shape, const uint16_t* dy_perm, const uint16_t* x_perm,
                                   const int32_t* offsets, const uint16_t* w_gate, const uint16_t* w_up,
                                   const uint16_t* w_down, const uint16_t* save_g, const uint16_t* save_u,
                                   uint16_t* dx_perm, float* dw_gate, float* dw_up, float* dw_down, int accumulate,
                                   void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  Dims D;
  WsLayout L;
  int rc = common_checks(shape, &D, ws, ws_bytes, &L);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(dy_perm); MOE_REQUIRE_PTR(x_perm); MOE_REQUIRE_PTR(offsets); MOE_REQUIRE_PTR(w_gate); MOE_REQUIRE_PTR(w_up);
  MOE_REQUIRE_PTR(w_down); MOE_REQUIRE_PTR(save_g); MOE_REQUIRE_PTR(save_u); MOE_REQUIRE_PTR(dx_perm);
  MOE_REQUIRE_PTR(dw_gate); MOE_REQUIRE_PTR(dw_up); MOE_REQUIRE_PTR(dw_down);
  MOE_REQUIRE_ALIGNED(dy_perm); MOE_REQUIRE_ALIGNED(x_perm); MOE_REQUIRE_ALIGNED(offsets); MOE_REQUIRE_ALIGNED(w_gate);
  MOE_REQUIRE_ALIGNED(w_up); MOE_REQUIRE_ALIGNED(w_down); MOE_REQUIRE_ALIGNED(save_g); MOE_REQUIRE_ALIGNED(save_u);
  MOE_REQUIRE_ALIGNED(dx_perm); MOE_REQUIRE_ALIGNED(dw_gate); MOE_REQUIRE_ALIGNED(dw_up); MOE_REQUIRE_ALIGNED(dw_down);
  hipStream_t st = (hipStream_t)stream;
  char* wsb = static_cast<char*>(ws);
  int32_t* sched = reinterpret_cast<int32_t*>(wsb + L.sched);
  uint16_t* h = reinterpret_cast<uint16_t*>(wsb + L.h);
  uint16_t* dg = reinterpret_cast<uint16_t*>(wsb + L.dg);
  uint16_t* du = reinterpret_cast<uint16_t*>(wsb + L.du);
  const int max_tiles = (int)sched_max_tiles(D);
  const long long ub_tiles = D.N / TP + D.Et;

  GemmArgs A = {};
  A.sched = sched; A.max_tiles = max_tiles; A.offsets = offsets; A.Et = D.Et; A.accumulate = accumulate ? 1 : 0;
  if (D.N > 0) {
    MOE_LAUNCH("ffn_schedule", st, build_schedule_kernel, dim3(1), dim3(1024), 0, st, offsets, sched, D.Et, max_tiles);
    // dH = dY Wd^T, then dG, dU and H from the saved G, U
    A.n_q_tiles = (D.f + TQ - 1) / TQ; A.q_dim = D.f; A.k_dim = D.d;
    A.p0 = dy_perm; A.p_ld = D.d;
    A.q0 = w_down; A.q_ld = D.d; A.q_expert_stride = (size_t)D.f * D.d;
    A.c0 = dg; A.c1 = du; A.c2 = h; A.c_ld = D.f; A.g_in = save_g; A.u_in = save_u;
    launch_gemm<0, false, false, 1, 1, EPI_DSWIGLU>("ffn_bwd_dh_dswiglu", A, ub_tiles * A.n_q_tiles, st);
    // dX = dG Wg^T + dU Wu^T
    A.n_q_tiles = (D.d + TQ - 1) / TQ; A.q_dim = D.d; A.k_dim = D.f;
    A.p0 = dg; A.p1 = du; A.p_ld = D.f;
    A.q0 = w_gate; A.q1 = w_up; A.q_ld = D.f; A.q_expert_stride = (size_t)D.d * D.f;
    A.c0 = dx_perm; A.c1 = nullptr; A.c2 = nullptr; A.c_ld = D.d;
    launch_gemm<0, false, false, 1, 2, EPI_BF16>("ffn_bwd_dx", A, ub_tiles * A.n_q_tiles, st);
  }
  // dWd[e] = H_e^T dY_e   (rows f, columns d)
  A.p_dim = D.f; A.n_p_tiles = (D.f + TP - 1) / TP; A.q_dim = D.d; A.n_q_tiles = (D.d + TQ - 1) / TQ;
  A.p0 = h; A.p1 = nullptr; A.p_ld = D.f;
  A.q0 = dy_perm; A.q1 = nullptr; A.q_ld = D.d;
  A.f0 = dw_down; A.f1 = nullptr; A.f_expert_stride = (size_t)D.f * D.d; A.c_ld = D.d;
  launch_gemm<1, true, true, 1, 1, EPI_F32>("ffn_bwd_dw_down", A, (long long)D.Et * A.n_p_tiles * A.n_q_tiles, st);
  // dWg[e], dWu[e] = X_e^T dG_e, X_e^T dU_e   (rows d, columns f)
  A.p_dim = D.d; A.n_p_tiles = (D.d + TP - 1) / TP; A.q_dim = D.f; A.n_q_tiles = (D.f + TQ - 1) / TQ;
  A.p0 = x_perm; A.p_ld = D.d;
  A.q0 = dg; A.q1 = du; A.q_ld = D.f;
  A.f0 = dw_gate; A.f1 = dw_up; A.f_expert_stride = (size_t)D.d * D.f; A.c_ld = D.f;
  launch_gemm<1, true, true, 2, 1, EPI_F32>("ffn_bwd_dw_gate_up", A, (long long)D.Et * A.n_p_tiles * A.n_q_tiles, st);
  return launch_status();
}
