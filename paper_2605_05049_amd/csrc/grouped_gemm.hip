// Grouped bf16 MFMA GEMMs of the SwiGLU expert FFNs over ragged per-expert row segments, forward and backward
// (Section III-A: W_up, W_gate in R^{d x f}, W_down in R^{f x d}, per-expert token counts s_e; these are the
// per-expert GEMMs of uneven, often small row counts that the abstract and Section II-A single out).
//
// One kernel template serves all seven contractions.  Every output tile is
//     C[p, q] = sum_k  P[p, k] * Q[q, k]          (p: 256 values, q: 256 values, k in steps of 64)
// where P is the operand whose index becomes the lane-column of the MFMA accumulator and Q the operand whose
// index becomes the accumulator register (so that each lane owns 4 consecutive q = 4 consecutive output
// elements of a row-major C).  An operand is "K-contiguous" (KC: element (r,k) at base[r*ld + k]) or
// "R-contiguous" (RC: element (r,k) at base[k*ld + r]).  KC tiles are read from LDS with 16-byte loads, RC tiles
// with the gfx950 transposing LDS read (ds_read_b64_tr_b16), so no operand is ever transposed in HBM.
//
//   forward   G,U = X Wg, X Wu     P = X (KC)        Q = Wg | Wu (RC)  two 128-wide halves, SwiGLU epilogue
//             Y   = H Wd           P = H (KC)        Q = Wd (RC)
//   backward  dH  = dY Wd^T        P = dY (KC)       Q = Wd (KC)       d(SwiGLU) epilogue -> dG, dU, H
//             dX  = dG Wg^T+dU Wu^T P = dG then dU (KC) Q = Wg then Wu (KC)  one accumulator, two K passes
//             dWd = H^T dY         P = H (RC)        Q = dY (RC)       ragged K = rows of the expert, fp32 out
//             dWg,dWu = X^T dG, X^T dU   P = X (RC)  Q = dG | dU (RC)  two 128-wide halves, ragged K, fp32 out
//
// Tiling: 512 threads = 8 wavefronts (2 along p x 4 along q); each wavefront owns 128 p x 64 q as 4x2 MFMA
// 32x32x16 blocks (128 fp32 accumulators per lane).  Tiles stream HBM/L2 -> LDS with the direct 16-byte
// global->LDS load (no register staging) into two 64 KB stages; step k+1 is in flight while step k is
// multiplied, one barrier per step.  A direct load is addressed by a scalar base (advanced once per step) plus one
// 32-bit per-lane offset that never changes, so the K loop does no per-lane address arithmetic.  The two wavefronts
// that share a SIMD request their parts of the next stage at different times of a step (one right after the
// barrier, the other half-way through its MFMAs): a wavefront is held up while its loads are accepted, and this way
// its partner has MFMAs to issue meanwhile; fragment reads run ahead of their MFMAs so that the partner, alone on
// the matrix pipe, does not stall on LDS latency.  The LDS destination of a direct load is fixed by the lane id, so bank
// conflicts are avoided by choosing WHICH 16-byte chunk each lane fetches (an XOR swizzle of the chunk index with
// row bits), and the fragment reads apply the same swizzle.  Every request is a whole 128-byte line (KC) or four of
// them (RC): the vector L1 handles about one line per two cycles whatever part of it is used.  Rows past the end of
// a ragged K (weight gradients) are fetched from a zeroed page.  Row tiles of the ragged dimension come from a
// device-built schedule (no host sync on the counts); the block-id -> tile map deals groups of 32 consecutive tiles
// (super-tiles of 8 x 4 tiles for the weight gradients) round-robin to the XCDs, so that tiles sharing a panel meet in
// one L2 and every XCD gets the same mix of experts; inside a group the tiles that take longest come first.
#include "common.h"

#include <algorithm>
#include <type_traits>

namespace moe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;                          // k step
constexpr int TILE = 256;                       // p extent, and (virtual) q extent, of a block tile
constexpr int NTHREADS = 512;
constexpr int TALL = TILE + 64;                 // rows of a tall tile: an expert's last full row tile plus up to 64 rows
constexpr int OPERAND_BYTES = TILE * BK * 2;    // 32 KB per 256-row operand per stage
constexpr int Q_STAGE_OFFSET = TALL * BK * 2;   // the Q operand follows the (up to 320-row, 40 KB) P operand
constexpr int P_AREA_BYTES = Q_STAGE_OFFSET;    // a stage's P operand
constexpr int STAGE_BYTES = Q_STAGE_OFFSET + OPERAND_BYTES;  // P + Q = 72 KB
                                                // two stages = 144 KB of the 160 KB of LDS
constexpr int kNumXcd = 8;
constexpr int kCusPerXcd = 32;
// A tile is cut along K only if it has at least MOE_SPLIT_MIN_STEPS k-steps, into parts of at least MOE_SPLIT_PART_STEPS
// (writing a part's fp32 tile and adding the parts costs about as much as 20 k-steps: a 32-step tile cut in four
// measured 4 % slower than left whole).
#ifndef MOE_SPLIT_MIN_STEPS
#define MOE_SPLIT_MIN_STEPS 48
#endif
#ifndef MOE_SPLIT_PART_STEPS
#define MOE_SPLIT_PART_STEPS 16
#endif
#ifndef MOE_WGRAD_PERSISTENT
#define MOE_WGRAD_PERSISTENT 1   // 0: never, 1: where the generic kernel's grid would be padded, 2: always
#endif
// How far ahead of their MFMAs a k-step reads its fragments (0: each group of 16 k reads its own; 1: half a group
// ahead; 2: rolling, see the k-step): for row tiles of up to 256 rows, for tall row tiles, for the tall row tiles of the
// SwiGLU forward, and for the weight gradients (whose transposing reads gained nothing from 2).
#ifndef MOE_FRAG_PIPELINE_ROW
#define MOE_FRAG_PIPELINE_ROW 2
#endif
#ifndef MOE_FRAG_PIPELINE_TALL
#define MOE_FRAG_PIPELINE_TALL 2
#endif
#ifndef MOE_FRAG_PIPELINE_TALL_SWIGLU
#define MOE_FRAG_PIPELINE_TALL_SWIGLU 1
#endif
#ifndef MOE_FRAG_PIPELINE_WGRAD
#define MOE_FRAG_PIPELINE_WGRAD 1
#endif
// k offset inside a step at which wavefronts 0..3 request their share of the next stage: half-way through it, or
// (weight gradients and the SwiGLU forward, where it measured 1-2 % faster; 2 % slower in the others) after three quarters
#ifndef MOE_EARLY_ISSUE_AT
#define MOE_EARLY_ISSUE_AT 32
#endif
#ifndef MOE_EARLY_ISSUE_AT_WIDE
#define MOE_EARLY_ISSUE_AT_WIDE 48
#endif

enum Epilogue { EPI_BF16 = 0, EPI_SWIGLU = 1, EPI_DSWIGLU = 2, EPI_F32 = 3 };

struct GemmArgs {
  // row-tile problems (forward / dgrad): schedule built on the device
  const int32_t* sched;    // [0] = number of row tiles; [64 + u] = expert of tile u; [64 + max_tiles + u] = its first tile
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
  const uint16_t* zero_page;  // 256 zeroed bytes: source of k-rows past the end of a ragged K
  float* partial;             // [kSplitParts][256][256] fp32: partial tiles of a split K range
  int32_t* counters;          // [kSplitCounters], zeroed by the schedule kernel and again by each tile's reducing part: parts of a split tile that have arrived
  // outputs
  uint16_t* c0; uint16_t* c1; uint16_t* c2; size_t c_ld;   // bf16 outputs (row-major, ld = q_dim)
  const uint16_t* g_in; const uint16_t* u_in;              // saved G, U for the d(SwiGLU) epilogue
  float* f0; float* f1; size_t f_expert_stride;            // fp32 outputs of the wgrads
  int sum_halves;          // NQ == 2 with fp32 output: write the sum of the two halves' results to f0 (f1 unused)
  int32_t* queue;          // weight gradients: 8 int32 (one per XCD), zeroed before the launch: tiles handed out so far
};

// One 256-wide operand of a tile, possibly made of two 128-wide halves from two tensors.
struct TileOperand {
  const uint16_t* base0;    // element (r = 0, k = 0) of the operand (of its first half when split)
  const uint16_t* base1;    // element (r = 0, k = 0) of the second half when split (else unused)
  size_t ld;                // elements between consecutive r (KC) or consecutive k (RC)
  int r_valid;              // valid r per half (<= 128 when split, <= 256 otherwise); beyond: clamped, never stored
};

// A 32 KB operand stage is filled by 32 direct-load instructions of 1 KB (instruction n fills LDS bytes [1024 n, +1024),
// lane L the 16 bytes at +16 L); wavefront w issues instructions 4w..4w+3.  This returns the byte offset of lane L's 16
// source bytes from the origin of the stage in global memory, i.e. from element (r = 0, k = first k of the step) of
// the tensor the instruction reads:
//   KC: instruction n = rows 8n..8n+7, whole 128-byte lines; LDS row r = 8 chunks of 8 k-values, chunk c at position
//       c ^ ((r >> 1) & 7).
//   RC: instruction n = k-rows 4(n/2)..+3, r-half n%2 (128 r-values, from the second tensor when split); inside the
//       1 KB, k-row j%4 takes 256 bytes = 16 chunks of 8 r-values, chunk c at position c ^ ((j & 3) << 2).
// The offset does not depend on the step, so one 32-bit register per instruction addresses the whole K loop on top
// of a scalar base that advances by one step at a time.
template <bool RC, bool SPLIT>
__device__ __forceinline__ unsigned load_offset(const TileOperand& op, int n, int lane) {
  static_assert(RC || !SPLIT, "split operands are R-contiguous");
  if (!RC) {
    const int r = n * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    const int rr = r < op.r_valid ? r : op.r_valid - 1;
    return (unsigned)(((size_t)rr * op.ld + c * 8) * 2);
  } else {
    const int kr = (n >> 1) * 4 + (lane >> 4);
    const int c = (lane & 15) ^ ((kr & 3) << 2);
    int col = c * 8 + ((!SPLIT && (n & 1)) ? 128 : 0);
    col = col < op.r_valid ? col : max(op.r_valid - 8, 0);  // (operands narrower than 8 are padded by their owner)
    return (unsigned)(((size_t)kr * op.ld + col) * 2);
  }
}

// Issues this wavefront's 4 direct loads of one operand stage for the 64 k-values starting at k0 (`delta`: element
// offset of the pass's tensors from the first pass's).
template <bool RC, bool SPLIT, bool NARROW = false>
__device__ __forceinline__ void issue_tile(const unsigned (&voff)[4], const TileOperand& op, ptrdiff_t delta, int k0, int k_end,
                                           const uint16_t* zero_page, char* lds_tile, int wave, int lane) {
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int n = wave * 4 + i;
    // Instructions that would only fetch rows or columns past the operand's valid extent are left out (short row
    // tiles, the last column tile of a width that is not a multiple of 256, the router's skinny problems); those LDS
    // rows then hold stale data, which only ever reaches accumulators that are never stored (an accumulator row or
    // column depends on its own operand row alone)
    if (NARROW && (RC ? (!SPLIT && (n & 1) && op.r_valid <= 128) : n * 8 >= op.r_valid)) continue;
    const uint16_t* sb = ((RC && SPLIT && (n & 1)) ? op.base1 : op.base0) + delta + (RC ? (size_t)k0 * op.ld : (size_t)k0);
    if (RC && k0 + BK > k_end) {  // the ragged end of K: k-rows past it come from the zeroed page
      const int kr = (n >> 1) * 4 + (lane >> 4);
      const char* g = (k0 + kr < k_end) ? reinterpret_cast<const char*>(sb) + voff[i] : reinterpret_cast<const char*>(zero_page);
      direct_load16(g, lds_tile + n * 1024);
    } else {
      direct_load16(sb, voff[i], lds_tile + n * 1024);
    }
  }
}

// 8 x 16 bytes that other CUs have written during this launch (32 bytes at each of four addresses): read at agent
// scope, so that this CU's vector L1 is bypassed whatever it holds (the partial tiles of a split K range).  One
// statement issues the eight loads and waits for them, so the compiler never sees a register whose load is in flight.
__device__ __forceinline__ void load8_agent(f32x4 (&v)[8], const float* p0, const float* p1, const float* p2, const float* p3) {
  asm volatile(
      "global_load_dwordx4 %0, %8, off sc1\n\tglobal_load_dwordx4 %1, %8, off offset:16 sc1\n\t"
      "global_load_dwordx4 %2, %9, off sc1\n\tglobal_load_dwordx4 %3, %9, off offset:16 sc1\n\t"
      "global_load_dwordx4 %4, %10, off sc1\n\tglobal_load_dwordx4 %5, %10, off offset:16 sc1\n\t"
      "global_load_dwordx4 %6, %11, off sc1\n\tglobal_load_dwordx4 %7, %11, off offset:16 sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
      : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
      : "memory");
}

// MFMA operand fragment: 32 r-values x 16 k-values; lane l gets r = r0 + l%32, k = kk + 8*(l/32) .. +7.
template <bool RC>
__device__ __forceinline__ bf16x8 read_frag(const char* tile, int r0, int kk, int lane) {
  if (!RC) {
    const int r = r0 + (lane & 31);
    const int c = (kk >> 3) + (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(tile + r * 128 + ((c ^ ((r >> 1) & 7)) << 4));
  } else {
    // Transposing read: inside each group of 16 lanes, lane p supplies the address of 4 consecutive r at k-row
    // p/4, r-chunk p%4, and receives the 4 k-rows of r = (group base) + p.
    const int p = lane & 15;
    const int k = kk + 8 * (lane >> 5) + (p >> 2);
    const int relem = r0 + 16 * ((lane >> 4) & 1) + 4 * (p & 3);
    const int c = relem >> 3;  // 0..31: bit 4 = r-half, bits 0..3 = chunk inside the half
    const char* a = tile + ((((k >> 2) << 1) + (c >> 4)) << 10) + ((k & 3) << 8) + (((c & 15) ^ ((k & 3) << 2)) << 4) +
                    ((relem & 7) << 1);
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(a));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(a + 2048));  // k + 4: the next group of 4 k-rows
    union { struct { s16x4 lo, hi; } s; bf16x8 v; } u;
    u.s.lo = lo;
    u.s.hi = hi;
    return u.v;
  }
}

// The same fragment addressed in three parts: `off` = the lane's byte offset inside an operand area for kk = 0
// (frag_offset), kk, and `area` = a wave-uniform constant (the LDS address of the operand area, plus 4096 bytes for every
// 32 rows further down a K-contiguous operand, whose swizzle has a period of 16 rows).  kk flips two address bits
// (K-contiguous: the 16-byte chunk index is XORed with the row's swizzle, and kk / 8 occupies bits of it that the
// lane's own part leaves clear) or adds 512 bytes per k-row pair (R-contiguous).  Written this way the loop-invariant
// part, off ^ 2 kk or off, is one register per operand and kk (K-contiguous) or per fragment (R-contiguous), and the
// rest goes into the read instruction's 16-bit offset field: 8 to 12 address registers over the K loop where one
// address per fragment, stage and kk took 48.
template <bool RC>
__device__ __forceinline__ unsigned frag_offset(int r0, int lane) {
  if (!RC) {
    const int r = r0 + (lane & 31);
    return (unsigned)(r * 128 + (((lane >> 5) ^ ((r >> 1) & 7)) << 4));
  } else {
    const int p = lane & 15;
    const int k = 8 * (lane >> 5) + (p >> 2);
    const int relem = r0 + 16 * ((lane >> 4) & 1) + 4 * (p & 3);
    const int c = relem >> 3;
    return (unsigned)(((((k >> 2) << 1) + (c >> 4)) << 10) + ((k & 3) << 8) + (((c & 15) ^ ((k & 3) << 2)) << 4) + ((relem & 7) << 1));
  }
}
template <bool RC>
__device__ __forceinline__ bf16x8 read_frag_at(unsigned off, int kk, unsigned area) {
  if (!RC) {
    typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
    return *reinterpret_cast<const lds_bf16x8*>((size_t)((off ^ (unsigned)(kk << 1)) + area));
  } else {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const unsigned a = off + (unsigned)(kk * 512) + area;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(size_t)a);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(size_t)(a + 2048u));
    union { struct { s16x4 lo, hi; } s; bf16x8 v; } u;
    u.s.lo = lo;
    u.s.hi = hi;
    return u.v;
  }
}

// Row tiles of an expert with n rows.  Without tall tiles: ceil(n / 256).  With them, a remainder of at most 64 rows
// does not get a tile of its own (which would stream the expert's whole weight panel once more for a handful of rows)
// but rides on the last full tile, which then has up to 320 rows: max(1, ceil((n - 64) / 256)).
__host__ __device__ __forceinline__ int row_tiles_of(int n, int tall) {
  if (n <= 0) return 0;
  return tall ? max(1, (n - 64 + TILE - 1) / TILE) : (n + TILE - 1) / TILE;
}

// KIND 0: row-tile problem (p = ragged rows of an expert, k = k_dim);  KIND 1: wgrad (k = ragged rows).
// NQ = 2: the q tile is two 128-wide halves from q0 and q1 (acc[0] = q0 result, acc[1] = q1 result at the same q).
template <int KIND, bool P_RC, bool Q_RC, int NQ, int NPASS, int EPI>
__global__ __launch_bounds__(NTHREADS) void grouped_gemm_kernel(const GemmArgs A) {
  // Two stages of P (up to 320 rows) | Q each.
  __shared__ __attribute__((aligned(1024))) char lds[2 * STAGE_BYTES];
  auto p_area = [&](int s) __attribute__((always_inline)) { return lds + s * STAGE_BYTES; };
  auto q_area = [&](int s) __attribute__((always_inline)) { return lds + s * STAGE_BYTES + P_AREA_BYTES; };
  constexpr int TQ = TILE / NQ;  // q extent per output tensor

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wq = wave >> 1;         // 0..3 along q
  const int late = wave >> 2;       // wavefronts 4..7 share their SIMDs with 0..3 and load at another time of the step

  // ---- block id -> tile ----
  int expert, p_row0 = 0, p_valid, q0_col, k_len;
  size_t krow0 = 0;
  // Tail split (row-tile problems with one output tile per block): when an XCD's last round of tiles would occupy at most half of its
  // 32 CUs, each of those tiles is cut along K into `split` parts that run side by side; a part writes its fp32
  // partial tile to the workspace and the part that arrives last adds them up (no part ever waits for another).
  constexpr bool SPLITK = (KIND == 0 && NQ == 1);   // (the SwiGLU forward, with two output tensors per tile, measured no gain)
  int split = 1, part = 0, part_slot = 0;
  int p_tile_idx;  // index of the tile along p
  if (KIND == 0) {
    // Groups of 32 consecutive tiles of the logical order (about 4 row tiles x 8 column tiles of one expert: the tiles
    // that share panels) are dealt round-robin to the XCDs, so that every XCD gets the same mix of experts and of tile
    // heights (contiguous runs had handed a whole expert, with its tall or short tiles, to one XCD).  What is left after
    // the last complete deal of 8 groups (fewer than 256 tiles) is cut into 8 equal runs, one per XCD.
    const int n_row_tiles = A.sched[0];
    const long long total = (long long)n_row_tiles * A.n_q_tiles;
    const long long within = blockIdx.x / kNumXcd;
    const int xcd = blockIdx.x % kNumXcd;
    const long long deals = total / (kCusPerXcd * kNumXcd);          // rounds of 32 tiles every XCD gets
    const long long dealt = deals * kCusPerXcd;                       // ... = tiles per XCD from the deals
    const long long rest = total - dealt * kNumXcd;                   // < 256 tiles left over
    const long long chunk = (rest + kNumXcd - 1) / kNumXcd;           // <= 32 per XCD
    const long long lo = dealt * kNumXcd + (long long)xcd * chunk;
    const long long cnt = max(min(chunk, total - lo), 0LL);           // left-over tiles of this XCD
    long long full = cnt;
    if (SPLITK) {
      const int rem = (int)(cnt % kCusPerXcd);
      const int nk_all = ((A.k_dim + BK - 1) / BK) * NPASS;
      if (rem > 0 && rem <= kCusPerXcd / 2 && nk_all >= MOE_SPLIT_MIN_STEPS) {
        split = min(min(kCusPerXcd / rem, 8), nk_all / MOE_SPLIT_PART_STEPS);
        full = cnt - rem;
      }
    }
    long long lid;
    if (within < dealt) {
      lid = ((within / kCusPerXcd) * kNumXcd + xcd) * kCusPerXcd + within % kCusPerXcd;
      split = 1;
    } else if (within - dealt < full) {
      lid = lo + (within - dealt);
      split = 1;
    } else {
      const long long u = within - dealt - full;
      if (u >= (cnt - full) * split) return;
      lid = lo + full + u / split;
      part = (int)(u % split);
      part_slot = xcd * kCusPerXcd + (int)u;
    }
    const int u = (int)(lid / A.n_q_tiles);  // some row tile of the expert this block works for
    expert = A.sched[64 + u];
    const int e_lo = A.offsets[expert], e_hi = A.offsets[expert + 1];
    const int e_tiles = row_tiles_of(e_hi - e_lo, A.sched[1]);
    const int first = A.sched[64 + A.max_tiles + u];  // index of the expert's first row tile
    // Order inside an expert: column tile after column tile, each with all its row tiles (32 consecutive tiles, which
    // an XCD runs together, are then about 4 row tiles x 8 column tiles: 4 + 8 panels), a tall last row tile first.
    // Blocks are handed to CUs in order as CUs become free, so a tile that takes longer should come early in its
    // group of 32: an expert of at most 4 row tiles, whose 8 column tiles fill a group, is therefore walked row
    // tile after row tile inside each band of 8 column tiles (the same 32 tiles, the 8 tall ones first: the CUs that
    // ran the previous group's tall tiles then get ordinary ones).
    const int local = (int)(lid - (long long)first * A.n_q_tiles);
    int qt, m;
    if (e_tiles <= 4) {
      const int band = local / (e_tiles * 8), in_band = local % (e_tiles * 8);
      const int band_q = min(8, A.n_q_tiles - band * 8);   // column tiles of this band
      qt = band * 8 + in_band % band_q;
      m = in_band / band_q;
    } else {
      qt = local / e_tiles;
      m = local % e_tiles;
    }
    const bool tall_last = (e_hi - e_lo) - (e_tiles - 1) * TILE > TILE;
    const int mt = tall_last ? (m == 0 ? e_tiles - 1 : m - 1) : m;
    p_row0 = e_lo + mt * TILE;
    p_valid = (mt == e_tiles - 1) ? e_hi - p_row0 : TILE;   // (the last tile may be a tall one: up to 320 rows)
    p_tile_idx = mt;
    q0_col = qt * TQ;
    k_len = A.k_dim;
  } else {
    // Tiles of an expert are walked in 8 x 4 super-tiles (8 along p, 4 along q = the 32 tiles one XCD runs at a
    // time): each p panel then meets 4 q panels and each q panel 8 p panels in that XCD's L2 instead of one
    // panel being re-fetched for every tile of the other dimension.  The grid is padded to whole super-tiles.
    // A tile's duration is proportional to its expert's row count, so the super-tiles are dealt round-robin to the
    // XCDs (not in contiguous runs, which would hand a whole large expert to one XCD), experts with the most rows
    // first (the tail of the launch is then made of short tiles).
    const int sp = (A.n_p_tiles + 7) / 8, sq = (A.n_q_tiles + 3) / 4;
    const int supers_per_e = sp * sq;
    const long long n_super = (long long)supers_per_e * A.Et;
    const long long within = blockIdx.x / kNumXcd;
    const long long sid = (within >> 5) * kNumXcd + (blockIdx.x % kNumXcd);
    if (sid >= n_super) return;
    expert = A.sched[64 + 2 * A.max_tiles + (int)(sid / supers_per_e)];  // the (sid / supers_per_e)-th largest expert
    const int super = (int)(sid % supers_per_e), in_super = (int)(within & 31);
    const int pt = (super % sp) * 8 + (in_super & 7);
    const int qt = (super / sp) * 4 + (in_super >> 3);
    if (pt >= A.n_p_tiles || qt >= A.n_q_tiles) return;  // padding of the super-tile grid
    p_tile_idx = pt;
    const int e_lo = A.offsets[expert], e_hi = A.offsets[expert + 1];
    k_len = e_hi - e_lo;
    krow0 = (size_t)e_lo;
    p_row0 = pt * TILE;
    p_valid = min(TILE, A.p_dim - p_row0);
    q0_col = qt * TQ;
    if (k_len == 0 && A.accumulate) return;  // nothing to add
  }
  const int q_valid = min(TQ, A.q_dim - q0_col);

  // LDS row origin of this wavefront's two q fragments
  const int qr0 = (NQ == 2) ? wq * 32 : wq * 64;
  const int qr1 = (NQ == 2) ? 128 + wq * 32 : wq * 64 + 32;

  TileOperand P, Q;
  ptrdiff_t p_pass_delta = 0, q_pass_delta = 0;  // second K pass (dX): same rows of the second pair of tensors
  if (KIND == 0) {
    P.base0 = P.base1 = P_RC ? A.p0 + p_row0 : A.p0 + (size_t)p_row0 * A.p_ld;
    P.ld = A.p_ld;
    P.r_valid = p_valid;
    const uint16_t* qa = A.q0 + (size_t)expert * A.q_expert_stride;
    Q.base0 = Q.base1 = Q_RC ? qa + q0_col : qa + (size_t)q0_col * A.q_ld;
    if (NQ == 2) Q.base1 = A.q1 + (size_t)expert * A.q_expert_stride + q0_col;
    Q.ld = A.q_ld;
    Q.r_valid = q_valid;
    if (NPASS == 2) {
      p_pass_delta = A.p1 - A.p0;
      q_pass_delta = A.q1 - A.q0;
    }
  } else {
    P.base0 = P.base1 = A.p0 + krow0 * A.p_ld + p_row0;
    P.ld = A.p_ld;
    P.r_valid = p_valid;
    Q.base0 = Q.base1 = A.q0 + krow0 * A.q_ld + q0_col;
    if (NQ == 2) Q.base1 = A.q1 + krow0 * A.q_ld + q0_col;
    Q.ld = A.q_ld;
    Q.r_valid = q_valid;
  }
  // Tiles that are neighbours along p share their q panel and run side by side on one XCD, in step with each other.
  // In every other one of them each wavefront issues the q loads of the wavefront that loads at the other time of
  // the step (any wavefront may issue any instruction of a stage: the LDS destination comes with the instruction).
  // Each half of the shared panel is then requested right after the barrier by half of its users, and the requests
  // the other half makes half a step later find it in, or on its way to, the L2.  (Left out where it measured
  // slower or was not measured: the forward down projection and the router's skinny problems.)
  constexpr bool ALTERNATE_Q = !(KIND == 0 && Q_RC && NQ == 1 && EPI == EPI_BF16);
  const int iwq = ALTERNATE_Q ? (wave ^ ((p_tile_idx & 1) << 2)) : wave;
  unsigned pvo[4], qvo[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    pvo[i] = load_offset<P_RC, false>(P, wave * 4 + i, lane);
    qvo[i] = load_offset<Q_RC, NQ == 2>(Q, iwq * 4 + i, lane);
  }
  const int nk_pass = (k_len + BK - 1) / BK;  // k-steps per K pass
  const int nk = nk_pass * NPASS;             // k-steps of the whole contraction
  // this wavefront's 8 direct loads of step j of the contraction
  auto issue_as = [&](auto narrow_p, int j, char* p_dst, char* q_dst) __attribute__((always_inline)) {
    const bool second = (NPASS == 2) && j >= nk_pass;
    const int k0 = (second ? j - nk_pass : j) * BK;
    issue_tile<P_RC, false, decltype(narrow_p)::value>(pvo, P, second ? p_pass_delta : (ptrdiff_t)0, k0, k_len, A.zero_page, p_dst, wave, lane);
    issue_tile<Q_RC, NQ == 2>(qvo, Q, second ? q_pass_delta : (ptrdiff_t)0, k0, k_len, A.zero_page, q_dst, iwq, lane);
  };
  // the k-steps this block multiplies: all of them, or its part of a split tile
  const int kt_per = (nk + split - 1) / split;
  const int kt_begin = part * kt_per, kt_end = min(nk, kt_begin + kt_per);
  // (the first stage is requested before anything else is set up; rows a short tile does not have are clamped here)
  if (kt_begin < kt_end) issue_as(std::false_type{}, kt_begin, p_area(0), q_area(0));
  // Height class of the tile: each of the two wavefronts along p multiplies PB blocks of 32 rows (4, 2 or 1), so a
  // ragged last row tile of an expert issues MFMAs and row loads for its class (256, 128 or 64 rows) only.
  auto run = [&](auto pb_c) __attribute__((always_inline)) {
  constexpr int PB = decltype(pb_c)::value;
  // (a short tile leaves out the loads of the rows it does not have)
  // a tall tile's rows 256.. are one more instruction per wavefront (instruction 32 + wave: rows 256 + 8 wave .. +7)
  const unsigned pvo_tall = (PB == 5) ? load_offset<P_RC, false>(P, 32 + wave, lane) : 0u;
  auto issue_tall = [&](int j, char* p_dst) __attribute__((always_inline)) {
    if (PB == 5 && (32 + wave) * 8 < p_valid) {
      const bool second = (NPASS == 2) && j >= nk_pass;
      const int k0 = (second ? j - nk_pass : j) * BK;
      direct_load16(P.base0 + (second ? p_pass_delta : (ptrdiff_t)0) + k0, pvo_tall, p_dst + (32 + wave) * 1024);
    }
  };
  auto issue = [&](int j, int s) __attribute__((always_inline)) {
    issue_as(std::integral_constant<bool, (PB < 4)>{}, j, p_area(s), q_area(s));
    issue_tall(j, p_area(s));
  };
  if (kt_begin < kt_end) issue_tall(kt_begin, p_area(0));   // (the rest of the first stage was requested above)
  const int wp = (wave & 1) * (PB * 32);  // p origin of this wavefront
  f32x16 acc[2][PB];  // [q sub-tile a][p sub-tile b]
#pragma unroll
  for (int a = 0; a < 2; a++)
#pragma unroll
    for (int b = 0; b < PB; b++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[a][b][v] = 0.f;

  // One k-step: wait for stage `cur`, multiply it, and meanwhile fill `nxt` with step kt+1.  The two wavefronts of a
  // SIMD request their share of the next stage at different times of the step (one before its MFMAs, the other
  // between its two halves of them), so that while one is held up issuing loads the other keeps the matrix pipe busy.
  // (next to a tall tile's 160 accumulator registers the SwiGLU forward, with its two q tensors, has room for half a
  // group of fragments in flight only; a register spilled inside the K loop is ruinous here: its reload waits on the
  // counter that the direct loads share)
  constexpr int FRAG_PIPELINE = (PB == 5) ? (EPI == EPI_SWIGLU ? MOE_FRAG_PIPELINE_TALL_SWIGLU : MOE_FRAG_PIPELINE_TALL)
                                          : (KIND == 0) ? MOE_FRAG_PIPELINE_ROW : MOE_FRAG_PIPELINE_WGRAD;
  // Per-lane LDS offsets of this wavefront's fragments (at kk = 0) from the start of a stage.
  unsigned p_off[PB], q_off[2];
#pragma unroll
  for (int b = 0; b < PB; b++) p_off[b] = frag_offset<P_RC>(wp + 32 * b, lane);
  q_off[0] = frag_offset<Q_RC>(qr0, lane);
  q_off[1] = frag_offset<Q_RC>(qr1, lane);
  auto k_step = [&](int cur, int nxt, int kt) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this thread's loads of step kt have landed in LDS
    __syncthreads();                     // ... and everyone's; everyone is also done reading the other stage
    if (late && kt + 1 < kt_end) issue(kt + 1, nxt);
    const unsigned p_base = (unsigned)(size_t)(lptr_t)p_area(cur), q_base = (unsigned)(size_t)(lptr_t)q_area(cur);
    // (K-contiguous operand: 32 rows further is 4096 bytes further with the same swizzle, so all fragments of the
    // operand share the address register of the first and differ in the instruction's offset field)
    auto rp = [&](int b, int kk) __attribute__((always_inline)) {
      return P_RC ? read_frag_at<P_RC>(p_off[b], kk, p_base) : read_frag_at<P_RC>(p_off[0], kk, p_base + 4096u * b);
    };
    auto rq = [&](int a, int kk) __attribute__((always_inline)) {
      return Q_RC ? read_frag_at<Q_RC>(q_off[a], kk, q_base) : read_frag_at<Q_RC>(q_off[0], kk, q_base + 128u * (NQ == 2 ? 128 : 32) * a);
    };
    constexpr int EARLY_AT = (KIND == 1 || EPI == EPI_SWIGLU) ? MOE_EARLY_ISSUE_AT_WIDE : MOE_EARLY_ISSUE_AT;
    auto early_issue = [&](int kk) __attribute__((always_inline)) {
      if (kk == EARLY_AT) {
        __builtin_amdgcn_sched_barrier(0);
        if (!late && kt + 1 < kt_end) issue(kt + 1, nxt);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if constexpr (FRAG_PIPELINE == 0) {
#pragma unroll
      for (int kk = 0; kk < BK; kk += 16) {
        early_issue(kk);
        bf16x8 pf[PB], qf[2];
        qf[0] = rq(0, kk);
        qf[1] = rq(1, kk);
#pragma unroll
        for (int b = 0; b < PB; b++) pf[b] = rp(b, kk);
#pragma unroll
        for (int b = 0; b < PB; b++)
#pragma unroll
          for (int a = 0; a < 2; a++)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[a], pf[b], acc[a][b], 0, 0, 0);
      }
    } else if constexpr (FRAG_PIPELINE == 1) {
      // The fragments of a group of 16 k are read half a group ahead of the MFMAs that use them: the p blocks of a
      // group's second half while its first half multiplies, the q fragments (two sets) and the first p blocks of
      // the next group while the second half does.
      constexpr int HA = (PB + 1) / 2;   // p blocks of the first half
      bf16x8 pf[PB], qf[2][2];
      auto read_half_a = [&](int kk, bf16x8 (&q)[2]) __attribute__((always_inline)) {
        q[0] = rq(0, kk);
        q[1] = rq(1, kk);
#pragma unroll
        for (int b = 0; b < HA; b++) pf[b] = rp(b, kk);
      };
      read_half_a(0, qf[0]);
#pragma unroll
      for (int g = 0; g < BK / 16; g++) {
        const int kk = 16 * g;
        early_issue(kk);
#pragma unroll
        for (int b = HA; b < PB; b++) pf[b] = rp(b, kk);
#pragma unroll
        for (int b = 0; b < HA; b++)
#pragma unroll
          for (int a = 0; a < 2; a++)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[g & 1][a], pf[b], acc[a][b], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (g + 1 < BK / 16) read_half_a(kk + 16, qf[(g + 1) & 1]);
#pragma unroll
        for (int b = HA; b < PB; b++)
#pragma unroll
          for (int a = 0; a < 2; a++)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[g & 1][a], pf[b], acc[a][b], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      // Rolling fragments: a p fragment is read again, for the next group of 16 k, right after the two MFMAs that use
      // it; the two q fragments, which every MFMA of a group uses, alternate between two sets.  A wavefront that is
      // alone on its SIMD's matrix pipe (its partner is held up issuing loads) then does not stall on the LDS latency
      // between groups, and the LDS reads are spread evenly between the MFMAs.
      bf16x8 pf[PB], qf[2][2];
      qf[0][0] = rq(0, 0);
      qf[0][1] = rq(1, 0);
#pragma unroll
      for (int b = 0; b < PB; b++) pf[b] = rp(b, 0);
#pragma unroll
      for (int g = 0; g < BK / 16; g++) {
        const int kk = 16 * g;
        const bool more = g + 1 < BK / 16;
        early_issue(kk);
#pragma unroll
        for (int b = 0; b < PB; b++) {
          acc[0][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[g & 1][0], pf[b], acc[0][b], 0, 0, 0);
          acc[1][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[g & 1][1], pf[b], acc[1][b], 0, 0, 0);
          if (more) {
            pf[b] = rp(b, kk + 16);
            if (b == 0) qf[(g + 1) & 1][0] = rq(0, kk + 16);
            if (b == (PB > 2 ? 1 : 0)) qf[(g + 1) & 1][1] = rq(1, kk + 16);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  };
  // Tiles of at most 64 rows (PB == 1) multiply little per step and are bound by the latency of their loads, and
  // their P operand needs 8 KB of a stage's 40: they run a ring of three slots, two steps ahead instead of one.
  //   slot 0: the first stage's areas (the first stage was requested above)
  //   slot 1: the second stage's areas
  //   slot 2: P at 8 KB into the second P area, Q at 8 KB into the first (rows 64.. of P areas, which these tiles never read)
  // Every wavefront issues one P instruction (rows 8 w .. 8 w + 7, clamped onto the tile's last row) and its four Q
  // instructions per step: 5 loads, the same for all, so that "all but the youngest step" is vmcnt(5).
  if constexpr (PB == 1) {
    const unsigned pvo1 = load_offset<P_RC, false>(P, wave, lane);
    auto issue1 = [&](int j, char* p_dst, char* q_dst) __attribute__((always_inline)) {
      const bool second = (NPASS == 2) && j >= nk_pass;
      const int k0 = (second ? j - nk_pass : j) * BK;
      direct_load16(P.base0 + (second ? p_pass_delta : (ptrdiff_t)0) + k0, pvo1, p_dst + wave * 1024);
      issue_tile<Q_RC, NQ == 2>(qvo, Q, second ? q_pass_delta : (ptrdiff_t)0, k0, k_len, A.zero_page, q_dst, iwq, lane);
    };
    auto ring_step = [&](const char* p_lds, const char* q_lds, char* p_fill, char* q_fill, int kt) {
      if (kt + 1 < kt_end) __builtin_amdgcn_s_waitcnt(0x0F75);  // vmcnt(5): all but the 5 loads of step kt + 1
      else __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();   // step kt has landed for everyone; everyone is done with step kt - 1, whose slot step kt + 2 takes
      if (late && kt + 2 < kt_end) issue1(kt + 2, p_fill, q_fill);
#pragma unroll
      for (int kk = 0; kk < BK; kk += 16) {
        if (kk == MOE_EARLY_ISSUE_AT) {
          __builtin_amdgcn_sched_barrier(0);
          if (!late && kt + 2 < kt_end) issue1(kt + 2, p_fill, q_fill);
          __builtin_amdgcn_sched_barrier(0);
        }
        const bf16x8 q0f = read_frag<Q_RC>(q_lds, qr0, kk, lane), q1f = read_frag<Q_RC>(q_lds, qr1, kk, lane);
        const bf16x8 p0f = read_frag<P_RC>(p_lds, wp, kk, lane);
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q0f, p0f, acc[0][0], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q1f, p0f, acc[1][0], 0, 0, 0);
      }
    };
    char* const rp[3] = {p_area(0), p_area(1), p_area(1) + 8192};
    char* const rq[3] = {q_area(0), q_area(1), p_area(0) + 8192};
    if (kt_begin + 1 < kt_end) issue1(kt_begin + 1, rp[1], rq[1]);
    for (int kt = kt_begin; kt < kt_end; kt += 3) {
      ring_step(rp[0], rq[0], rp[2], rq[2], kt);
      if (kt + 1 < kt_end) ring_step(rp[1], rq[1], rp[0], rq[0], kt + 1);
      if (kt + 2 < kt_end) ring_step(rp[2], rq[2], rp[1], rq[1], kt + 2);
    }
  } else {
    for (int kt = kt_begin; kt < kt_end; kt += 2) {
      k_step(0, 1, kt);
      if (kt + 1 < kt_end) k_step(1, 0, kt + 1);
    }
  }

  // ---- epilogue.  acc[a][b][v] holds  p = wp + 32b + lane%32,  q (inside the output's tile) =
  //      NQ == 1: 64 wq + 32a + 8(v/4) + 4(lane/32) + v%4      NQ == 2: 32 wq + 8(v/4) + 4(lane/32) + v%4 of output a.
  // Lanes 0..31 of an accumulator own 32 different rows, so storing from the accumulators would touch 64 cache lines
  // per instruction.  Instead each wavefront bounces 32 rows at a time through its own 16 KB of the (now idle) LDS
  // and reads them back row-wise: every global access is then 16 bytes per lane over 64..256 contiguous bytes per row,
  // and the SwiGLU element-wise math runs on that side (8 consecutive q per lane).
  constexpr int W = (NQ == 2) ? 32 : 64;       // q extent this wavefront owns per output tensor
  constexpr int PITCH = W * 4 + 16;            // bytes per staged fp32 row; the +16 keeps 16-byte accesses conflict-free
  __syncthreads();                             // every wavefront has finished reading the stages
  char* wlds = lds + wave * 16384;
  const int q_base = wq * W;                   // first q of this wavefront inside the output's tile
  // 8 consecutive outputs of a row: x (and, for the SwiGLU forward, the matching values y of the second tensor) ->
  // the kernel's bf16 outputs at element offset o
  auto emit8 = [&](size_t o, const float (&x)[8], const float (&y)[8]) __attribute__((always_inline)) {
    if (EPI == EPI_BF16) {
      *reinterpret_cast<uint4*>(A.c0 + o) =
          make_uint4(pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7]));
    } else if (EPI == EPI_SWIGLU) {  // x = G, y = U
      float h[8];
#pragma unroll
      for (int i = 0; i < 8; i++) h[i] = x[i] * __builtin_amdgcn_rcpf(1.0f + __expf(-x[i])) * y[i];   // (rcp: 1 ulp, bf16 result)
      *reinterpret_cast<uint4*>(A.c0 + o) =
          make_uint4(pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7]));
      *reinterpret_cast<uint4*>(A.c1 + o) =
          make_uint4(pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3]), pack_bf16(y[4], y[5]), pack_bf16(y[6], y[7]));
      *reinterpret_cast<uint4*>(A.c2 + o) =
          make_uint4(pack_bf16(h[0], h[1]), pack_bf16(h[2], h[3]), pack_bf16(h[4], h[5]), pack_bf16(h[6], h[7]));
    } else if (EPI == EPI_DSWIGLU) {  // x = dH; read saved G, U; write dG, dU, H
      const uint4 gi = *reinterpret_cast<const uint4*>(A.g_in + o);
      const uint4 ui = *reinterpret_cast<const uint4*>(A.u_in + o);
      const float g[8] = {bf16lo(gi.x), bf16hi(gi.x), bf16lo(gi.y), bf16hi(gi.y), bf16lo(gi.z), bf16hi(gi.z), bf16lo(gi.w), bf16hi(gi.w)};
      const float u[8] = {bf16lo(ui.x), bf16hi(ui.x), bf16lo(ui.y), bf16hi(ui.y), bf16lo(ui.z), bf16hi(ui.z), bf16lo(ui.w), bf16hi(ui.w)};
      float dg[8], du[8], h[8];
#pragma unroll
      for (int i = 0; i < 8; i++) {
        const float sg = __builtin_amdgcn_rcpf(1.0f + __expf(-g[i]));   // (rcp: 1 ulp, bf16 results)
        const float sl = g[i] * sg;
        h[i] = sl * u[i];
        du[i] = x[i] * sl;
        dg[i] = x[i] * u[i] * (sg * (1.0f + g[i] * (1.0f - sg)));
      }
      *reinterpret_cast<uint4*>(A.c0 + o) =
          make_uint4(pack_bf16(dg[0], dg[1]), pack_bf16(dg[2], dg[3]), pack_bf16(dg[4], dg[5]), pack_bf16(dg[6], dg[7]));
      *reinterpret_cast<uint4*>(A.c1 + o) =
          make_uint4(pack_bf16(du[0], du[1]), pack_bf16(du[2], du[3]), pack_bf16(du[4], du[5]), pack_bf16(du[6], du[7]));
      *reinterpret_cast<uint4*>(A.c2 + o) =
          make_uint4(pack_bf16(h[0], h[1]), pack_bf16(h[2], h[3]), pack_bf16(h[4], h[5]), pack_bf16(h[6], h[7]));
    }
  };
  if (SPLITK && split > 1) {
    // ---- a part of a split tile: fp32 partial tile [row][256] -> workspace, then whoever arrives last reduces
    float* mine = A.partial + (size_t)part_slot * (TALL * TILE);
#pragma unroll
    for (int b = 0; b < PB; b++) {
#pragma unroll
      for (int a = 0; a < 2; a++)
#pragma unroll
        for (int v4 = 0; v4 < 4; v4++) {
          const int q = 32 * a + 8 * v4 + 4 * (lane >> 5);
          float4 r = make_float4(acc[a][b][4 * v4], acc[a][b][4 * v4 + 1], acc[a][b][4 * v4 + 2], acc[a][b][4 * v4 + 3]);
          *reinterpret_cast<float4*>(wlds + (lane & 31) * PITCH + q * 4) = r;
        }
      __builtin_amdgcn_s_waitcnt(0xC07F);
      __builtin_amdgcn_wave_barrier();
      constexpr int LPR = W / 4;          // lanes per row (4 fp32 per lane)
      constexpr int RPI = 64 / LPR;       // rows per instruction
#pragma unroll
      for (int it = 0; it < 32 / RPI; it++) {
        const int r = it * RPI + lane / LPR;
        const int q = (lane % LPR) * 4;
        if (wp + 32 * b + r < p_valid && q_base + q < q_valid) {  // (the reduction reads only valid rows and columns)
          *reinterpret_cast<float4*>(mine + (size_t)(wp + 32 * b + r) * TILE + q_base + q) =
              *reinterpret_cast<const float4*>(wlds + r * PITCH + q * 4);
        }
      }
      __builtin_amdgcn_s_waitcnt(0xC07F);
      __builtin_amdgcn_wave_barrier();
    }
    // All parts of a tile carry the same blockIdx.x % 8 and so run on one XCD, whose L2 they share: a store that has
    // been acknowledged (vmcnt) is then visible to the other parts at the L2, and no cache has to be written back or
    // invalidated; the reducing part reads the partial tiles at agent scope, i.e. past its own vector L1.  That
    // placement is checked, not assumed: a part that finds itself on another XCD falls back to device-wide fences and
    // says so in the upper half of the counter, which makes the reducing part fence as well.
    __shared__ int arrived_before;
    const bool on_home_xcd = (__builtin_amdgcn_s_getreg((31 << 11) | 20) & 0xF) == (unsigned)(blockIdx.x % kNumXcd);
    if (on_home_xcd) __builtin_amdgcn_s_waitcnt(0x0F70);  // this thread's part of the partial tile has reached the L2
    else __threadfence();
    __syncthreads();   // ... and so has every other thread's, before the arrival is counted
    int32_t* const arrivals = A.counters + (part_slot / kCusPerXcd) * (kCusPerXcd / 2) + (part_slot % kCusPerXcd) / split;
    if (tid == 0) arrived_before = atomicAdd(arrivals, on_home_xcd ? 1 : 0x10001);
    __syncthreads();
    if ((arrived_before & 0xFFFF) != split - 1) return;
    if (tid == 0) *arrivals = 0;   // every part has arrived: the counter is clear again for the next kernel that splits tiles
    if (!on_home_xcd || (arrived_before >> 16)) __threadfence();  // some part wrote through another XCD's L2
    const float* parts = A.partial + (size_t)(part_slot - part) * (TALL * TILE);
    // the valid part of the tile only: p_valid rows of ceil(q_valid / 8) groups of 8 columns, spread over all threads;
    // the parts are added in part order
    const int nqv = (q_valid + 7) >> 3;
    const int n_items = p_valid * nqv;
    for (int idx = tid; idx < n_items; idx += NTHREADS) {
      const int p = idx / nqv, q = (idx - p * nqv) * 8;
      float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      const float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      const float* src = parts + p * TILE + q;
      for (int sp = 0; sp < split; sp += 4) {   // four parts' 32 bytes in flight (parts past the last: the last again, not added)
        f32x4 v[8];
        load8_agent(v, src + (size_t)sp * (TALL * TILE), src + (size_t)min(sp + 1, split - 1) * (TALL * TILE),
                    src + (size_t)min(sp + 2, split - 1) * (TALL * TILE), src + (size_t)min(sp + 3, split - 1) * (TALL * TILE));
#pragma unroll
        for (int j = 0; j < 4; j++) {
          if (sp + j < split) {
            x[0] += v[2 * j].x; x[1] += v[2 * j].y; x[2] += v[2 * j].z; x[3] += v[2 * j].w;
            x[4] += v[2 * j + 1].x; x[5] += v[2 * j + 1].y; x[6] += v[2 * j + 1].z; x[7] += v[2 * j + 1].w;
          }
        }
      }
      emit8((size_t)(p_row0 + p) * A.c_ld + q0_col + q, x, y);
    }
    return;
  }
#pragma unroll
  for (int b = 0; b < PB; b++) {
    // registers -> LDS (fp32), 32 rows x W columns per output tensor (second tensor at +8 KB when NQ == 2)
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
      for (int v4 = 0; v4 < 4; v4++) {
        const int q = (NQ == 2 ? 0 : 32 * a) + 8 * v4 + 4 * (lane >> 5);
        float4 r = make_float4(acc[a][b][4 * v4], acc[a][b][4 * v4 + 1], acc[a][b][4 * v4 + 2], acc[a][b][4 * v4 + 3]);
        *reinterpret_cast<float4*>(wlds + (NQ == 2 ? a * 8192 : 0) + (lane & 31) * PITCH + q * 4) = r;
      }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wavefront's own LDS writes are done
    __builtin_amdgcn_wave_barrier();
    if (EPI == EPI_F32) {
      // 4 q per lane (16 bytes of fp32)
      constexpr int LPR = W / 4;          // lanes per row
      constexpr int RPI = 64 / LPR;       // rows per instruction
#pragma unroll
      for (int it = 0; it < 32 / RPI; it++) {
        const int r = it * RPI + lane / LPR;
        const int q = (lane % LPR) * 4;
        const int p = wp + 32 * b + r;
        if (p < p_valid && q_base + q < q_valid) {
          const size_t o = (size_t)expert * A.f_expert_stride + (size_t)(p_row0 + p) * A.c_ld + q0_col + q_base + q;
#pragma unroll
          for (int n = 0; n < NQ; n++) {
            float4 v = *reinterpret_cast<const float4*>(wlds + n * 8192 + r * PITCH + q * 4);
            if (NQ == 2 && A.sum_halves) {   // (uniform over the launch)
              if (n == 1) break;
              const float4 v1 = *reinterpret_cast<const float4*>(wlds + 8192 + r * PITCH + q * 4);
              v.x += v1.x; v.y += v1.y; v.z += v1.z; v.w += v1.w;
            }
            float* dst = (n == 0 ? A.f0 : A.f1) + o;
            // (16-byte stores: the row pitch is a multiple of 4 and a row has room for whole groups of 4: d_model and
            // d_ffn are multiples of 64, the router's partial results are padded to 4)
            if (A.accumulate) {
              const float4 old = *reinterpret_cast<const float4*>(dst);
              v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w;
            }
            *reinterpret_cast<float4*>(dst) = v;
          }
        }
      }
    } else {
      // 8 q per lane (16 bytes of bf16)
      constexpr int LPR = W / 8;
      constexpr int RPI = 64 / LPR;
#pragma unroll
      for (int it = 0; it < 32 / RPI; it++) {
        const int r = it * RPI + lane / LPR;
        const int q = (lane % LPR) * 8;
        const int p = wp + 32 * b + r;
        if (p < p_valid && q_base + q < q_valid) {
          const size_t o = (size_t)(p_row0 + p) * A.c_ld + q0_col + q_base + q;
          const float4 x0 = *reinterpret_cast<const float4*>(wlds + r * PITCH + q * 4);
          const float4 x1 = *reinterpret_cast<const float4*>(wlds + r * PITCH + q * 4 + 16);
          const float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
          float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          if (EPI == EPI_SWIGLU) {  // the second staged tensor is U
            const float4 y0 = *reinterpret_cast<const float4*>(wlds + 8192 + r * PITCH + q * 4);
            const float4 y1 = *reinterpret_cast<const float4*>(wlds + 8192 + r * PITCH + q * 4 + 16);
            y[0] = y0.x; y[1] = y0.y; y[2] = y0.z; y[3] = y0.w; y[4] = y1.x; y[5] = y1.y; y[6] = y1.z; y[7] = y1.w;
          }
          emit8(o, x, y);
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // the read-back is complete before the next 32 rows overwrite the buffer
    __builtin_amdgcn_wave_barrier();
  }
  };
  constexpr bool CAN_BE_TALL = (KIND == 0 && !P_RC);   // (tall tiles add rows to a K-contiguous P stage)
  if (CAN_BE_TALL && p_valid > TILE) run(std::integral_constant<int, CAN_BE_TALL ? 5 : 4>{});
  else if (KIND == 1 || p_valid > 128) run(std::integral_constant<int, 4>{});
  else if (p_valid > 64) run(std::integral_constant<int, 2>{});
  else run(std::integral_constant<int, 1>{});
}

// ---------------------------------------------------------------------------------------------------------
// Weight gradients as a persistent kernel: one block per CU takes tile after tile from a queue per XCD (the tile order
// and the 8 x 4 super-tiles are those described above), so that a tile's start-up -- the block launch and the
// latency of the first stage's loads, about 3 us against 16 k-steps of 1.8 us at an expert's 1000 rows, and against 5
// at 300 -- hides behind the previous tile's stores: the next tile's first stage is requested right after the last
// k-step, into stage 0, while the fp32 results bounce through stage 1 only.  (What it cannot hide: the first k-step's
// wait counts the stores as well, so it also waits for their acknowledgement, which a block that simply ends leaves to
// the next block's launch.)  Both operands R-contiguous, ragged K, one fp32 output tensor or the pair dW_gate | dW_up.
// Where the generic kernel's grid has no padding this one is 1-4 % slower; where it has, dW_down gained up to 22 % (the
// fine-grained workload's 0.72 -> 0.56 ms) and the pair 1-5 % (the Zipf shard's 0.92 -> 0.87 ms).
// ---------------------------------------------------------------------------------------------------------
struct WgradTile {
  int state;   // 0: nothing to do (padding of the super-tile grid, or no rows to add), 1: a tile, 2: the queue has run out
  int expert, k_len, p_row0, p_valid, q0_col, q_valid, p_tile_idx;
  size_t krow0;
};

template <int NQ>
__global__ __launch_bounds__(NTHREADS) void wgrad_persistent_kernel(const GemmArgs A) {
  __shared__ __attribute__((aligned(1024))) char stage0[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char stage1[STAGE_BYTES];
  __shared__ long long next_ticket;
  constexpr int TQ = TILE / NQ;
  constexpr int PB = 4;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wq = wave >> 1;
  const int late = wave >> 2;
  const int xcd = blockIdx.x % kNumXcd;
  const int sp = (A.n_p_tiles + 7) / 8, sq = (A.n_q_tiles + 3) / 4;
  const int supers_per_e = sp * sq;
  const long long n_super = (long long)supers_per_e * A.Et;
  const long long per_xcd = (n_super + kNumXcd - 1) / kNumXcd * kCusPerXcd;   // tickets of an XCD: 32 per super-tile

  auto decode = [&](long long within) __attribute__((always_inline)) -> WgradTile {
    WgradTile t = {};
    if (within >= per_xcd) { t.state = 2; return t; }
    const long long sid = (within >> 5) * kNumXcd + xcd;
    if (sid >= n_super) return t;
    t.expert = A.sched[64 + 2 * A.max_tiles + (int)(sid / supers_per_e)];   // the (sid / supers_per_e)-th largest expert
    const int super = (int)(sid % supers_per_e), in_super = (int)(within & 31);
    const int pt = (super % sp) * 8 + (in_super & 7);
    const int qt = (super / sp) * 4 + (in_super >> 3);
    if (pt >= A.n_p_tiles || qt >= A.n_q_tiles) return t;
    const int e_lo = A.offsets[t.expert], e_hi = A.offsets[t.expert + 1];
    t.k_len = e_hi - e_lo;
    if (t.k_len == 0 && A.accumulate) return t;
    t.krow0 = (size_t)e_lo;
    t.p_tile_idx = pt;
    t.p_row0 = pt * TILE;
    t.p_valid = min(TILE, A.p_dim - t.p_row0);
    t.q0_col = qt * TQ;
    t.q_valid = min(TQ, A.q_dim - t.q0_col);
    t.state = 1;
    return t;
  };
  // operands and per-lane load offsets of a tile, and this wavefront's 8 loads of its k-step j
  auto describe = [&](const WgradTile& t, TileOperand& P, TileOperand& Q, unsigned (&pvo)[4], unsigned (&qvo)[4], int& iwq)
                      __attribute__((always_inline)) {
    P.base0 = P.base1 = A.p0 + t.krow0 * A.p_ld + t.p_row0;
    P.ld = A.p_ld;
    P.r_valid = t.p_valid;
    Q.base0 = Q.base1 = A.q0 + t.krow0 * A.q_ld + t.q0_col;
    if (NQ == 2) Q.base1 = A.q1 + t.krow0 * A.q_ld + t.q0_col;
    Q.ld = A.q_ld;
    Q.r_valid = t.q_valid;
    iwq = wave ^ ((t.p_tile_idx & 1) << 2);   // (see ALTERNATE_Q in the kernel above)
#pragma unroll
    for (int i = 0; i < 4; i++) {
      pvo[i] = load_offset<true, false>(P, wave * 4 + i, lane);
      qvo[i] = load_offset<true, NQ == 2>(Q, iwq * 4 + i, lane);
    }
  };
  auto issue = [&](const TileOperand& P, const TileOperand& Q, const unsigned (&pvo)[4], const unsigned (&qvo)[4], int iwq, int k_len, int j,
                   char* stage) __attribute__((always_inline)) {
    issue_tile<true, false>(pvo, P, (ptrdiff_t)0, j * BK, k_len, A.zero_page, stage, wave, lane);
    issue_tile<true, NQ == 2>(qvo, Q, (ptrdiff_t)0, j * BK, k_len, A.zero_page, stage + Q_STAGE_OFFSET, iwq, lane);
  };

  const int qr0 = (NQ == 2) ? wq * 32 : wq * 64;
  const int qr1 = (NQ == 2) ? 128 + wq * 32 : wq * 64 + 32;
  const int wp = (wave & 1) * (PB * 32);
  constexpr int W = (NQ == 2) ? 32 : 64;       // q extent this wavefront owns per output tensor
  constexpr int PITCH = W * 4 + 16;            // bytes per staged fp32 row
  char* const wlds = stage1 + wave * (STAGE_BYTES / 8);   // this wavefront's 9 KB of stage 1: NQ tensors of 32 x PITCH bytes
  const int q_base = wq * W;

  unsigned p_off[PB], q_off[2];   // per-lane LDS offsets of this wavefront's fragments inside an operand area (kk = 0)
#pragma unroll
  for (int b = 0; b < PB; b++) p_off[b] = frag_offset<true>(wp + 32 * b, lane);
  q_off[0] = frag_offset<true>(qr0, lane);
  q_off[1] = frag_offset<true>(qr1, lane);

  WgradTile cur = decode(blockIdx.x / kNumXcd);   // the first tile of a block is its own index in its XCD
  bool first_stage_requested = false;
  // Whether the stores of the previous tile's epilogue were exactly 32 instructions per wavefront, issued
  // after the first stage's loads and with no other vector-memory instruction between them and the first k-step's wait.
  bool stores_behind_loads = false;
  // (32 = 4 p blocks x 8 row groups of one tensor, or x 4 row groups x 2 tensors)
  while (cur.state != 2) {
    // The ticket for the next tile is drawn now and not looked at before the k-steps are done: whoever needs the
    // value of an atomic waits for everything the wavefront has in flight, which here would be the previous tile's
    // stores and this tile's first stage.
    int my_draw;   // (thread 0 only; left undefined elsewhere on purpose: a defined value would be merged in, i.e. waited for, right here)
    if (tid == 0) {
      // (an address the compiler cannot prove wave-uniform: for a uniform one it rewrites the atomic into "one lane adds
      // the number of active lanes, the others derive theirs", which reads the result at once)
      int zero = 0;
      asm volatile("" : "+v"(zero));
      my_draw = atomicAdd(A.queue + xcd + zero, 1);
    }
    f32x16 acc[2][PB];
    if (cur.state == 1) {
      TileOperand P, Q;
      unsigned pvo[4], qvo[4];
      int iwq;
      describe(cur, P, Q, pvo, qvo, iwq);
      const int nk = (cur.k_len + BK - 1) / BK;
      if (!first_stage_requested && nk > 0) issue(P, Q, pvo, qvo, iwq, cur.k_len, 0, stage0);
#pragma unroll
      for (int a = 0; a < 2; a++)
#pragma unroll
        for (int b = 0; b < PB; b++)
#pragma unroll
          for (int v = 0; v < 16; v++) acc[a][b][v] = 0.f;
      auto k_step = [&](auto first_c, const char* stg, char* nxt, int kt) {
        // This thread's loads of step kt have landed.  The counter is in issue order, loads and stores alike: the first
        // stage was requested before the previous tile's stores, so after a full tile's epilogue "all but the
        // youngest 32" means the loads, and the stores drain while the tile's first step multiplies.
        if (decltype(first_c)::value && stores_behind_loads) __builtin_amdgcn_s_waitcnt(0x8F70);  // vmcnt(32)
        else __builtin_amdgcn_s_waitcnt(0x0F70);                                                   // vmcnt(0)
        __syncthreads();
        if (late && kt + 1 < nk) issue(P, Q, pvo, qvo, iwq, cur.k_len, kt + 1, nxt);
        const unsigned p_base = (unsigned)(size_t)(lptr_t)stg, q_base = p_base + Q_STAGE_OFFSET;
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
          if (kk == MOE_EARLY_ISSUE_AT) {
            __builtin_amdgcn_sched_barrier(0);
            if (!late && kt + 1 < nk) issue(P, Q, pvo, qvo, iwq, cur.k_len, kt + 1, nxt);
            __builtin_amdgcn_sched_barrier(0);
          }
          bf16x8 pf[PB], qf[2];
          qf[0] = read_frag_at<true>(q_off[0], kk, q_base);
          qf[1] = read_frag_at<true>(q_off[1], kk, q_base);
#pragma unroll
          for (int b = 0; b < PB; b++) pf[b] = read_frag_at<true>(p_off[b], kk, p_base);
#pragma unroll
          for (int b = 0; b < PB; b++)
#pragma unroll
            for (int a = 0; a < 2; a++)
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[a], pf[b], acc[a][b], 0, 0, 0);
        }
      };
      if (nk > 0) k_step(std::true_type{}, stage0, stage1, 0);
      for (int kt = 1; kt < nk; kt += 2) {
        k_step(std::false_type{}, stage1, stage0, kt);
        if (kt + 1 < nk) k_step(std::false_type{}, stage0, stage1, kt + 1);
      }
    }
    asm volatile("" : "+v"(my_draw));   // (nothing that needs the drawn value may move up across the k-steps)
    if (tid == 0) next_ticket = kCusPerXcd + (long long)my_draw;
    __syncthreads();   // every wavefront has finished reading the stages; the next ticket is visible
    const long long drawn = next_ticket;   // (the same for every lane: said so, which keeps the tile's description in scalar registers)
    const WgradTile nxt = decode(((long long)__builtin_amdgcn_readfirstlane((int)(drawn >> 32)) << 32) |
                                 (unsigned)__builtin_amdgcn_readfirstlane((int)drawn));
    first_stage_requested = false;
    if (nxt.state == 1 && nxt.k_len > 0) {
      TileOperand P, Q;
      unsigned pvo[4], qvo[4];
      int iwq;
      describe(nxt, P, Q, pvo, qvo, iwq);
      issue(P, Q, pvo, qvo, iwq, nxt.k_len, 0, stage0);
      first_stage_requested = true;
    }
    if (cur.state == 1) {
      // ---- epilogue (see the kernel above): 32 rows at a time through this wavefront's patch of stage 1
      // (the lane index as this part sees it: opaque, so that its address arithmetic is redone per tile instead of
      // being held in registers across the K loops)
      int elane = lane;
      asm volatile("" : "+v"(elane));
#pragma unroll
      for (int b = 0; b < PB; b++) {
#pragma unroll
        for (int a = 0; a < 2; a++)
#pragma unroll
          for (int v4 = 0; v4 < 4; v4++) {
            const int q = (NQ == 2 ? 0 : 32 * a) + 8 * v4 + 4 * (elane >> 5);
            float4 r = make_float4(acc[a][b][4 * v4], acc[a][b][4 * v4 + 1], acc[a][b][4 * v4 + 2], acc[a][b][4 * v4 + 3]);
            *reinterpret_cast<float4*>(wlds + (NQ == 2 ? a * (32 * PITCH) : 0) + (elane & 31) * PITCH + q * 4) = r;
          }
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wavefront's own LDS writes are done
        __builtin_amdgcn_wave_barrier();
        constexpr int LPR = W / 4;          // lanes per row (4 q = 16 bytes of fp32 per elane)
        constexpr int RPI = 64 / LPR;       // rows per instruction
#pragma unroll
        for (int it = 0; it < 32 / RPI; it++) {
          const int r = it * RPI + elane / LPR;
          const int q = (elane % LPR) * 4;
          const int p = wp + 32 * b + r;
          if (p < cur.p_valid && q_base + q < cur.q_valid) {
            const size_t o = (size_t)cur.expert * A.f_expert_stride + (size_t)(cur.p_row0 + p) * A.c_ld + cur.q0_col + q_base + q;
#pragma unroll
            for (int n = 0; n < NQ; n++) {
              float4 v = *reinterpret_cast<const float4*>(wlds + n * (32 * PITCH) + r * PITCH + q * 4);
              float* dst = (n == 0 ? A.f0 : A.f1) + o;
              if (A.accumulate) {
                const float4 old = *reinterpret_cast<const float4*>(dst);
                v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w;
              }
              *reinterpret_cast<float4*>(dst) = v;
            }
          }
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);  // the read-back is complete before the next 32 rows overwrite the patch
        __builtin_amdgcn_wave_barrier();
      }
    }
    stores_behind_loads = first_stage_requested && cur.state == 1 && !A.accumulate && cur.p_valid == TILE && cur.q_valid == TQ;
    __syncthreads();   // (the ticket slot may be rewritten)
    cur = nxt;
  }
}

// Row-tile schedule: one thread per expert.  sched[0] = number of row tiles; sched[1] = whether an expert's last tile
// may be a tall one; sched[64 + u] = expert of tile u;
// sched[64 + max_tiles + u] = index of that expert's first tile; sched[64 + 2 max_tiles + i] = expert with the i-th most rows.
// Also clears the zero page and the split-tile counters.
__global__ __launch_bounds__(1024) void build_schedule_kernel(const int32_t* __restrict__ offsets, int32_t* __restrict__ sched,
                                                              uint32_t* __restrict__ zero_page, int32_t* __restrict__ counters,
                                                              int Et, int max_tiles, int tall) {
  __shared__ int32_t scan[kMaxExperts];
  const int e = threadIdx.x;
  if (e < 64) zero_page[e] = 0u;
  if (e < kSplitCounters) counters[e] = 0;
  const int n = (e < Et) ? offsets[e + 1] - offsets[e] : 0;
  const int nt = row_tiles_of(n, tall);
  if (e == 0) sched[1] = tall;
  if (e >= 16 && e < 48) sched[e] = 0;   // tile queues of the weight-gradient launches that follow
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
  // experts by descending row count (ties: lower id first): sched[64 + 2 max_tiles + rank] = expert
  __shared__ int32_t rows_of[kMaxExperts];
  rows_of[e] = (e < Et) ? n : -1;
  __syncthreads();
  if (e < Et) {
    int rank = 0;
    for (int o = 0; o < Et; o++) rank += (rows_of[o] > n) || (rows_of[o] == n && o < e);
    sched[64 + 2 * max_tiles + rank] = e;
  }
  for (int i = 0; i < nt; i++) {
    if (first + i < max_tiles) {
      sched[64 + first + i] = e;
      sched[64 + max_tiles + first + i] = first;
    }
  }
}

// Blocks of a weight-gradient launch: whole rounds of one 32-tile super-tile per XCD.
static long long wgrad_blocks(int Et, int n_p_tiles, int n_q_tiles) {
  const long long n_super = (long long)Et * ((n_p_tiles + 7) / 8) * ((n_q_tiles + 3) / 4);
  return (n_super + kNumXcd - 1) / kNumXcd * kNumXcd * 32;
}

template <int KIND, bool P_RC, bool Q_RC, int NQ, int NPASS, int EPI>
static int launch_gemm(const char* label, const GemmArgs& A, long long max_blocks, hipStream_t st) {
  auto kern = grouped_gemm_kernel<KIND, P_RC, Q_RC, NQ, NPASS, EPI>;
  // bf16-output row-tile problems may cut the tiles of an XCD's last round into up to 32 parts in all
  const long long per_xcd = (max_blocks + kNumXcd - 1) / kNumXcd + ((KIND == 0 && NQ == 1) ? kCusPerXcd : 0);
  const long long grid = per_xcd * kNumXcd;
  if (max_blocks <= 0) return MOE_OK;
  MOE_LAUNCH(label, st, kern, dim3((unsigned)grid), dim3(NTHREADS), 0, st, A);
  return MOE_OK;
}

// Weight gradients.  The generic kernel, one block per tile; or, where the tiles do not fill whole 8 x 4 super-tiles
// (tiles along p not a multiple of 8 or along q not a multiple of 4: up to half of the generic kernel's blocks would
// then be padding that starts, looks up its tile and ends), one persistent block per CU (256) that takes its
// tiles from a queue per XCD, zeroed by the caller.
template <int NQ>
static int launch_wgrad(const char* label, const GemmArgs& A, hipStream_t st) {
  if (A.Et <= 0 || A.n_p_tiles <= 0 || A.n_q_tiles <= 0) return MOE_OK;
  const bool padded = (A.n_p_tiles % 8 != 0) || (A.n_q_tiles % 4 != 0);
  // (not the router's launch, which adds the two halves in the epilogue and has 16 tiles per part: 18 -> 32 us this way)
  if (!A.sum_halves && (MOE_WGRAD_PERSISTENT == 2 || (MOE_WGRAD_PERSISTENT == 1 && padded))) {
    MOE_LAUNCH(label, st, wgrad_persistent_kernel<NQ>, dim3(kNumXcd * kCusPerXcd), dim3(NTHREADS), 0, st, A);
    return MOE_OK;
  }
  return launch_gemm<1, true, true, NQ, 1, EPI_F32>(label, A, wgrad_blocks(A.Et, A.n_p_tiles, A.n_q_tiles), st);
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

#define MOE_TRY(call) do { int rc_ = (call); if (rc_ != MOE_OK) return rc_; } while (0)

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
  MOE_REQUIRE_PTR(y_perm);
  if ((save_g == nullptr) != (save_u == nullptr)) return MOE_ERR_NULL;  // kept together or not at all
  MOE_REQUIRE_ALIGNED(x_perm); MOE_REQUIRE_ALIGNED(offsets); MOE_REQUIRE_ALIGNED(w_gate); MOE_REQUIRE_ALIGNED(w_up);
  MOE_REQUIRE_ALIGNED(w_down); MOE_REQUIRE_ALIGNED(y_perm); MOE_REQUIRE_ALIGNED(save_g); MOE_REQUIRE_ALIGNED(save_u);
  if (D.N == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)stream;
  char* wsb = static_cast<char*>(ws);
  if (save_g == nullptr) {  // checkpointed forward: G and U go to the workspace and are not kept
    save_g = reinterpret_cast<uint16_t*>(wsb + L.g_re);
    save_u = reinterpret_cast<uint16_t*>(wsb + L.u_re);
  }
  int32_t* sched = reinterpret_cast<int32_t*>(wsb + L.sched);
  uint32_t* zero_page = reinterpret_cast<uint32_t*>(wsb + L.zero_page);
  int32_t* counters = reinterpret_cast<int32_t*>(wsb + L.splitk_counters);
  uint16_t* h = reinterpret_cast<uint16_t*>(wsb + L.h);
  const int max_tiles = (int)sched_max_tiles(D);
  const long long ub_tiles = D.N / TILE + D.Et;  // sum_e ceil(n_e/256) <= N/256 + E'
  MOE_LAUNCH("ffn_schedule", st, build_schedule_kernel, dim3(1), dim3(1024), 0, st, offsets, sched, zero_page, counters, D.Et, max_tiles, 1);

  GemmArgs A = {};
  A.sched = sched; A.max_tiles = max_tiles; A.offsets = offsets; A.Et = D.Et;
  A.zero_page = reinterpret_cast<const uint16_t*>(zero_page);
  A.partial = reinterpret_cast<float*>(wsb + L.splitk_partial); A.counters = counters;
  // G, U = X Wg, X Wu ; H = silu(G) * U
  A.n_q_tiles = (D.f + 127) / 128; A.q_dim = D.f; A.k_dim = D.d;
  A.p0 = x_perm; A.p_ld = D.d;
  A.q0 = w_gate; A.q1 = w_up; A.q_ld = D.f; A.q_expert_stride = (size_t)D.d * D.f;
  A.c0 = save_g; A.c1 = save_u; A.c2 = h; A.c_ld = D.f;
  MOE_TRY((launch_gemm<0, false, true, 2, 1, EPI_SWIGLU>("ffn_fwd_gate_up_swiglu", A, ub_tiles * A.n_q_tiles, st)));
  // Y = H Wd
  A.n_q_tiles = (D.d + TILE - 1) / TILE; A.q_dim = D.d; A.k_dim = D.f;
  A.p0 = h; A.p_ld = D.f;
  A.q0 = w_down; A.q1 = nullptr; A.q_ld = D.d; A.q_expert_stride = (size_t)D.f * D.d;
  A.c0 = y_perm; A.c1 = nullptr; A.c2 = nullptr; A.c_ld = D.d;
  MOE_TRY((launch_gemm<0, false, true, 1, 1, EPI_BF16>("ffn_fwd_down", A, ub_tiles * A.n_q_tiles, st)));
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
  uint32_t* zero_page = reinterpret_cast<uint32_t*>(wsb + L.zero_page);
  int32_t* counters = reinterpret_cast<int32_t*>(wsb + L.splitk_counters);
  uint16_t* h = reinterpret_cast<uint16_t*>(wsb + L.h);
  uint16_t* dg = reinterpret_cast<uint16_t*>(wsb + L.dg);
  uint16_t* du = reinterpret_cast<uint16_t*>(wsb + L.du);
  const int max_tiles = (int)sched_max_tiles(D);
  const long long ub_tiles = D.N / TILE + D.Et;

  GemmArgs A = {};
  A.sched = sched; A.max_tiles = max_tiles; A.offsets = offsets; A.Et = D.Et; A.accumulate = accumulate ? 1 : 0;
  A.zero_page = reinterpret_cast<const uint16_t*>(zero_page);
  A.partial = reinterpret_cast<float*>(wsb + L.splitk_partial); A.counters = counters;
  // (also with no rows at all: the weight gradients read the expert order from the schedule)
  MOE_LAUNCH("ffn_schedule", st, build_schedule_kernel, dim3(1), dim3(1024), 0, st, offsets, sched, zero_page, counters, D.Et, max_tiles, 1);
  if (D.N > 0) {
    // dH = dY Wd^T, then dG, dU and H from the saved G, U
    A.n_q_tiles = (D.f + TILE - 1) / TILE; A.q_dim = D.f; A.k_dim = D.d;
    A.p0 = dy_perm; A.p_ld = D.d;
    A.q0 = w_down; A.q_ld = D.d; A.q_expert_stride = (size_t)D.f * D.d;
    A.c0 = dg; A.c1 = du; A.c2 = h; A.c_ld = D.f; A.g_in = save_g; A.u_in = save_u;
    MOE_TRY((launch_gemm<0, false, false, 1, 1, EPI_DSWIGLU>("ffn_bwd_dh_dswiglu", A, ub_tiles * A.n_q_tiles, st)));
    // dX = dG Wg^T + dU Wu^T
    A.n_q_tiles = (D.d + TILE - 1) / TILE; A.q_dim = D.d; A.k_dim = D.f;
    A.p0 = dg; A.p1 = du; A.p_ld = D.f;
    A.q0 = w_gate; A.q1 = w_up; A.q_ld = D.f; A.q_expert_stride = (size_t)D.d * D.f;
    A.c0 = dx_perm; A.c1 = nullptr; A.c2 = nullptr; A.c_ld = D.d;
    MOE_TRY((launch_gemm<0, false, false, 1, 2, EPI_BF16>("ffn_bwd_dx", A, ub_tiles * A.n_q_tiles, st)));
  }
  // dWd[e] = H_e^T dY_e   (rows f, columns d)
  A.p_dim = D.f; A.n_p_tiles = (D.f + TILE - 1) / TILE; A.q_dim = D.d; A.n_q_tiles = (D.d + TILE - 1) / TILE;
  A.p0 = h; A.p1 = nullptr; A.p_ld = D.f;
  A.q0 = dy_perm; A.q1 = nullptr; A.q_ld = D.d;
  A.f0 = dw_down; A.f1 = nullptr; A.f_expert_stride = (size_t)D.f * D.d; A.c_ld = D.d;
  A.queue = sched + 16;
  MOE_TRY((launch_wgrad<1>("ffn_bwd_dw_down", A, st)));
  // dWg[e], dWu[e] = X_e^T dG_e, X_e^T dU_e   (rows d, columns f)
  A.p_dim = D.d; A.n_p_tiles = (D.d + TILE - 1) / TILE; A.q_dim = D.f; A.n_q_tiles = (D.f + 127) / 128;
  A.p0 = x_perm; A.p_ld = D.d;
  A.q0 = dg; A.q1 = du; A.q_ld = D.f;
  A.f0 = dw_gate; A.f1 = dw_up; A.f_expert_stride = (size_t)D.d * D.f; A.c_ld = D.f;
  A.queue = sched + 24;
  MOE_TRY((launch_wgrad<2>("ffn_bwd_dw_gate_up", A, st)));
  return launch_status();
}

extern "C" int moe_router_bwd(const moe_shape* shape, const uint16_t* x, const uint16_t* w_router, const float* dlogits,
                              uint16_t* dx_router, float* dw_router, int accumulate, void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  Dims D;
  WsLayout L;
  int rc = common_checks(shape, &D, ws, ws_bytes, &L);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(x); MOE_REQUIRE_PTR(w_router); MOE_REQUIRE_PTR(dlogits); MOE_REQUIRE_PTR(dx_router); MOE_REQUIRE_PTR(dw_router);
  MOE_REQUIRE_ALIGNED(x); MOE_REQUIRE_ALIGNED(w_router); MOE_REQUIRE_ALIGNED(dlogits); MOE_REQUIRE_ALIGNED(dx_router);
  MOE_REQUIRE_ALIGNED(dw_router);
  if (D.T == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)stream;
  char* wsb = static_cast<char*>(ws);
  int32_t* sched = reinterpret_cast<int32_t*>(wsb + L.sched);
  uint32_t* zero_page = reinterpret_cast<uint32_t*>(wsb + L.zero_page);
  int32_t* counters = reinterpret_cast<int32_t*>(wsb + L.splitk_counters);
  int32_t* offs = reinterpret_cast<int32_t*>(wsb + L.router_offsets);
  uint16_t* dl_hi = reinterpret_cast<uint16_t*>(wsb + L.dl_hi);
  uint16_t* dl_lo = reinterpret_cast<uint16_t*>(wsb + L.dl_lo);
  const int max_tiles = (int)sched_max_tiles(D);
  const int Epad = (int)round_up((size_t)D.E, 64);
  const bool skinny_dx = D.E <= 128;                          // (the dx kernel keeps W_r^T for 128 experts in registers)
  const int Ek = D.E <= 32 ? 32 : (D.E <= 64 ? 64 : 128);    // experts padded to the dx kernel's k-groups
  uint16_t* w_t = reinterpret_cast<uint16_t*>(wsb + L.w_router_t);
  float* partial = reinterpret_cast<float*>(wsb + L.router_dw_partial);
  // dW_r: the token range is cut into S parts, each a "segment" of the weight-gradient kernel with its own fp32 output
  // [d, ldp] in the workspace
  const int n_p_tiles = (int)((D.d + TILE - 1) / TILE), n_q_tiles = (int)((D.E + 127) / 128);
  const int ldp = (int)round_up((size_t)D.E, 4);
  const int S = router_dw_parts(D);
  const int part_rows = (int)round_up((size_t)((D.T + S - 1) / S), 64);
  launch_router_prepare(st, dlogits, w_router, dl_hi, dl_lo, skinny_dx ? w_t : nullptr, offs, sched + 64 + 2 * max_tiles, sched + 32, zero_page,
                        (int)D.T, (int)D.E, Epad, Ek, (int)D.d, (int)S, part_rows);
  GemmArgs A = {};
  A.sched = sched; A.max_tiles = max_tiles; A.Et = 1; A.accumulate = 0;
  A.zero_page = reinterpret_cast<const uint16_t*>(zero_page);
  A.partial = reinterpret_cast<float*>(wsb + L.splitk_partial); A.counters = counters;
  if (skinny_dx) {
    launch_router_bwd_dx(st, dl_hi, dl_lo, w_t, dx_router, (int)D.T, (int)D.d, (int)D.E, Epad);
  } else {
    // dx_router[T,d] = dlogits W_r on the grouped GEMM kernel: rows = tokens, columns = d, K = E in two passes (head,
    // remainder of dlogits); P K-contiguous in the padded copies, Q = W_r read with k = expert row (R-contiguous)
    MOE_LAUNCH("router_schedule", st, build_schedule_kernel, dim3(1), dim3(1024), 0, st, offs, sched, zero_page, counters, 1, max_tiles, 0);
    A.offsets = offs;
    A.n_q_tiles = (D.d + TILE - 1) / TILE; A.q_dim = D.d; A.k_dim = D.E;
    A.p0 = dl_hi; A.p1 = dl_lo; A.p_ld = Epad;
    A.q0 = w_router; A.q1 = w_router; A.q_ld = D.d; A.q_expert_stride = 0;
    A.c0 = dx_router; A.c_ld = D.d;
    const long long row_tiles = (D.T + TILE - 1) / TILE;
    MOE_TRY((launch_gemm<0, false, true, 1, 2, EPI_BF16>("router_bwd_dx", A, row_tiles * A.n_q_tiles, st)));
  }
  // dW_r^T[c, e] per part = X_part^T dlogits_part: the weight-gradient kernel with p = columns of x, q = experts (the
  // head and the remainder of dlogits as the two halves of the q tile, their results added in the epilogue), k = the
  // part's tokens; then the parts are added in order and transposed into dW_r.  (The segment order and the zero page
  // that this kernel reads of a schedule were written by the prepare kernel; a dx launch above leaves them as they are.)
  GemmArgs B = {};
  B.sched = sched; B.max_tiles = max_tiles; B.offsets = offs + 8; B.Et = (int)S; B.accumulate = 0;
  B.zero_page = reinterpret_cast<const uint16_t*>(zero_page);
  B.p_dim = D.d; B.n_p_tiles = n_p_tiles; B.q_dim = D.E; B.n_q_tiles = n_q_tiles;
  B.p0 = x; B.p_ld = D.d;
  B.q0 = dl_hi; B.q1 = dl_lo; B.q_ld = Epad;
  B.f0 = partial; B.f1 = nullptr; B.f_expert_stride = (size_t)D.d * ldp; B.c_ld = ldp; B.sum_halves = 1;
  B.queue = sched + 32;
  MOE_TRY((launch_wgrad<2>("router_bwd_dw", B, st)));
  launch_router_dw_reduce(st, partial, dw_router, (int)S, (int)D.E, (int)D.d, ldp, accumulate ? 1 : 0);
  return launch_status();
}

extern "C" int moe_grouped_ffn_bwd_recompute(const moe_shape* shape, const uint16_t* dy_perm, const uint16_t* x_perm,
                                             const int32_t* offsets, const uint16_t* w_gate, const uint16_t* w_up,
                                             const uint16_t* w_down, uint16_t* dx_perm, float* dw_gate, float* dw_up,
                                             float* dw_down, int accumulate, void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  Dims D;
  WsLayout L;
  int rc = common_checks(shape, &D, ws, ws_bytes, &L);
  if (rc != MOE_OK) return rc;
  // every argument is checked before the first launch (the call below checks them again)
  MOE_REQUIRE_PTR(dy_perm); MOE_REQUIRE_PTR(x_perm); MOE_REQUIRE_PTR(offsets); MOE_REQUIRE_PTR(w_gate); MOE_REQUIRE_PTR(w_up);
  MOE_REQUIRE_PTR(w_down); MOE_REQUIRE_PTR(dx_perm); MOE_REQUIRE_PTR(dw_gate); MOE_REQUIRE_PTR(dw_up); MOE_REQUIRE_PTR(dw_down);
  MOE_REQUIRE_ALIGNED(dy_perm); MOE_REQUIRE_ALIGNED(x_perm); MOE_REQUIRE_ALIGNED(offsets); MOE_REQUIRE_ALIGNED(w_gate);
  MOE_REQUIRE_ALIGNED(w_up); MOE_REQUIRE_ALIGNED(w_down); MOE_REQUIRE_ALIGNED(dx_perm); MOE_REQUIRE_ALIGNED(dw_gate);
  MOE_REQUIRE_ALIGNED(dw_up); MOE_REQUIRE_ALIGNED(dw_down);
  char* wsb = static_cast<char*>(ws);
  uint16_t* g_re = reinterpret_cast<uint16_t*>(wsb + L.g_re);
  uint16_t* u_re = reinterpret_cast<uint16_t*>(wsb + L.u_re);
  if (D.N > 0) {
    // G, U = X Wg, X Wu once more (the same kernel as in forward, hence the same bits); its H output is overwritten
    // by the backward's own
    hipStream_t st = (hipStream_t)stream;
    int32_t* sched = reinterpret_cast<int32_t*>(wsb + L.sched);
    uint32_t* zero_page = reinterpret_cast<uint32_t*>(wsb + L.zero_page);
    int32_t* counters = reinterpret_cast<int32_t*>(wsb + L.splitk_counters);
    const int max_tiles = (int)sched_max_tiles(D);
    const long long ub_tiles = D.N / TILE + D.Et;
    MOE_LAUNCH("ffn_schedule", st, build_schedule_kernel, dim3(1), dim3(1024), 0, st, offsets, sched, zero_page, counters, D.Et, max_tiles, 1);
    GemmArgs A = {};
    A.sched = sched; A.max_tiles = max_tiles; A.offsets = offsets; A.Et = D.Et;
    A.zero_page = reinterpret_cast<const uint16_t*>(zero_page);
    A.partial = reinterpret_cast<float*>(wsb + L.splitk_partial); A.counters = counters;
    A.n_q_tiles = (D.f + 127) / 128; A.q_dim = D.f; A.k_dim = D.d;
    A.p0 = x_perm; A.p_ld = D.d;
    A.q0 = w_gate; A.q1 = w_up; A.q_ld = D.f; A.q_expert_stride = (size_t)D.d * D.f;
    A.c0 = g_re; A.c1 = u_re; A.c2 = reinterpret_cast<uint16_t*>(wsb + L.h); A.c_ld = D.f;
    MOE_TRY((launch_gemm<0, false, true, 2, 1, EPI_SWIGLU>("ffn_bwd_recompute_gate_up", A, ub_tiles * A.n_q_tiles, st)));
  }
  return moe_grouped_ffn_bwd(shape, dy_perm, x_perm, offsets, w_gate, w_up, w_down, g_re, u_re, dx_perm, dw_gate, dw_up, dw_down,
                             accumulate, ws, ws_bytes, stream);
}
