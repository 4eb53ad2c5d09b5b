// The steps of the hierarchical all-to-all (Section V, Algorithm 1) that touch only one GPU's memory: the pack of the
// rows bound for other nodes (phase 2), the (M, R, D) -> (R, M D) repack between the inter-node and the second
// intra-node exchange (phase 3), and the final placement of both results in the output buffer.  All three move
// whole rows of `row_bytes` bytes from a computed source row to a computed destination row, so they are one
// HBM-bound copy kernel with three row maps.  The exchanges themselves are not part of this library.
#include "common.h"

namespace moe {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

enum HaloMap { HALO_PACK = 0, HALO_REPACK = 1, HALO_UNPACK = 2 };

struct HaloArgs {
  const u32x4* src0;   // S (pack), F2r (repack), P1 (unpack)
  const u32x4* src1;   // F3r (unpack only)
  u32x4* dst;
  int num_nodes, R, M, node_id;
  long long out_rows;
  unsigned vec_per_row;  // row_bytes / 16
};

// Source of output row `o` (an index into src0 or, when *second, src1; rows of vec_per_row vectors each).
template <int MAP>
__device__ __forceinline__ long long halo_source_row(const HaloArgs& a, long long o, bool* second) {
  *second = false;
  if (MAP == HALO_PACK) {          // F2s[i R + r] = S[n_i R + r], n_i = the i-th node other than node_id
    const long long i = o / a.R, r = o % a.R;
    const long long n = i < a.node_id ? i : i + 1;
    return n * a.R + r;
  } else if (MAP == HALO_REPACK) {  // F3s[r][i] = F2r[i R + r]   (output row index o = r M + i)
    const long long r = o / a.M, i = o % a.M;
    return i * a.R + r;
  } else {                          // O[node_id R + r] = P1[r];  O[n_i R + p] = F3r[p][i]  (source row index p M + i)
    const long long n = o / a.R, p = o % a.R;
    if (n == a.node_id) return p;
    *second = true;
    const long long i = n < a.node_id ? n : n - 1;
    return p * a.M + i;
  }
}

template <int MAP>
__global__ __launch_bounds__(256) void halo_rows_kernel(const HaloArgs a) {
  constexpr int U = 4;  // 16-byte vectors per thread in flight
  const long long total = a.out_rows * a.vec_per_row;
  const long long stride = (long long)gridDim.x * 256;
  for (long long v0 = (long long)blockIdx.x * 256 + threadIdx.x; v0 < total; v0 += stride * U) {
    u32x4 val[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
      const long long v = v0 + u * stride;
      if (v < total) {
        bool second;
        const long long o = v / a.vec_per_row, c = v % a.vec_per_row;
        const long long s = halo_source_row<MAP>(a, o, &second);
        val[u] = __builtin_nontemporal_load((second ? a.src1 : a.src0) + s * a.vec_per_row + c);
      }
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
      const long long v = v0 + u * stride;
      if (v < total) __builtin_nontemporal_store(val[u], a.dst + v);
    }
  }
}

static int halo_checks(int num_nodes, int R, size_t row_bytes, int node_id) {
  if (num_nodes < 1 || R < 1 || node_id < 0 || node_id >= num_nodes) return MOE_ERR_SHAPE;
  if (row_bytes == 0 || row_bytes % 16 || row_bytes / 16 > 0xFFFFFFFFull) return MOE_ERR_SHAPE;
  if ((long long)num_nodes * R > (1LL << 24)) return MOE_ERR_SHAPE;
  return MOE_OK;
}

template <int MAP>
static int halo_launch(const char* label, const HaloArgs& a, hipStream_t st) {
  const long long total = a.out_rows * a.vec_per_row;
  if (total == 0) return MOE_OK;
  long long blocks = (total + 256 * 4 - 1) / (256 * 4);
  if (blocks > 256 * 16) blocks = 256 * 16;  // grid-stride beyond 16 blocks per CU
  MOE_LAUNCH(label, st, halo_rows_kernel<MAP>, dim3((unsigned)blocks), dim3(256), 0, st, a);
  return launch_status();
}

}  // namespace moe

extern "C" int moe_halo_pack_remote(const void* S, void* F2s, int num_nodes, int R, size_t row_bytes, int node_id, void* stream) {
  using namespace moe;
  int rc = halo_checks(num_nodes, R, row_bytes, node_id);
  if (rc != MOE_OK) return rc;
  if (num_nodes == 1) return MOE_OK;  // no remote node: nothing to pack
  MOE_REQUIRE_PTR(S); MOE_REQUIRE_PTR(F2s);
  MOE_REQUIRE_ALIGNED(S); MOE_REQUIRE_ALIGNED(F2s);
  HaloArgs a = {};
  a.src0 = static_cast<const u32x4*>(S); a.dst = static_cast<u32x4*>(F2s);
  a.num_nodes = num_nodes; a.R = R; a.M = num_nodes - 1; a.node_id = node_id;
  a.out_rows = (long long)(num_nodes - 1) * R; a.vec_per_row = (unsigned)(row_bytes / 16);
  return halo_launch<HALO_PACK>("halo_pack_remote", a, (hipStream_t)stream);
}

extern "C" int moe_halo_repack(const void* F2r, void* F3s, int M, int R, size_t row_bytes, void* stream) {
  using namespace moe;
  int rc = halo_checks(M + 1, R, row_bytes, 0);
  if (rc != MOE_OK) return rc;
  if (M == 0) return MOE_OK;
  MOE_REQUIRE_PTR(F2r); MOE_REQUIRE_PTR(F3s);
  MOE_REQUIRE_ALIGNED(F2r); MOE_REQUIRE_ALIGNED(F3s);
  HaloArgs a = {};
  a.src0 = static_cast<const u32x4*>(F2r); a.dst = static_cast<u32x4*>(F3s);
  a.num_nodes = M + 1; a.R = R; a.M = M; a.node_id = 0;
  a.out_rows = (long long)M * R; a.vec_per_row = (unsigned)(row_bytes / 16);
  return halo_launch<HALO_REPACK>("halo_repack", a, (hipStream_t)stream);
}

extern "C" int moe_halo_unpack(const void* P1, const void* F3r, void* O, int num_nodes, int R, size_t row_bytes, int node_id,
                               void* stream) {
  using namespace moe;
  int rc = halo_checks(num_nodes, R, row_bytes, node_id);
  if (rc != MOE_OK) return rc;
  MOE_REQUIRE_PTR(P1); MOE_REQUIRE_PTR(O);
  MOE_REQUIRE_ALIGNED(P1); MOE_REQUIRE_ALIGNED(O);
  if (num_nodes > 1) { MOE_REQUIRE_PTR(F3r); MOE_REQUIRE_ALIGNED(F3r); }
  HaloArgs a = {};
  a.src0 = static_cast<const u32x4*>(P1); a.src1 = static_cast<const u32x4*>(F3r); a.dst = static_cast<u32x4*>(O);
  a.num_nodes = num_nodes; a.R = R; a.M = num_nodes - 1; a.node_id = node_id;
  a.out_rows = (long long)num_nodes * R; a.vec_per_row = (unsigned)(row_bytes / 16);
  return halo_launch<HALO_UNPACK>("halo_unpack", a, (hipStream_t)stream);
}
