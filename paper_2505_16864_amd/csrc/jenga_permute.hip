// Eq. 2 of the paper as a data-movement kernel: curve-order gather fused with the change from the
// token-major thw-side layout to the head-major curve-side layout, and its inverse.
//
// HBM-bound.  One (token, head) row is head_dim*2 bytes (256 B at d=128) and is moved as 16-byte
// pieces by a group of lanes; a workgroup covers 256/chunks consecutive curve positions, so for one
// head it touches one contiguous span on the curve side, while on the thw side each lane group
// walks the contiguous heads of its token.
#include <hip/hip_runtime.h>

#include "jenga_internal.h"

namespace {

template <bool FORWARD>
__global__ __launch_bounds__(256) void permute_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                      const int32_t* __restrict__ src_of_pos, int n_src,
                                                      int n_pad, int heads, int chunks, int heads_per_wg) {
  const int groups = 256 / chunks;
  const int c = threadIdx.x % chunks;
  const int g = threadIdx.x / chunks;
  const int i = blockIdx.x * groups + g;
  if (i >= n_pad) return;
  const int b = blockIdx.z;
  const int h0 = blockIdx.y * heads_per_wg;
  const int h1 = min(h0 + heads_per_wg, heads);
  const int s = src_of_pos[i];
  if (FORWARD) {
    const uint4 zero = make_uint4(0, 0, 0, 0);
    const uint4* in = src + (((size_t)b * n_src + (s >= 0 ? s : 0)) * heads) * chunks + c;
    uint4* o = dst + (((size_t)b * heads) * n_pad + i) * chunks + c;
    int h = h0;
    for (; h + 4 <= h1; h += 4) {
      uint4 v0 = zero, v1 = zero, v2 = zero, v3 = zero;
      if (s >= 0) {
        v0 = in[(size_t)(h + 0) * chunks];
        v1 = in[(size_t)(h + 1) * chunks];
        v2 = in[(size_t)(h + 2) * chunks];
        v3 = in[(size_t)(h + 3) * chunks];
      }
      o[(size_t)(h + 0) * n_pad * chunks] = v0;
      o[(size_t)(h + 1) * n_pad * chunks] = v1;
      o[(size_t)(h + 2) * n_pad * chunks] = v2;
      o[(size_t)(h + 3) * n_pad * chunks] = v3;
    }
    for (; h < h1; ++h) {
      uint4 v = zero;
      if (s >= 0) v = in[(size_t)h * chunks];
      o[(size_t)h * n_pad * chunks] = v;
    }
  } else {
    if (s < 0) return;
    const uint4* in = src + (((size_t)b * heads) * n_pad + i) * chunks + c;
    uint4* o = dst + (((size_t)b * n_src + s) * heads) * chunks + c;
    int h = h0;
    for (; h + 4 <= h1; h += 4) {
      const uint4 v0 = in[(size_t)(h + 0) * n_pad * chunks];
      const uint4 v1 = in[(size_t)(h + 1) * n_pad * chunks];
      const uint4 v2 = in[(size_t)(h + 2) * n_pad * chunks];
      const uint4 v3 = in[(size_t)(h + 3) * n_pad * chunks];
      o[(size_t)(h + 0) * chunks] = v0;
      o[(size_t)(h + 1) * chunks] = v1;
      o[(size_t)(h + 2) * chunks] = v2;
      o[(size_t)(h + 3) * chunks] = v3;
    }
    for (; h < h1; ++h) o[(size_t)h * chunks] = in[(size_t)h * n_pad * chunks];
  }
}

}  // namespace

namespace jenga {

int launch_permute(const jenga_plan* p, const void* src, void* dst, bool forward, void* stream) {
  const jenga_config& c = p->cfg;
  const int chunks = c.head_dim * 2 / 16;
  const int groups = 256 / chunks;
  const int heads_per_wg = 8;
  dim3 grid((p->info.N_pad + groups - 1) / groups, (c.heads + heads_per_wg - 1) / heads_per_wg, c.batch);
  const int n_src = p->info.N_v + c.n_text;
  hipStream_t st = (hipStream_t)stream;
  if (forward)
    permute_kernel<true><<<grid, 256, 0, st>>>((const uint4*)src, (uint4*)dst, p->d_src_of_pos, n_src,
                                               p->info.N_pad, c.heads, chunks, heads_per_wg);
  else
    permute_kernel<false><<<grid, 256, 0, st>>>((const uint4*)src, (uint4*)dst, p->d_src_of_pos, n_src,
                                                p->info.N_pad, c.heads, chunks, heads_per_wg);
  return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_EHIP;
}

int launch_permute_rows(const jenga_plan* p, const void* src, void* dst, int row_bytes, void* stream) {
  // a per-token table is the one-head, one-batch case of the same kernel with a row of row_bytes/16 pieces
  const int chunks = row_bytes / 16;
  const int groups = 256 / chunks;
  dim3 grid((p->info.N_pad + groups - 1) / groups, 1, 1);
  permute_kernel<true><<<grid, 256, 0, (hipStream_t)stream>>>((const uint4*)src, (uint4*)dst, p->d_src_of_pos,
                                                              p->info.N_v + p->cfg.n_text, p->info.N_pad, 1, chunks, 1);
  return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_EHIP;
}

}  // namespace jenga
