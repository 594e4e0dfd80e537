// Block selection (Sec. 3.1 Eq. 3; appendix Alg. 3 and Eq. 5) in three kernels:
//   pool_kernel    BlockPool: per-block mean of Q (vision blocks) and K (all blocks)   HBM-bound
//   scores_kernel  S = Q^ K^T / sqrt(d_k), a small float64 GEMM per (batch, head)       ALU-bound
//   select_kernel  one wavefront per query block: softmax, N_k, top-N_k, union, compaction
//
// All arithmetic is float64: the outcome is a set of integers, and in float64 the sums of bf16
// inputs are exact and the remaining rounding (1e-16 relative) is far below the spacing of the
// block probabilities, so the sets do not depend on the order of summation.
//
// select_kernel keeps a row of R in registers (NT values per lane) and never sorts.  Positive
// doubles order like their bit patterns, so the N-th largest value is found by building its bit
// pattern from the top bit down, counting with wave ballots; the cumulative-probability rule uses
// the same descent on the sum of the values at or above the candidate.
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>

#include "jenga_internal.h"

// Workspace of jenga_select_blocks_static: one copy per GPU, held from module load to process end.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)JENGA_SELECT_STATIC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

__device__ inline double bf16_bits_to_double(uint32_t bits16) {
  return (double)__uint_as_float(bits16 << 16);
}

__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ inline double wave_max(double v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
  return v;
}

// grid (M, batch*heads, 2): z = 0 pools Q (vision blocks only), z = 1 pools K (all blocks).
// q, k: curve side [bh][n_pad][D]; qh: [bh][M_v][D]; kh: [bh][M][D].  A thread issues up to four row
// loads before it adds them, so that enough bytes are in flight to stream from HBM.
template <int D>
__global__ __launch_bounds__(256) void pool_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                   double* __restrict__ qh, double* __restrict__ kh,
                                                   const int32_t* __restrict__ blk_valid, int n_pad, int m, int M_v,
                                                   int M) {
  constexpr int CH = D / 8;      // 16-byte chunks per row
  constexpr int G = 256 / CH;    // rows in flight per pass
  __shared__ double red[G][D];
  const int j = blockIdx.x, bh = blockIdx.y;
  const bool is_q = blockIdx.z == 0;
  if (is_q && j >= M_v) return;
  const uint16_t* x = is_q ? q : k;
  double* out = is_q ? qh : kh;
  const int n_blk = is_q ? M_v : M;
  const int c = threadIdx.x % CH, g = threadIdx.x / CH;
  const int nv = blk_valid[j];
  double acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.0;
  const uint4* base = (const uint4*)(x + ((size_t)bh * n_pad + (size_t)j * m) * D);
  for (int r0 = g; r0 < nv; r0 += 4 * G) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = r0 + u * G;
      v[u] = r < nv ? base[(size_t)r * CH + c] : make_uint4(0, 0, 0, 0);   // +0.0 for the rows past the end
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] += bf16_bits_to_double(w[e] & 0xFFFFu);
        acc[2 * e + 1] += bf16_bits_to_double(w[e] >> 16);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[g][c * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    double s = 0.0;
#pragma unroll
    for (int gg = 0; gg < G; ++gg) s += red[gg][threadIdx.x];
    out[((size_t)bh * n_blk + j) * D + threadIdx.x] = s / (double)nv;
  }
}

// S[bh][i][j] = sum_d qh[bh][i][d] * kh[bh][j][d] / sqrt(D).  128 x 128 tile per workgroup, 8 x 8 per
// thread with rows ty + 16 r and columns tx + 16 c: the 16 lanes that differ in tx read consecutive
// doubles of a K^ row slice (no bank conflicts) and share one address of the Q^ slice (broadcast),
// and 64 FMAs stand against 16 LDS reads.
template <int D>
__global__ __launch_bounds__(256) void scores_kernel(const double* __restrict__ qh, const double* __restrict__ kh,
                                                     double* __restrict__ S, int M_v, int M) {
  constexpr int DC = 8, T = 128;
  __shared__ double As[DC][T];
  __shared__ double Bs[DC][T];
  const int bh = blockIdx.z;
  const int i0 = blockIdx.y * T, j0 = blockIdx.x * T;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int lr = threadIdx.x / 2, ld = (threadIdx.x % 2) * 4;   // loader: row of the tile, first of 4 d's
  const double* qa = qh + ((size_t)bh * M_v + min(i0 + lr, M_v - 1)) * D + ld;
  const double* kb = kh + ((size_t)bh * M + min(j0 + lr, M - 1)) * D + ld;
  double acc[8][8];
#pragma unroll
  for (int r = 0; r < 8; ++r)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[r][c] = 0.0;
  for (int d0 = 0; d0 < D; d0 += DC) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      As[ld + e][lr] = qa[d0 + e];
      Bs[ld + e][lr] = kb[d0 + e];
    }
    __syncthreads();
#pragma unroll
    for (int dd = 0; dd < DC; ++dd) {
      double a[8], b[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) a[r] = As[dd][ty + 16 * r];
#pragma unroll
      for (int c = 0; c < 8; ++c) b[c] = Bs[dd][tx + 16 * c];
#pragma unroll
      for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[r][c] = fma(a[r], b[c], acc[r][c]);
    }
    __syncthreads();
  }
  const double inv = 1.0 / sqrt((double)D);
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int i = i0 + ty + 16 * r;
    if (i >= M_v) continue;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int j = j0 + tx + 16 * c;
      if (j < M) S[((size_t)bh * M_v + i) * M + j] = acc[r][c] * inv;
    }
  }
}

// One wavefront per (batch, head, query block).  NT = values per lane, M <= 64*NT.
template <int NT>
__global__ __launch_bounds__(256) void select_kernel(const double* __restrict__ S,
                                                     const uint64_t* __restrict__ fixed_bits,
                                                     int32_t* __restrict__ sel_count, int32_t* __restrict__ sel_index,
                                                     uint8_t* __restrict__ mask, int M_v, int M, int n_rows,
                                                     int K_top, double p, int nt64) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const int bh = row / M, i = row % M;
  int32_t* idx_out = sel_index + (size_t)row * M;
  uint8_t* mask_out = mask ? mask + (size_t)row * M : nullptr;
  const uint64_t lt_mask = (1ull << lane) - 1ull;

  if (i >= M_v) {   // text query block: sees every block (Alg. 2)
    for (int j = lane; j < M; j += 64) {
      idx_out[j] = j;
      if (mask_out) mask_out[j] = 1;
    }
    if (lane == 0) sel_count[row] = M;
    return;
  }

  const double* srow = S + ((size_t)bh * M_v + i) * M;
  double r[NT];
  double mx = -INFINITY;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int j = t * 64 + lane;
    r[t] = j < M ? srow[j] : -INFINITY;
    mx = fmax(mx, r[t]);
  }
  mx = wave_max(mx);
  double z = 0.0;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int j = t * 64 + lane;
    r[t] = j < M ? exp(r[t] - mx) : 0.0;
    z += r[t];
  }
  z = wave_sum(z);
  uint64_t key[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    r[t] = r[t] / z;
    key[t] = (uint64_t)__double_as_longlong(r[t]);   // R >= 0: bit order is value order
  }

  // value of the K_top-th largest: largest pattern with count(key >= pattern) >= K_top
  // The descent stops as soon as exactly K_top values lie at or above the pattern built so far: that set is the
  // answer whatever the remaining bits are (typically after 20-25 of the 63 bits).
  uint64_t tau_k = 0;
  for (int bit = 62; bit >= 0; --bit) {
    const uint64_t cand = tau_k | (1ull << bit);
    int cnt = 0;
#pragma unroll
    for (int t = 0; t < NT; ++t) cnt += __popcll(__ballot(key[t] >= cand));
    if (cnt >= K_top) {
      tau_k = cand;
      if (cnt == K_top) break;
    }
  }
  int cnt_gt = 0;
  double sum_gt = 0.0;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const bool gt = key[t] > tau_k;
    cnt_gt += __popcll(__ballot(gt));
    sum_gt += gt ? r[t] : 0.0;
  }
  sum_gt = wave_sum(sum_gt);
  const double topk_mass = sum_gt + (double)(K_top - cnt_gt) * __longlong_as_double((long long)tau_k);

  uint64_t tau = tau_k;
  int n_keep = K_top;
  if (!(topk_mass > p)) {
    // cumulative-probability rule: largest pattern whose upper set still sums to more than p
    // The answer is one of the row's values.  After bit b it lies in [tau_p, tau_p + 2^b); once that interval
    // holds a single value, that value is the answer and the remaining bits are its bits.
    uint64_t tau_p = 0;
    for (int bit = 62; bit >= 0; --bit) {
      const uint64_t cand = tau_p | (1ull << bit);
      double f = 0.0;
#pragma unroll
      for (int t = 0; t < NT; ++t) f += key[t] >= cand ? r[t] : 0.0;
      f = wave_sum(f);
      if (f > p) tau_p = cand;
      const uint64_t hi = tau_p + (1ull << bit);     // exclusive end of the interval that still holds the answer
      int inside = 0;
      uint64_t mine = 0;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const bool in = key[t] >= tau_p && key[t] < hi;
        inside += __popcll(__ballot(in));
        if (in) mine = key[t];
      }
      if (inside == 1) {
        const uint64_t who = __ballot(mine != 0);
        const int src = __builtin_ctzll(who);
        const uint32_t lo32 = __builtin_amdgcn_readlane((uint32_t)mine, src);
        const uint32_t hi32 = __builtin_amdgcn_readlane((uint32_t)(mine >> 32), src);
        tau_p = ((uint64_t)hi32 << 32) | lo32;
        break;
      }
    }
    int g_cnt = 0, e_cnt = 0;
    double g_sum = 0.0;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const bool valid = t * 64 + lane < M;
      const bool gt = key[t] > tau_p;
      g_cnt += __popcll(__ballot(gt));
      e_cnt += __popcll(__ballot(valid && key[t] == tau_p));
      g_sum += gt ? r[t] : 0.0;
    }
    g_sum = wave_sum(g_sum);
    const double tv = __longlong_as_double((long long)tau_p);
    int tn = 1;
    while (tn < e_cnt && !(g_sum + (double)tn * tv > p)) ++tn;
    const int n_star = g_cnt + tn;
    if (n_star > K_top) {
      n_keep = n_star;
      tau = tau_p;
      cnt_gt = g_cnt;
    }
  }
  n_keep = min(n_keep, M);
  const int need = n_keep - cnt_gt;   // taken from the values equal to tau, lowest index first

  int taken = 0, out_pos = 0;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int j = t * 64 + lane;
    const bool valid = j < M;
    const bool eq = valid && key[t] == tau;
    const uint64_t eq_mask = __ballot(eq);
    bool sel = (valid && key[t] > tau) || (eq && taken + (int)__popcll(eq_mask & lt_mask) < need);
    taken += (int)__popcll(eq_mask);
    if (t < nt64) sel = sel || ((fixed_bits[(size_t)i * nt64 + t] >> lane) & 1ull);
    sel = sel && valid;
    const uint64_t sel_mask = __ballot(sel);
    if (sel) idx_out[out_pos + __popcll(sel_mask & lt_mask)] = j;
    out_pos += __popcll(sel_mask);
    if (mask_out && valid) mask_out[j] = sel ? 1 : 0;
  }
  if (lane == 0) sel_count[row] = out_pos;
}

template <int D>
int run_select(const jenga_plan* p, const void* q, const void* k, int32_t* sel_count, int32_t* sel_index,
               uint8_t* mask, void* ws, hipStream_t st) {
  const jenga_config& c = p->cfg;
  const jenga_plan_info_t& f = p->info;
  const int bh = c.batch * c.heads;
  auto align256 = [](size_t x) { return (x + 255) & ~(size_t)255; };
  char* w = (char*)ws;
  double* qh = (double*)w;
  w += align256((size_t)bh * f.M_v * D * 8);
  double* kh = (double*)w;
  w += align256((size_t)bh * f.M * D * 8);
  double* S = (double*)w;
  if (f.M_v > 0) {
    pool_kernel<D><<<dim3(f.M, bh, 2), 256, 0, st>>>((const uint16_t*)q, (const uint16_t*)k, qh, kh, p->d_blk_valid,
                                                    f.N_pad, c.block, f.M_v, f.M);
    scores_kernel<D><<<dim3((f.M + 127) / 128, (f.M_v + 127) / 128, bh), 256, 0, st>>>(qh, kh, S, f.M_v, f.M);
  }
  const int n_rows = bh * f.M;
  const dim3 grid((n_rows + 3) / 4);
#define JENGA_SELECT(NTV)                                                                                      \
  select_kernel<NTV><<<grid, 256, 0, st>>>(S, p->d_fixed_bits, sel_count, sel_index, mask, f.M_v, f.M, n_rows, \
                                           f.K_top, c.cum_prob, p->nt64)
  if (p->nt64 <= 1) JENGA_SELECT(1);
  else if (p->nt64 <= 2) JENGA_SELECT(2);
  else if (p->nt64 <= 4) JENGA_SELECT(4);
  else if (p->nt64 <= 8) JENGA_SELECT(8);
  else if (p->nt64 <= 16) JENGA_SELECT(16);
  else JENGA_SELECT(32);
#undef JENGA_SELECT
  return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_EHIP;
}

// ---- scratch of the allocation-free entry point ------------------------------------------------
// One array per GPU, resident from module load until the process ends.  The name below is only a
// host-side handle: device code and HIP calls get the address hipGetSymbolAddress returns for the
// device that is current, looked up once per device and kept here.
constexpr int MAX_DEVICES = 64;
void* scratch_of_device[MAX_DEVICES] = {};
std::mutex scratch_lock;

// Address of `scratch` on `device`, which must be the current device; nullptr on failure.
void* scratch_address(int device) {
  if (device < 0 || device >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> guard(scratch_lock);
  if (scratch_of_device[device] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    scratch_of_device[device] = ptr;
  }
  return scratch_of_device[device];
}

}  // namespace

namespace jenga {

int select_scratch_init(int device) { return scratch_address(device) != nullptr ? JENGA_OK : JENGA_EHIP; }

int launch_select(const jenga_plan* p, const void* q, const void* k, int32_t* sel_count, int32_t* sel_index,
                  uint8_t* mask, void* ws, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  if (p->cfg.head_dim == 128) return run_select<128>(p, q, k, sel_count, sel_index, mask, ws, st);
  return run_select<64>(p, q, k, sel_count, sel_index, mask, ws, st);
}

}  // namespace jenga

extern "C" int jenga_select_blocks_static(const jenga_plan* p, const void* q_curve, const void* k_curve,
                                          int32_t* sel_count, int32_t* sel_index, uint8_t* mask_or_null,
                                          void* stream) {
  if (!p || !q_curve || !k_curve || !sel_count || !sel_index) return JENGA_EINVAL;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != p->device) return JENGA_EINVAL;
  if (p->info.select_workspace_bytes > STATIC_SCRATCH_BYTES) return JENGA_EWORKSPACE;
  void* ws = scratch_address(dev);   // looked up when the plan was created; never allocates
  if (ws == nullptr) return JENGA_EHIP;
  // every byte of the scratch that select_kernel reads is written first by pool_kernel and
  // scores_kernel of this same call, so nothing has to be cleared between calls
  return jenga::launch_select(p, q_curve, k_curve, sel_count, sel_index, mask_or_null, ws, stream);
}
