// Progressive-resolution stage switch (Sec. 3.2, Eq. 4): clean-latent estimate, 3D area upsampling and
// re-noising in one pass over the output latent.  HBM-bound and elementwise.  Two kernels: the tiled
// one stages the input rows a group of output rows needs in LDS with 16-byte loads (the windows are
// then LDS reads); the direct one reads the windows from global memory and takes every shape.
#include <hip/hip_runtime.h>

#include <cmath>

#include "jenga_internal.h"

namespace {

// [start, end) of the input cells averaged by output cell o: floor(o*I/O) .. ceil((o+1)*I/O).
// All sizes are at most 2^14, so the products fit 32 bits.
__device__ inline void area_window(uint32_t o, uint32_t n_in, uint32_t n_out, uint32_t* s, uint32_t* e) {
  *s = (o * n_in) / n_out;
  *e = ((o + 1) * n_in + n_out - 1) / n_out;
}

// One thread = four consecutive w of one output row (c, t, h); VEC: 16-byte loads and stores of the
// noise and the result (W_out divisible by 4 and both pointers 16-byte aligned).
template <bool VEC>
__global__ __launch_bounds__(256) void stage_switch_direct_kernel(const float* __restrict__ x_t,
                                                           const float* __restrict__ eps_t,
                                                           const float* __restrict__ eps_tilde,
                                                           float* __restrict__ x_out, uint32_t n_quads,
                                                           uint32_t quads_per_row, uint32_t T, uint32_t H, uint32_t W,
                                                           uint32_t To, uint32_t Ho, uint32_t Wo, float sigma) {
  const uint32_t id = blockIdx.x * 256u + threadIdx.x;
  if (id >= n_quads) return;
  const uint32_t row = id / quads_per_row, wq = (id - row * quads_per_row) * 4u;
  const uint32_t ct = row / Ho, h = row - ct * Ho;
  const uint32_t c = ct / To, t = ct - c * To;
  uint32_t t0, t1, h0, h1;
  area_window(t, T, To, &t0, &t1);
  area_window(h, H, Ho, &h0, &h1);
  const size_t plane = (size_t)c * T * H * W;
  const float* xc = x_t + plane;
  const float* ec = eps_t + plane;
  const size_t o = (size_t)row * Wo + wq;
  float nz[4] = {0.f, 0.f, 0.f, 0.f}, res[4];
  if (VEC) {
    const float4 v = *(const float4*)(eps_tilde + o);
    nz[0] = v.x; nz[1] = v.y; nz[2] = v.z; nz[3] = v.w;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (wq + i < Wo) nz[i] = eps_tilde[o + i];
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t w = min(wq + i, Wo - 1);
    uint32_t w0, w1;
    area_window(w, W, Wo, &w0, &w1);
    float sum = 0.f;
    for (uint32_t a = t0; a < t1; ++a)
      for (uint32_t b = h0; b < h1; ++b) {
        const size_t r = ((size_t)a * H + b) * W;
        for (uint32_t d = w0; d < w1; ++d) sum += fmaf(-sigma, ec[r + d], xc[r + d]);   // x0_hat = x_t - sigma eps_t
      }
    const float mean = sum / (float)((t1 - t0) * (h1 - h0) * (w1 - w0));
    res[i] = fmaf(sigma, nz[i], (1.0f - sigma) * mean);
  }
  if (VEC) {
    *(float4*)(x_out + o) = make_float4(res[0], res[1], res[2], res[3]);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (wq + i < Wo) x_out[o + i] = res[i];
  }
}

// a / b for a < 2^28 + 2^15 and a quotient of at most 2^14: the float estimate is off by at most one.
__device__ inline uint32_t div_small_quotient(uint32_t a, uint32_t b, float rcp_b) {
  uint32_t q = (uint32_t)((float)a * rcp_b);
  const int32_t r = (int32_t)(a - q * b);
  if (r < 0) --q;
  else if (r >= (int32_t)b) ++q;
  return q;
}

constexpr int TILE_FLOATS = 12288;   // 48 KB of LDS for the staged clean-latent estimate

// grid (channels * T_out, row groups).  A workgroup produces `rows_per_wg` consecutive output rows h of
// one (c, t) plane.  It first stages x0_hat = x_t - sigma eps_t of every input row these outputs touch
// ([t0, t1) x [H0, H1) x W, contiguous per t) in LDS with 16-byte loads, then every thread averages
// the windows of four consecutive w from LDS.  Needs W_in % 4 == 0, 16-byte aligned inputs and a tile
// of at most TILE_FLOATS; the host falls back to stage_switch_direct_kernel otherwise.  The sums run
// in the same (t, h, w) order as there, so both kernels give the same bits.
template <bool VEC, bool UP>
__global__ __launch_bounds__(256) void stage_switch_tiled_kernel(const float* __restrict__ x_t,
                                                                 const float* __restrict__ eps_t,
                                                                 const float* __restrict__ eps_tilde,
                                                                 float* __restrict__ x_out, uint32_t quads_per_row,
                                                                 uint32_t rows_per_wg, uint32_t T, uint32_t H,
                                                                 uint32_t W, uint32_t To, uint32_t Ho, uint32_t Wo,
                                                                 uint32_t tile_floats, float sigma) {
  extern __shared__ float4 xs_raw[];   // tile_floats floats, sized by the host
  float* xs = (float*)xs_raw;
  const uint32_t ct = blockIdx.x;
  const uint32_t c = ct / To, t = ct - c * To;
  const uint32_t hb = blockIdx.y * rows_per_wg, he = min(hb + rows_per_wg, Ho);   // output rows [hb, he)
  uint32_t t0, t1, H0, H1, tmp;
  area_window(t, T, To, &t0, &t1);
  area_window(hb, H, Ho, &H0, &tmp);
  area_window(he - 1, H, Ho, &tmp, &H1);
  const uint32_t nh = H1 - H0, plane = nh * W;   // staged rows per t, floats per t
  if ((t1 - t0) * plane > tile_floats) return;   // cannot happen: the host sizes the tile for it
  for (uint32_t a = t0; a < t1; ++a) {
    const size_t src = (((size_t)c * T + a) * H + H0) * W;
    float* dst = xs + (a - t0) * plane;
    for (uint32_t i = threadIdx.x * 4u; i < plane; i += 1024u) {
      const float4 x = *(const float4*)(x_t + src + i);
      const float4 e = *(const float4*)(eps_t + src + i);
      *(float4*)(dst + i) = make_float4(fmaf(-sigma, e.x, x.x), fmaf(-sigma, e.y, x.y), fmaf(-sigma, e.z, x.z),
                                        fmaf(-sigma, e.w, x.w));
    }
  }
  __syncthreads();

  const uint32_t slots = rows_per_wg > 1 ? quads_per_row : 256u;   // quads a row gets per pass
  const uint32_t r_local = threadIdx.x / slots;
  const uint32_t q0 = threadIdx.x - r_local * slots;
  const uint32_t h = hb + r_local;
  if (r_local >= rows_per_wg || h >= Ho) return;
  const float rcp_ho = 1.0f / (float)Ho, rcp_wo = 1.0f / (float)Wo;
  const uint32_t h0 = div_small_quotient(h * H, Ho, rcp_ho);
  const uint32_t h1 = div_small_quotient((h + 1) * H + Ho - 1, Ho, rcp_ho);
  const size_t row = (size_t)ct * Ho + h;
  for (uint32_t quad = q0; quad < quads_per_row; quad += slots) {
    const uint32_t wq = quad * 4u;
    const size_t o = row * Wo + wq;
    float nz[4] = {0.f, 0.f, 0.f, 0.f}, res[4];
    if (VEC) {
      const float4 v = *(const float4*)(eps_tilde + o);
      nz[0] = v.x; nz[1] = v.y; nz[2] = v.z; nz[3] = v.w;
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (wq + i < Wo) nz[i] = eps_tilde[o + i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t w = min(wq + i, Wo - 1);
      const uint32_t w0 = div_small_quotient(w * W, Wo, rcp_wo);
      const uint32_t w1 = div_small_quotient((w + 1) * W + Wo - 1, Wo, rcp_wo);
      float sum = 0.f;
      if (UP) {
        // no axis shrinks: every window is one or two cells long, so the 2 x 2 x 2 candidates are read
        // without branches and the ones outside the window add 0 (same order of additions)
        const uint32_t nt = t1 - t0, nb = h1 - h0, nd = w1 - w0;
#pragma unroll
        for (uint32_t a = 0; a < 2; ++a)
#pragma unroll
          for (uint32_t b = 0; b < 2; ++b)
#pragma unroll
            for (uint32_t d = 0; d < 2; ++d) {
              const float v = xs[min(a, nt - 1) * plane + (h0 - H0 + min(b, nb - 1)) * W + w0 + min(d, nd - 1)];
              sum += (a < nt && b < nb && d < nd) ? v : 0.f;
            }
      } else {
        for (uint32_t a = 0; a < t1 - t0; ++a)
          for (uint32_t b = h0; b < h1; ++b) {
            const float* r = xs + a * plane + (b - H0) * W;
            for (uint32_t d = w0; d < w1; ++d) sum += r[d];
          }
      }
      const float mean = sum / (float)((t1 - t0) * (h1 - h0) * (w1 - w0));
      res[i] = fmaf(sigma, nz[i], (1.0f - sigma) * mean);
    }
    if (VEC) {
      *(float4*)(x_out + o) = make_float4(res[0], res[1], res[2], res[3]);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (wq + i < Wo) x_out[o + i] = res[i];
    }
  }
}

}  // namespace

extern "C" int jenga_stage_switch(const float* x_t, const float* eps_t, const float* eps_tilde, float* x_out,
                                  int32_t channels, int32_t T_in, int32_t H_in, int32_t W_in, int32_t T_out,
                                  int32_t H_out, int32_t W_out, float sigma_t, void* stream) {
  if (!x_t || !eps_t || !eps_tilde || !x_out) return JENGA_EINVAL;
  if (channels < 1 || T_in < 1 || H_in < 1 || W_in < 1 || T_out < 1 || H_out < 1 || W_out < 1) return JENGA_EINVAL;
  if (!(sigma_t >= 0.0f && sigma_t <= 1.0f)) return JENGA_EINVAL;
  const int32_t lim = 1 << 14;   // keeps the window arithmetic in 32 bits
  if (T_in > lim || H_in > lim || W_in > lim || T_out > lim || H_out > lim || W_out > lim) return JENGA_EUNSUPPORTED;
  const unsigned quads_per_row = ((unsigned)W_out + 3u) / 4u;
  const unsigned long long n_quads = (unsigned long long)channels * T_out * H_out * quads_per_row;
  if (n_quads > 0xFFFFFF00ull) return JENGA_EUNSUPPORTED;
  const bool vec = (W_out % 4 == 0) && ((((uintptr_t)eps_tilde) | ((uintptr_t)x_out)) & 15u) == 0;
  hipStream_t st = (hipStream_t)stream;

  // Tiled path: largest group of output rows whose input rows fit the LDS tile.
  auto window_len_max = [](long long n_in, long long n_out) { return (n_in + n_out - 1) / n_out + 1; };
  const bool in_vec = (W_in % 4 == 0) && ((((uintptr_t)x_t) | ((uintptr_t)eps_t)) & 15u) == 0;
  unsigned rows_per_wg = quads_per_row >= 256u ? 1u : 256u / quads_per_row;
  if (rows_per_wg > (unsigned)H_out) rows_per_wg = (unsigned)H_out;
  const long long nt_max = window_len_max(T_in, T_out);
  auto tile_floats = [&](unsigned rows) {
    // input rows touched by `rows` consecutive output rows: at most floor((rows-1)*H_in/H_out) + window + 1
    const long long nh = ((long long)(rows - 1) * H_in) / H_out + window_len_max(H_in, H_out) + 1;
    return nt_max * (nh < H_in ? nh : H_in) * W_in;
  };
  while (rows_per_wg > 1 && tile_floats(rows_per_wg) > TILE_FLOATS) --rows_per_wg;
  if (in_vec && (unsigned long long)channels * T_out <= 0x7FFFFFFFull && tile_floats(rows_per_wg) <= TILE_FLOATS) {
    const dim3 grid((unsigned)(channels * T_out), ((unsigned)H_out + rows_per_wg - 1) / rows_per_wg);
    const bool up = T_in <= T_out && H_in <= H_out && W_in <= W_out;
    const long long need = tile_floats(rows_per_wg);
    const size_t lds_bytes = (size_t)need * sizeof(float);
#define JENGA_TILED(V, U)                                                                                          \
  stage_switch_tiled_kernel<V, U><<<grid, 256, lds_bytes, st>>>(x_t, eps_t, eps_tilde, x_out, quads_per_row,       \
                                                                rows_per_wg, T_in, H_in, W_in, T_out, H_out, W_out, \
                                                                (uint32_t)need, sigma_t)
    if (vec && up) JENGA_TILED(true, true);
    else if (vec) JENGA_TILED(true, false);
    else if (up) JENGA_TILED(false, true);
    else JENGA_TILED(false, false);
#undef JENGA_TILED
    return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_EHIP;
  }

  const dim3 grid((unsigned)((n_quads + 255) / 256));
  if (vec)
    stage_switch_direct_kernel<true><<<grid, 256, 0, st>>>(x_t, eps_t, eps_tilde, x_out, (uint32_t)n_quads,
                                                          (uint32_t)quads_per_row, T_in, H_in, W_in, T_out, H_out,
                                                          W_out, sigma_t);
  else
    stage_switch_direct_kernel<false><<<grid, 256, 0, st>>>(x_t, eps_t, eps_tilde, x_out, (uint32_t)n_quads,
                                                           (uint32_t)quads_per_row, T_in, H_in, W_in, T_out, H_out,
                                                           W_out, sigma_t);
  return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_EHIP;
}
