// Progressive-resolution stage switch (Sec. 3.2, Eq. 4): clean-latent estimate, 3D area upsampling and
// re-noising in one pass over the output latent.  HBM-bound and elementwise: one thread per four
// consecutive output cells of a row, so stores and the noise reads are coalesced 16-byte accesses and
// neighbouring threads share the few input cells of their windows through the caches.
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
__global__ __launch_bounds__(256) void stage_switch_kernel(const float* __restrict__ x_t,
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

}  // namespace

extern "C" int jenga_stage_switch(const float* x_t, const float* eps_t, const float* eps_tilde, float* x_out,
                                  int32_t channels, int32_t T_in, int32_t H_in, int32_t W_in, int32_t T_out,
                                  int32_t H_out, int32_t W_out, float sigma_t, void* stream) {
  if (!x_t || !eps_t || !eps_tilde || !x_out) return JENGA_EINVAL;
  if (channels < 1 || T_in < 1 || H_in < 1 || W_in < 1 || T_out < 1 || H_out < 1 || W_out < 1) return JENGA_EINVAL;
  if (!(sigma_t >= 0.0f && sigma_t <= 1.0f)) return JENGA_EINVAL;
  const int32_t lim = 1 << 14;   // keeps the window arithmetic in 32 bits
  if (T_in > lim || H_in > lim || W_in > lim || T_out > lim || H_out > lim || W_out > lim) return JENGA_EUNSUPPORTED;
  const unsigned long long quads_per_row = ((unsigned)W_out + 3u) / 4u;
  const unsigned long long n_quads = (unsigned long long)channels * T_out * H_out * quads_per_row;
  if (n_quads > 0xFFFFFF00ull || (unsigned long long)channels * T_out * H_out > 0xFFFFFFFFull) return JENGA_EUNSUPPORTED;
  const bool vec = (W_out % 4 == 0) && ((((uintptr_t)eps_tilde) | ((uintptr_t)x_out)) & 15u) == 0;
  const dim3 grid((unsigned)((n_quads + 255) / 256));
  if (vec)
    stage_switch_kernel<true><<<grid, 256, 0, (hipStream_t)stream>>>(x_t, eps_t, eps_tilde, x_out, (uint32_t)n_quads,
                                                                    (uint32_t)quads_per_row, T_in, H_in, W_in, T_out,
                                                                    H_out, W_out, sigma_t);
  else
    stage_switch_kernel<false><<<grid, 256, 0, (hipStream_t)stream>>>(x_t, eps_t, eps_tilde, x_out, (uint32_t)n_quads,
                                                                     (uint32_t)quads_per_row, T_in, H_in, W_in, T_out,
                                                                     H_out, W_out, sigma_t);
  return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_EHIP;
}
