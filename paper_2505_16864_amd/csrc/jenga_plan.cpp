// Host-side plan: curve permutation, padded layout, adjacency bits.
//
// Sec. 3.1 of the paper: the re-ordering G (Eq. 2) and the masks B_cond and B_adja depend only
// on the resolution, so they are computed once per grid on the host (Alg. 1, "compute block
// reordering and adjacency masks") and kept on the device inside the plan.
//
// The curve restates the published generalized-Hilbert recursion that Sec. 3.1 cites for Eq. 2 (the
// paper only names it); the slab fallback and the choice of the outermost travel axis (longest
// side, ties w, h, t) are this library's.  Equality with the cited project's exact ordering is not
// claimed.  A box with corner p and signed edge vectors A (travel axis), B, C is visited from p
// to the neighbouring corner along A:
//   - two sides of length 1: a straight line;
//   - one side of length 1: the planar rule in the other two axes;
//   - A long (2a > 3b and 2a > 3c): two halves across A;
//   - one side axis clearly longer than the other (3b > 4c or 3c > 4b): three pieces in the
//     plane of A and that axis (out over the first half of A, across, back);
//   - otherwise five pieces along the 8-cell Hilbert path with face-sharing cells merged.
// Cuts are at floor(n/2), raised by one when odd and n > 2.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>

#include "jenga_internal.h"

namespace jenga {
namespace {

struct V3 {
  int x[3];
};
inline V3 operator+(V3 a, V3 b) { return {{a.x[0] + b.x[0], a.x[1] + b.x[1], a.x[2] + b.x[2]}}; }
inline V3 operator-(V3 a) { return {{-a.x[0], -a.x[1], -a.x[2]}}; }
inline V3 operator-(V3 a, V3 b) { return a + (-b); }
inline V3 operator*(V3 a, int s) { return {{a.x[0] * s, a.x[1] * s, a.x[2] * s}}; }
inline int length(V3 a) { return std::abs(a.x[0]) + std::abs(a.x[1]) + std::abs(a.x[2]); }
inline int sgn(int v) { return (v > 0) - (v < 0); }
inline V3 unit(V3 a) { return {{sgn(a.x[0]), sgn(a.x[1]), sgn(a.x[2])}}; }
inline int half_cut(int n) {
  int h = n / 2;
  if ((h & 1) && n > 2) ++h;
  return h;
}

struct Walker {
  int H, W;
  int32_t* out;
  size_t n;

  void emit(V3 p) { out[n++] = (int32_t)((p.x[0] * H + p.x[1]) * W + p.x[2]); }

  void line(V3 p, V3 step, int count) {
    for (int i = 0; i < count; ++i) emit(p + step * i);
  }

  // slab: travel axis A (a > 1), side axis B (b > 1), flat axis F (length 1)
  void planar(V3 p, V3 A, V3 B, V3 F) {
    const int a = length(A), b = length(B);
    const V3 dA = unit(A), dB = unit(B);
    const int a2 = half_cut(a), b2 = half_cut(b);
    const V3 A2 = dA * a2, B2 = dB * b2, Ar = dA * (a - a2), Br = dB * (b - b2);
    if (2 * a > 3 * b) {
      box(p, A2, B, F);
      box(p + A2, Ar, B, F);
      return;
    }
    box(p, B2, A2, F);
    box(p + B2, A, Br, F);
    box(p + (A - dA) + (B2 - dB), -B2, -Ar, F);
  }

  void box(V3 p, V3 A, V3 B, V3 C) {
    const int a = length(A), b = length(B), c = length(C);
    const V3 dA = unit(A), dB = unit(B), dC = unit(C);
    if (b == 1 && c == 1) return line(p, dA, a);
    if (a == 1 && c == 1) return line(p, dB, b);
    if (a == 1 && b == 1) return line(p, dC, c);
    if (a == 1) return (b >= c) ? box(p, B, C, A) : box(p, C, B, A);
    if (b == 1) return planar(p, A, C, B);
    if (c == 1) return planar(p, A, B, C);

    const int a2 = half_cut(a), b2 = half_cut(b), c2 = half_cut(c);
    const V3 A2 = dA * a2, B2 = dB * b2, C2 = dC * c2;
    const V3 Ar = dA * (a - a2), Br = dB * (b - b2), Cr = dC * (c - c2);
    const V3 endA = A - dA, endB2 = B2 - dB, endC = C - dC, endC2 = C2 - dC;

    if (2 * a > 3 * b && 2 * a > 3 * c) {
      box(p, A2, B, C);
      box(p + A2, Ar, B, C);
    } else if (3 * b > 4 * c) {
      box(p, B2, C, A2);
      box(p + B2, A, Br, C);
      box(p + endA + endB2, -B2, C, -Ar);
    } else if (3 * c > 4 * b) {
      box(p, C2, A2, B);
      box(p + C2, A, B, Cr);
      box(p + endA + endC2, -C2, -Ar, B);
    } else {
      box(p, B2, C2, A2);
      box(p + B2, C, A2, Br);
      box(p + endB2 + endC, A, -B2, -Cr);
      box(p + endA + B2 + endC, -C, -Ar, Br);
      box(p + endA + endB2, -B2, C2, -Ar);
    }
  }
};

}  // namespace

void curve_order(int T, int H, int W, bool use_curve, std::vector<int32_t>& perm) {
  const size_t n = (size_t)T * H * W;
  perm.resize(n);
  if (!use_curve) {
    for (size_t i = 0; i < n; ++i) perm[i] = (int32_t)i;
    return;
  }
  // outermost travel axis: the longest side; ties prefer w, then h, then t
  struct Side {
    int len, axis, pref;
  } s[3] = {{W, 2, 0}, {H, 1, 1}, {T, 0, 2}};
  std::sort(s, s + 3, [](const Side& l, const Side& r) {
    return l.len != r.len ? l.len > r.len : l.pref < r.pref;
  });
  V3 v[3];
  for (int i = 0; i < 3; ++i) {
    v[i] = {{0, 0, 0}};
    v[i].x[s[i].axis] = s[i].len;
  }
  Walker w{H, W, perm.data(), 0};
  w.box({{0, 0, 0}}, v[0], v[1], v[2]);
}

int build_host_tables(jenga_plan* plan) {
  const jenga_config& c = plan->cfg;
  jenga_plan_info_t& f = plan->info;
  const int m = c.block;
  const long long nv = (long long)c.T * c.H * c.W;
  f.N_v = (int32_t)nv;
  f.M_v = (int32_t)((nv + m - 1) / m);
  f.M_c = (c.n_text + m - 1) / m;
  f.M = f.M_v + f.M_c;
  f.N_pad = f.M * m;
  f.pad_v = f.M_v * m - f.N_v;
  f.pad_c = f.M_c * m - c.n_text;
  // Alg. 3 uses k*M_v as a slice bound without saying how it is rounded: floor, guarded against
  // products such as 0.3*260 that land a hair below an integer, and never less than one block.
  f.K_top = f.M_v > 0 ? std::max(1, (int)std::floor(c.topk_ratio * f.M_v + 1e-6)) : 0;
  plan->nt64 = (f.M + 63) / 64;

  curve_order(c.T, c.H, c.W, (c.flags & JENGA_FLAG_CURVE) != 0, plan->perm);
  plan->inv_perm.assign(f.N_v, 0);
  for (int i = 0; i < f.N_v; ++i) plan->inv_perm[plan->perm[i]] = i;

  plan->src_of_pos.assign(f.N_pad, -1);
  for (int i = 0; i < f.N_v; ++i) plan->src_of_pos[i] = plan->perm[i];
  for (int i = 0; i < c.n_text; ++i) plan->src_of_pos[(size_t)f.M_v * m + i] = f.N_v + i;

  plan->blk_valid.assign(f.M, m);
  if (f.M_v > 0) plan->blk_valid[f.M_v - 1] = m - f.pad_v;
  if (f.M_c > 0) plan->blk_valid[f.M - 1] = m - f.pad_c;

  // fixed bits of query block i: text key blocks (condition mask) and blocks holding a token
  // within Chebyshev distance 1 of one of i's tokens (adjacency mask, 26-neighbourhood + self)
  plan->fixed_bits.assign((size_t)f.M_v * plan->nt64, 0);
  auto set_bit = [&](int i, int j) { plan->fixed_bits[(size_t)i * plan->nt64 + (j >> 6)] |= 1ull << (j & 63); };
  if (c.flags & JENGA_FLAG_CONDITION)
    for (int i = 0; i < f.M_v; ++i)
      for (int j = f.M_v; j < f.M; ++j) set_bit(i, j);
  if (c.flags & JENGA_FLAG_ADJACENCY) {
    for (int t = 0; t < c.T; ++t)
      for (int h = 0; h < c.H; ++h)
        for (int w = 0; w < c.W; ++w) {
          const int bi = plan->inv_perm[((size_t)t * c.H + h) * c.W + w] / m;
          for (int dt = -1; dt <= 1; ++dt) {
            const int t2 = t + dt;
            if (t2 < 0 || t2 >= c.T) continue;
            for (int dh = -1; dh <= 1; ++dh) {
              const int h2 = h + dh;
              if (h2 < 0 || h2 >= c.H) continue;
              for (int dw = -1; dw <= 1; ++dw) {
                const int w2 = w + dw;
                if (w2 < 0 || w2 >= c.W) continue;
                set_bit(bi, plan->inv_perm[((size_t)t2 * c.H + h2) * c.W + w2] / m);
              }
            }
          }
        }
  }

  // workspaces
  const uint64_t bh = (uint64_t)c.batch * c.heads;
  auto align256 = [](uint64_t x) { return (x + 255) & ~255ull; };
  // select: pooled Q [bh][M_v][d] f64, pooled K [bh][M][d] f64, scores [bh][M_v][M] f64
  f.select_workspace_bytes = align256(bh * f.M_v * c.head_dim * 8) + align256(bh * f.M * c.head_dim * 8) +
                             align256(bh * (uint64_t)f.M_v * f.M * 8);
  // attention: K and V re-tiled, bf16, one tile per (batch, head, block)
  f.attn_workspace_bytes = 2 * align256(bh * (uint64_t)f.N_pad * c.head_dim * 2) + 256;   // packed K, packed V, launch parameters
  return JENGA_OK;
}

}  // namespace jenga
