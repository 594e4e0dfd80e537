// Block-sparse flash attention for gfx950 (appendix Alg. 4; Alg. 2 for the text rows; Eq. 1 inside
// the visited blocks).
//
// One workgroup owns one query block of BLK rows of one (batch, head): BLK/32 wavefronts, each with
// 32 query rows.  It walks the ascending list of selected key blocks.  Per key block:
//     S^T = K Q^T         v_mfma_f32_32x32x16_bf16, K fragments from LDS, Q fragments in registers
//     online softmax      float32, base-2 exponent, statistics per query row; the reference the
//                         exponent is taken against moves lazily (128-token blocks: only when a row
//                         sum leaves its range), row sums are float32 sums of P
//     O^T += V^T P^T      v_mfma_f32_32x32x16_bf16, V^T fragments from LDS, P^T straight from the
//                         S^T accumulators
// Working on the transposed products keeps one query row in one lane (column) of every
// accumulator, so the row maximum and row sum are lane-local (one cross-half exchange), and the
// accumulator layout of S^T is already the B-operand layout PV needs: P never goes through LDS.
//
// K and V are first re-tiled once per call (pack_kernel) into "fragment order": for every block a
// 16-byte piece per (fragment, lane) in exactly the order the LDS reads want them, so that a tile
// moves global -> LDS as a straight copy and every LDS read is a conflict-free 1 KB wave read.
// The V tile is stored transposed, with its key index permuted to match the accumulator layout:
//     accumulator register r of kv-tile mt, lane l  <->  key 32*mt + 8*(r/4) + 4*(l/32) + r%4,
//     query (l%32).
#include <hip/hip_runtime.h>

#include <cmath>

#include <type_traits>
#include <utility>

#include "jenga_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// grid (M, batch*heads).  K tile -> fragment order; V tile -> transposed fragment order, pad rows zeroed.
template <int BLK, int D>
__global__ __launch_bounds__(256) void pack_kernel(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                   uint4* __restrict__ kp, uint4* __restrict__ vp,
                                                   const int32_t* __restrict__ blk_valid, int M, int n_pad) {
  constexpr int KS = D / 16, PS = BLK / 16, CH = D / 8;
  constexpr int TILE_CHUNKS = BLK * D / 8;
  constexpr int LDV = D + 8;   // padded row length (elements) of the staged V tile
  __shared__ uint16_t vl[BLK * LDV];
  const int j = blockIdx.x, bh = blockIdx.y;
  const int nv = blk_valid[j];
  const size_t row0 = (size_t)bh * n_pad + (size_t)j * BLK;
  const uint4* ksrc = (const uint4*)(k + row0 * D);
  const uint4* vsrc = (const uint4*)(v + row0 * D);
  uint4* kdst = kp + ((size_t)bh * M + j) * TILE_CHUNKS;
  uint4* vdst = vp + ((size_t)bh * M + j) * TILE_CHUNKS;

  for (int o = threadIdx.x; o < TILE_CHUNKS; o += 256) {
    const int lane = o & 63, f = o >> 6;
    const int ks = f % KS, mt = f / KS;
    const int row = 32 * mt + (lane & 31);
    kdst[o] = ksrc[row * CH + 2 * ks + (lane >> 5)];
  }
  for (int o = threadIdx.x; o < TILE_CHUNKS; o += 256) {
    const int row = o / CH, cc = o % CH;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (row < nv) val = vsrc[o];
    *(uint4*)&vl[row * LDV + cc * 8] = val;
  }
  __syncthreads();
  for (int o = threadIdx.x; o < TILE_CHUNKS; o += 256) {
    const int lane = o & 63, f = o >> 6;
    const int ps = f % PS, dt = f / PS;
    const int hl = lane >> 5, d = 32 * dt + (lane & 31);
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const int e = 2 * e2;
      const int kv0 = 16 * ps + 8 * (e / 4) + 4 * hl + (e % 4);
      w[e2] = (uint32_t)vl[kv0 * LDV + d] | ((uint32_t)vl[(kv0 + 1) * LDV + d] << 16);
    }
    vdst[o] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// One DMA instruction, global -> LDS without passing through registers: every lane hands over its
// own 16-byte global address (wave-uniform 64-bit base in SGPRs + 32-bit per-lane byte offset); the
// data of the wave lands contiguously (1 KB) behind the wave-uniform LDS byte address in M0.
// Written as asm so that the compiler does not track these copies: it would otherwise order every
// later LDS read of the same array behind them with a full vmcnt(0) wait.  Completion is tracked by
// vmcnt and waited for explicitly (wait_vmem) before the barrier that publishes a tile.
// dma_1kb_to_lds_at takes the LDS byte address as a number the caller keeps in an SGPR;
// dma_1kb_to_lds derives it from a pointer (a few more instructions per copy).
__device__ inline void dma_1kb_to_lds_at(const void* uniform_base, uint32_t lane_byte_off, uint32_t lds_addr) {
  const uint64_t b = (uint64_t)uniform_base;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
  const uint64_t base = ((uint64_t)hi << 32) | lo;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(lane_byte_off), "s"(base)
               : "memory", "m0");
}
__device__ inline void dma_1kb_to_lds(const void* uniform_base, uint32_t lane_byte_off, const void* lds_dst) {
  dma_1kb_to_lds_at(uniform_base, lane_byte_off,
                    __builtin_amdgcn_readfirstlane(
                        (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)lds_dst));
}

// Straight copy of one packed tile (global, fragment order) into LDS without passing through
// registers.
template <int NTHR, int CPT>
__device__ inline void tile_to_lds(const u32x4* __restrict__ src_tile, u32x4* lds, int tid, int wave) {
#pragma unroll
  for (int c = 0; c < CPT; ++c)
    dma_1kb_to_lds((const char*)src_tile + (size_t)c * NTHR * 16, (uint32_t)tid * 16u, lds + c * NTHR + wave * 64);
}

__device__ inline void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0) only

// Online-softmax bookkeeping with a lazily moved reference (Alg. 4 keeps a running maximum m and
// rescales l and O whenever it grows).  Here the reference m_run only moves when some row's new
// maximum exceeds it by more than LAZY_LOG2 (in base-2 logit units): until then the probabilities are
// formed against the old reference and stay below 2^LAZY_LOG2, which the float32 sums and the bf16
// products hold without loss (bf16 has float32's exponent range), and the final division by l
// cancels the common factor exactly as it does for the running maximum.  The branch is uniform over
// the wavefront; after the first few blocks it is almost never taken.
constexpr float LAZY_LOG2 = 8.0f;
template <int DT>
__device__ __forceinline__ void rescale_if_grown(float cand, float& m_run, float& l_run, f32x16 (&O)[DT]) {
  if (__ballot(cand > m_run + LAZY_LOG2)) {   // also taken by the first block with a valid key (m_run = -inf)
    asm volatile("");                         // keep it a real branch
    const float m_new = fmaxf(m_run, cand);
    const float alpha = m_new == m_run ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
    l_run *= alpha;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
  }
}

// Work mapping shared by the attention kernels.  The text query blocks of every (batch, head) are
// dense rows, several times longer than a vision row: they are dealt out first, ahead of all vision
// blocks, so that none of them starts late and runs on alone at the end.  The vision blocks follow
// head by head; workgroups are dealt round-robin to the 8 XCDs, and each XCD gets a contiguous run
// of query blocks of the head, so that the whole chip works on one head at a time (its K and V stay
// in the last-level cache) and neighbouring query blocks, whose selections overlap, share an L2.
// Returns false for the filler workgroups of the last run.
__device__ inline bool map_work(int n, int n_bh, int M, int M_v, int chunk, int* bh, int* i) {
  const int M_c = M - M_v;
  const int n_text = n_bh * M_c;
  if (n < n_text) {
    *bh = n / M_c;
    *i = M_v + n % M_c;
    return true;
  }
  n -= n_text;
  const int xcd = n & 7, s = n >> 3;
  *bh = s / chunk;
  *i = xcd * chunk + s % chunk;
  return *i < M_v;
}

template <int BLK, int D>
struct AttnTraits {
  static constexpr int NW = BLK / 32;          // wavefronts per workgroup
  static constexpr int NTHR = NW * 64;
  static constexpr int MT = BLK / 32;          // 32-key tiles per key block
  static constexpr int KS = D / 16;            // k-steps of K Q^T
  static constexpr int DT = D / 32;            // 32-channel tiles of the output
  static constexpr int PS = BLK / 16;          // k-steps of V^T P^T
  static constexpr int TILE_CHUNKS = BLK * D / 8;
  static constexpr int CPT = TILE_CHUNKS / NTHR;   // 16-byte pieces per thread per tile
  static constexpr int MIN_WAVES = (BLK == 128 && D == 128) ? 2 : 1;
};

template <int BLK, int D>
__global__ __launch_bounds__((AttnTraits<BLK, D>::NTHR), (AttnTraits<BLK, D>::MIN_WAVES)) void attn_kernel(
    const uint16_t* __restrict__ q, const u32x4* __restrict__ kp, const u32x4* __restrict__ vp,
    const int32_t* __restrict__ sel_count, const int32_t* __restrict__ sel_index,
    const int32_t* __restrict__ blk_valid, uint16_t* __restrict__ out, float* __restrict__ lse, int n_bh, int M,
    int M_v, int n_pad, int chunk, float scale_log2e, float bias_log2e) {
  using TR = AttnTraits<BLK, D>;
  constexpr int NTHR = TR::NTHR, MT = TR::MT, KS = TR::KS, DT = TR::DT, PS = TR::PS;
  constexpr int TILE_CHUNKS = TR::TILE_CHUNKS, CPT = TR::CPT;
  __shared__ u32x4 Ks[TILE_CHUNKS];
  __shared__ u32x4 Vs[TILE_CHUNKS];

  int bh, i;
  if (!map_work(blockIdx.x, n_bh, M, M_v, chunk, &bh, &i)) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, lets LDS bases live in SGPRs
  const int hl = lane >> 5, ql = lane & 31;
  const int qrow = i * BLK + 32 * wave + ql;

  bf16x8 qf[KS];
  {
    const u32x4* qp = (const u32x4*)(q + ((size_t)bh * n_pad + qrow) * D);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, qp[2 * ks + hl]);
  }

  int cnt = sel_count[(size_t)bh * M + i];
  cnt = min(max(cnt, 0), M);
  const int32_t* idx = sel_index + ((size_t)bh * M + i) * M;
  const u32x4* kbase = kp + (size_t)bh * M * TILE_CHUNKS;
  const u32x4* vbase = vp + (size_t)bh * M * TILE_CHUNKS;

  float m_run = -INFINITY, l_run = 0.f;
  f32x16 O[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[dt][r] = 0.f;

  if (cnt > 0) {
    const int j0 = min(max(idx[0], 0), M - 1);
    tile_to_lds<NTHR, CPT>(kbase + (size_t)j0 * TILE_CHUNKS, Ks, tid, wave);
  }

  for (int it = 0; it < cnt; ++it) {
    const int j = min(max(idx[it], 0), M - 1);
    wait_vmem();       // this wave's part of the K tile has landed
    __syncthreads();   // K tile of this step is in LDS; every wave is past the previous PV
    tile_to_lds<NTHR, CPT>(vbase + (size_t)j * TILE_CHUNKS, Vs, tid, wave);

    f32x16 S[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) S[mt][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, Ks[(mt * KS + ks) * 64 + lane]);
        S[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], S[mt], 0, 0, 0);
      }
    }

    // ---- online softmax on S^T (lane = query row, registers = keys) ----
    const int nv = blk_valid[j];
    if (nv < BLK) {   // sequence-length mask: pad keys of a ragged block
      asm volatile("");   // keep this a real (rarely taken) branch instead of 64 selects per tile
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = 32 * mt + 8 * (r / 4) + 4 * hl + (r % 4);
          if (kv >= nv) S[mt][r] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[mt][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float bias = (i < M_v && j >= M_v) ? bias_log2e : 0.f;
    rescale_if_grown(fmaf(mx, scale_log2e, bias), m_run, l_run, O);
    const float off = m_run == -INFINITY ? 0.f : bias - m_run;   // every key so far was padding: keep it finite
    float rs0 = 0.f, rs1 = 0.f;
    bf16x8 pb[PS];
#pragma unroll
    for (int ps = 0; ps < PS; ++ps) {
      uint32_t w[4];
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(S[ps >> 1][8 * (ps & 1) + 2 * e2], scale_log2e, off));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(S[ps >> 1][8 * (ps & 1) + 2 * e2 + 1], scale_log2e, off));
        w[e2] = pack_bf16x2(p0, p1);
        rs0 += p0;
        rs1 += p1;
      }
      u32x4 pw = {w[0], w[1], w[2], w[3]};
      pb[ps] = __builtin_bit_cast(bf16x8, pw);
    }
    l_run += rs0 + rs1;

    wait_vmem();       // this wave's part of the V tile has landed
    __syncthreads();   // V tile is in LDS; every wave is done reading the K tile
    if (it + 1 < cnt) {
      const int jn = min(max(idx[it + 1], 0), M - 1);
      tile_to_lds<NTHR, CPT>(kbase + (size_t)jn * TILE_CHUNKS, Ks, tid, wave);
    }

#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int ps = 0; ps < PS; ++ps) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, Vs[(dt * PS + ps) * 64 + lane]);
        O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[ps], O[dt], 0, 0, 0);
      }
    }
  }

  // ---- normalise and store: lane holds row qrow, channels 32*dt + 8*g + 4*hl + {0..3} ----
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const bool row_ok = (32 * wave + ql) < blk_valid[i] && l_tot > 0.f;
  const float inv = row_ok ? 1.0f / l_tot : 0.f;
  // natural-log sum of exp(logit) over the visited keys: the running maximum is in base-2 units
  if (lse != nullptr && hl == 0)
    lse[(size_t)bh * n_pad + qrow] = row_ok ? (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
  uint16_t* orow = out + ((size_t)bh * n_pad + qrow) * D;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 w;
      w.x = row_ok ? pack_bf16x2(O[dt][4 * g] * inv, O[dt][4 * g + 1] * inv) : 0u;
      w.y = row_ok ? pack_bf16x2(O[dt][4 * g + 2] * inv, O[dt][4 * g + 3] * inv) : 0u;
      *(uint2*)(orow + 32 * dt + 8 * g + 4 * hl) = w;
    }
}

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// One 1 KB MFMA fragment (16 bytes per lane) from LDS, issued here and now: the compiler's own
// scheduling reads one fragment, waits, multiplies, and so leaves the LDS latency open before
// every MFMA.  Reads issued through lds_frag are complete only after lds_wait on their registers.
// Between the two asm statements the destination registers are in flight: the code is correct only
// as long as the compiler does not copy or reuse them there.  lds_wait ties them ("+v") so that the
// allocator has no reason to, and tests/test_kernel_listing.py checks the generated listing of every
// build for exactly this (no instruction between a read and its wait touches the read's registers).
// Folding read, MFMAs and wait of a group into one asm statement removes the assumption but was
// measured 4 % slower here: with S live the register budget of three wavefronts per SIMD only leaves
// room for groups of two, and the compiler can no longer lay the softmax arithmetic under the MFMAs.
template <int BYTE_OFF>
__device__ __forceinline__ void lds_frag(u32x4& dst, uint32_t lane_addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(lane_addr), "n"(BYTE_OFF) : "memory");
}
__device__ __forceinline__ void lds_wait(u32x4 (&g)[4]) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(g[0]), "+v"(g[1]), "+v"(g[2]), "+v"(g[3]) : : "memory");
}

// max over the two lanes l and l ^ 32 (the two halves of a query row's keys), in the vector ALU
__device__ inline float max_with_other_half(float x) {
#if defined(__HIP_DEVICE_COMPILE__)
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
#else
  return x;   // host pass only; never executed
#endif
}

// attn_h_kernel takes the lazy reference one step further and drops the row maximum from the common
// path: the maximum over the 32 logits of a lane (16 v_max3, a cross-half exchange, a compare) is a
// chain that has to finish after the last MFMA of S and before the first exponential can issue, in
// every step of every wavefront.  Without it a step forms its probabilities against the reference as
// it stands and only looks at the sum: while a lane's 32 probabilities add up to at most P_SUM_MAX they
// are all representable, and so are the float32 sums and products built from them (bf16 and float32
// share the exponent range; 2^30 times the row length times |V| stays far below 2^127).  A sum above
// the bound, infinite or undefined sends the step down the exact path: logits again (the K half is
// still in LDS), row maximum, rescale, probabilities <= 1.  The first step of a row starts there.
// The reference never exceeds the largest logit seen, so the largest term is never lost to underflow.
constexpr float P_SUM_MAX = 1073741824.0f;   // 2^30

// ---------------------------------------------------------------------------------------------
// attn_h_kernel: blocks of 128 tokens, walked in half blocks of 64 keys.
//
// A wavefront does its softmax between its two runs of MFMAs, so it is the other wavefronts of the
// SIMD that keep the MFMA pipe fed meanwhile: occupancy matters.  A step over 64 keys needs half
// the S and P registers and half the LDS of a step over 128, which lets three workgroups (twelve
// wavefronts) live on a CU instead of two; everything else is attn_kernel: 4 waves x 32 query
// rows, transposed products, K and V^T fragments straight from the packed tiles, DMA to LDS.
//
// PACED (JENGA_FLAG_PACED_WALK): the selected blocks are not visited in list order.  A position G sweeps
// over the key blocks once per lap, derived from the constant-frequency clock that every CU reads
// (s_memrealtime), and a workgroup always takes the first block of its list that it has not visited yet
// at or after G (wrapping around).  Softmax attention does not depend on the order of the keys, so the
// result is the same up to rounding; what changes is when a tile is asked for: all workgroups of an XCD
// now ask for neighbouring tiles at neighbouring times, and the 4 MB L2, which catches a seventh of the
// tile reads of the in-order walk, catches more than half of them (measured on the 720p workload).
// The price: the order, and with it the last bits of the output, can differ from run to run.
// ---------------------------------------------------------------------------------------------
template <int D, bool PACED>
__global__ __launch_bounds__(256, 3) void attn_h_kernel(
    const uint16_t* __restrict__ q, const u32x4* __restrict__ kp, const u32x4* __restrict__ vp,
    const int32_t* __restrict__ sel_count, const int32_t* __restrict__ sel_index,
    const int32_t* __restrict__ blk_valid, uint16_t* __restrict__ out, float* __restrict__ lse, int n_bh, int M,
    int M_v, int n_pad, int chunk, int pad_v, int pad_c, float scale_log2e, float bias_log2e,
    const uint32_t* __restrict__ pace_params) {
  constexpr int BLK = 128, KS = D / 16, DT = D / 32, PS = BLK / 16, MH = 2, PH = 4;
  constexpr int TILE_CHUNKS = BLK * D / 8, HALF_CHUNKS = TILE_CHUNKS / 2, CPT = HALF_CHUNKS / 256;
  __shared__ u32x4 Ks[HALF_CHUNKS];   // fragments (m2, ks) of the current 64 keys
  __shared__ u32x4 Vs[HALF_CHUNKS];   // fragments (dt, p2) of the current 64 keys
  __shared__ uint32_t rem_bits[PACED ? 64 : 1];   // PACED: bitmap of the blocks still to visit, 32 per word
  __shared__ int pace_slot[2];                    // PACED: G for the next pick, published by thread 0

  int bh, i;
  if (!map_work(blockIdx.x, n_bh, M, M_v, chunk, &bh, &i)) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hl = lane >> 5, ql = lane & 31;
  const int qrow = i * BLK + 32 * wave + ql;

  bf16x8 qf[KS];
  {
    const u32x4* qp = (const u32x4*)(q + ((size_t)bh * n_pad + qrow) * D);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, qp[2 * ks + hl]);
  }

  int cnt = sel_count[(size_t)bh * M + i];
  cnt = min(max(cnt, 0), M);
  const int32_t* idx = sel_index + ((size_t)bh * M + i) * M;
  uint32_t rem = 0, pace_k = 0;
  if constexpr (PACED) {
    // the list as a bitmap (a block listed twice is visited once); lane w of every wavefront holds word w
    pace_k = pace_params[0];
    if (tid < 64) rem_bits[tid] = 0;
    __syncthreads();
    for (int t = tid; t < cnt; t += 256) {
      const int jj = min(max(idx[t], 0), M - 1);
      atomicOr(&rem_bits[jj >> 5], 1u << (jj & 31));
    }
    __syncthreads();
    rem = rem_bits[lane];
    int pc = __popc(rem);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) pc += __shfl_xor(pc, o, 64);
    cnt = __builtin_amdgcn_readfirstlane(pc);
  }
  // G: the low 32 bits of the clock times 2^32 / lap wrap once per lap; the high half of that times M is the block
  auto pace_now = [&]() { return (int)__umulhi((uint32_t)__builtin_amdgcn_s_memrealtime() * pace_k, (uint32_t)M); };
  // The first remaining block at or after G, else the first one after the wrap.  Every wavefront runs this on its
  // own copy of the bitmap with the same G, so the four agree without exchanging the result.  Needs rem != 0.
  // G is wave-uniform, so most of this is scalar arithmetic.
  auto pick = [&](int G_any_lane) {
    const int G = __builtin_amdgcn_readfirstlane(G_any_lane);
    const int w0 = G >> 5;
    const uint32_t low = (1u << (G & 31)) - 1u;
    uint32_t mw = lane == w0 ? rem & ~low : rem;
    uint64_t bal = __builtin_amdgcn_ballot_w64(mw != 0) & (~0ull << w0);
    if (bal == 0) {   // nothing left at or after G: every remaining block lies before it
      mw = rem;
      bal = __builtin_amdgcn_ballot_w64(rem != 0);
    }
    const int src = __builtin_ctzll(bal);
    const int bit = __builtin_ctz(__builtin_amdgcn_readlane(mw, src));
    rem &= lane == src ? ~(1u << bit) : ~0u;
    return src * 32 + bit;
  };
  const int steps = 2 * cnt;
  const u32x4* kbase = kp + (size_t)bh * M * TILE_CHUNKS;
  const u32x4* vbase = vp + (size_t)bh * M * TILE_CHUNKS;

  // K half h of block j is one contiguous run of the packed tile; V half h is PH fragments out of
  // every PS of each channel tile: wave w copies fragments f = c*4 + w, f = dt*PH + p2
  const uint32_t ks_wave = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)Ks + (uint32_t)wave * 1024u);
  const uint32_t vs_wave = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)Vs + (uint32_t)wave * 1024u);
  auto k_half_to_lds = [&](int j, int h) {
    const char* kt = (const char*)(kbase + (size_t)j * TILE_CHUNKS + h * HALF_CHUNKS);
#pragma unroll
    for (int c = 0; c < CPT; ++c) dma_1kb_to_lds_at(kt + (size_t)c * 4096, (uint32_t)tid * 16u, ks_wave + c * 4096u);
  };
  auto v_half_to_lds = [&](int j, int h) {
    const u32x4* vt = vbase + (size_t)j * TILE_CHUNKS + (PH * h) * 64;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int f = c * 4 + wave, dt = f / PH, p2 = f % PH;
      dma_1kb_to_lds_at(vt + (size_t)(dt * PS + p2) * 64, (uint32_t)lane * 16u, vs_wave + c * 4096u);
    }
  };

  float m_run = -INFINITY, l_run = 0.f;
  bool unset = true;   // no row has a reference yet (uniform: every row sees the same keys)
  f32x16 O[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[dt][r] = 0.f;
  const uint32_t ks_lane = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)Ks + lane * 16;
  const uint32_t vs_lane = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)Vs + lane * 16;

  // The block index of the next step is fetched a step ahead, and the valid-token count of a
  // block follows from its index, so no step waits on a scalar load it has just issued.
  int j_next = 0;
  if constexpr (PACED) {
    if (tid == 0) pace_slot[0] = pace_now();
    __syncthreads();
    if (cnt > 0) j_next = pick(pace_slot[0]);
  } else {
    if (cnt > 0) j_next = min(max(idx[0], 0), M - 1);
  }
  if (cnt > 0) k_half_to_lds(j_next, 0);

  for (int st = 0; st < steps; ++st) {
    const int h = st & 1;
    const int j = j_next;
    wait_vmem();       // this wave's part of the K half has landed
    __syncthreads();   // K half of this step is in LDS; every wave is past the previous PV
    v_half_to_lds(j, h);

    // S^T = K Q^T for the 64 keys of this step, with the pad keys of a ragged block set to -inf.  Fragments come in
    // groups of four, (m2, ks) = (e & 1, 2g + e / 2); group g + 1 is in flight while the MFMAs of group g run, and
    // the two accumulators alternate.
    f32x16 S[MH];
    const int nv = BLK - (j == M_v - 1 ? pad_v : (j == M - 1 ? pad_c : 0));
    auto logits = [&]() {
#pragma unroll
      for (int m2 = 0; m2 < MH; ++m2)
#pragma unroll
        for (int r = 0; r < 16; ++r) S[m2][r] = 0.f;
      {
        constexpr int NG = KS / 2;
        u32x4 A[2][4];
        static_for<4>([&](auto E) {
          constexpr int e = decltype(E)::value;
          lds_frag<((e & 1) * KS + e / 2) * 1024>(A[0][e], ks_lane);
        });
        static_for<NG>([&](auto G) {
          constexpr int g = decltype(G)::value;
          lds_wait(A[g & 1]);
          if constexpr (g + 1 < NG)
            static_for<4>([&](auto E) {
              constexpr int e = decltype(E)::value;
              lds_frag<((e & 1) * KS + 2 * (g + 1) + e / 2) * 1024>(A[(g + 1) & 1][e], ks_lane);
            });
          static_for<4>([&](auto E) {
            constexpr int e = decltype(E)::value, m2 = e & 1, ks = 2 * g + e / 2;
            S[m2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, A[g & 1][e]), qf[ks], S[m2],
                                                            0, 0, 0);
          });
        });
      }

      if (nv < BLK) {   // sequence-length mask: pad keys of a ragged block
        asm volatile("");   // a real, rarely taken branch
#pragma unroll
        for (int m2 = 0; m2 < MH; ++m2)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kv = 64 * h + 32 * m2 + 8 * (r / 4) + 4 * hl + (r % 4);
            if (kv >= nv) S[m2][r] = -INFINITY;
          }
      }
    };

    // ---- online softmax on S^T (lane = query row, registers = keys) ----
    const float bias = (i < M_v && j >= M_v) ? bias_log2e : 0.f;
    bf16x8 pb[PH];
    // P = 2^(S * scale + off) as bf16 fragments for the second product; returns this lane's sum of them
    auto probabilities = [&](float off) {
      float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
      for (int p2 = 0; p2 < PH; ++p2) {
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(S[p2 >> 1][8 * (p2 & 1) + 2 * e2], scale_log2e, off));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(S[p2 >> 1][8 * (p2 & 1) + 2 * e2 + 1], scale_log2e, off));
          w[e2] = pack_bf16x2(p0, p1);
          rs0 += p0;
          rs1 += p1;
        }
        u32x4 pw = {w[0], w[1], w[2], w[3]};
        pb[p2] = __builtin_bit_cast(bf16x8, pw);
      }
      return rs0 + rs1;
    };
    // the block of the next step, looked up under the arithmetic of this one
    auto advance = [&]() {
      if constexpr (PACED) {
        // G is sampled during the first half step of a block (the clock read has time to return under the
        // softmax) and turned into the next block by every wavefront during the second half step
        if (h == 0) {
          if (tid == 0) pace_slot[((st >> 1) + 1) & 1] = pace_now();
        } else if (st + 1 < steps) {
          j_next = pick(pace_slot[((st >> 1) + 1) & 1]);                 // used after the next barrier
        }
      } else {
        j_next = min(max(idx[min(st + 1, steps - 1) >> 1], 0), M - 1);   // used after the next barrier
      }
    };
    // Common path: probabilities against the reference as it stands, no row maximum (see P_SUM_MAX).  Exact
    // path: the logits again, the reference moved to the row maximum (the rescaling step of Alg. 4), and
    // probabilities <= 1 in place of the first attempt.  Each branch forms and consumes its own S, so S never
    // occupies registers beside a finished P.
    float rs = 0.f;
    bool in_range = false;
    const bool first = unset;
    if (!first) {
      logits();
      advance();
      rs = probabilities(bias - m_run);
      in_range = __ballot(!(rs <= P_SUM_MAX)) == 0;
    }
    if (!in_range) {
      asm volatile("");   // a real branch: the first step of a row, then almost never
      logits();
      if (first) advance();
      float mx = -INFINITY;
#pragma unroll
      for (int m2 = 0; m2 < MH; ++m2)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[m2][r]);
      mx = max_with_other_half(mx);
      const float m_new = fmaxf(m_run, fmaf(mx, scale_log2e, bias));
      const float alpha = m_new == m_run ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= alpha;
      m_run = m_new;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
      rs = probabilities(m_run == -INFINITY ? 0.f : bias - m_run);   // every key so far was padding: keep it finite
      unset = __ballot(m_run == -INFINITY) != 0;
    }
    l_run += rs;

    wait_vmem();       // this wave's part of the V half has landed
    __syncthreads();   // V half is in LDS; every wave is done reading the K half
    if (st + 1 < steps) k_half_to_lds(j_next, (st + 1) & 1);

    // O^T += V^T P^T, fragments (dt, p2) = (2 (g / 2) + (e & 1), 2 (g % 2) + e / 2), pipelined as above
    {
      constexpr int NG = DT;
      u32x4 A[2][4];
      static_for<4>([&](auto E) {
        constexpr int e = decltype(E)::value;
        lds_frag<((e & 1) * PH + e / 2) * 1024>(A[0][e], vs_lane);
      });
      static_for<NG>([&](auto G) {
        constexpr int g = decltype(G)::value;
        lds_wait(A[g & 1]);
        if constexpr (g + 1 < NG)
          static_for<4>([&](auto E) {
            constexpr int e = decltype(E)::value, g1 = g + 1;
            lds_frag<((2 * (g1 / 2) + (e & 1)) * PH + 2 * (g1 % 2) + e / 2) * 1024>(A[g1 & 1][e], vs_lane);
          });
        static_for<4>([&](auto E) {
          constexpr int e = decltype(E)::value, dt = 2 * (g / 2) + (e & 1), p2 = 2 * (g % 2) + e / 2;
          O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, A[g & 1][e]), pb[p2], O[dt],
                                                          0, 0, 0);
        });
      });
    }
  }

  // ---- normalise and store: lane holds row qrow, channels 32*dt + 8*g + 4*hl + {0..3} ----
  // The indices are derived again from the thread index (through an opaque copy, so that they are not the values
  // computed before the loop): kept live across the loop they would cost registers there.
  int tid_e = threadIdx.x;
  asm volatile("" : "+v"(tid_e));
  const int hl_e = (tid_e >> 5) & 1, ql_e = tid_e & 31;
  const int row_e = 32 * wave + ql_e;
  const size_t qrow_e = (size_t)bh * n_pad + (size_t)i * BLK + row_e;
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const int rows_valid = BLK - (i == M_v - 1 ? pad_v : (i == M - 1 ? pad_c : 0));   // = blk_valid[i], without the load
  const bool row_ok = row_e < rows_valid && l_tot > 0.f;
  const float inv = row_ok ? 1.0f / l_tot : 0.f;
  // natural-log sum of exp(logit) over the visited keys: the running maximum is in base-2 units
  if (lse != nullptr && hl_e == 0)
    lse[qrow_e] = row_ok ? (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
  uint16_t* orow = out + qrow_e * D;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 w;
      w.x = row_ok ? pack_bf16x2(O[dt][4 * g] * inv, O[dt][4 * g + 1] * inv) : 0u;
      w.y = row_ok ? pack_bf16x2(O[dt][4 * g + 2] * inv, O[dt][4 * g + 3] * inv) : 0u;
      *(uint2*)(orow + 32 * dt + 8 * g + 4 * hl_e) = w;
    }
}

// Lap of the paced walk, common to all workgroups of a launch: a fixed fraction of the time a workgroup needs for
// a list of mean length (a tuning constant: between 0.45 and 0.9 the measured time is flat, at 1.0 and above the
// workgroups run ahead of the sweep and the gain goes).  Writes 2^32 / lap (in ticks of
// the 100 MHz clock) to params[0].  One workgroup.
#ifndef JENGA_PACE_FACTOR
#define JENGA_PACE_FACTOR 0.6f
#endif
__global__ __launch_bounds__(1024) void walk_pace_kernel(const int32_t* __restrict__ sel_count, int n_rows, int M,
                                                         float ticks_per_block, uint32_t* __restrict__ params) {
  __shared__ float part[16];
  float s = 0.f;
  for (int t0 = threadIdx.x; t0 < n_rows; t0 += 4096) {   // four loads in flight per thread
    int c[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) c[u] = t0 + u * 1024 < n_rows ? sel_count[t0 + u * 1024] : 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) s += (float)min(max(c[u], 0), M);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float total = 0.f;
    for (int w = 0; w < 16; ++w) total += part[w];
    const float mean = total / (float)max(n_rows, 1);
    const float lap = fminf(fmaxf(JENGA_PACE_FACTOR * mean * ticks_per_block, 1024.f), 1e9f);
    params[0] = (uint32_t)(4294967296.0 / (double)lap);
  }
}

template <int BLK, int D>
int run_pack(const jenga_plan* p, const void* k, const void* v, void* ws, hipStream_t st) {
  const jenga_config& c = p->cfg;
  const jenga_plan_info_t& f = p->info;
  const int bh = c.batch * c.heads;
  const size_t half = (((size_t)bh * f.N_pad * D * 2) + 255) & ~(size_t)255;
  uint4* kp = (uint4*)ws;
  uint4* vp = (uint4*)((char*)ws + half);
  pack_kernel<BLK, D><<<dim3(f.M, bh), 256, 0, st>>>((const uint16_t*)k, (const uint16_t*)v, kp, vp,
                                                     p->d_blk_valid, f.M, f.N_pad);
  return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_EHIP;
}

template <int BLK, int D>
int run_attention(const jenga_plan* p, const void* q, void* ws, const int32_t* sel_count,
                  const int32_t* sel_index, void* out, float* lse, hipStream_t st) {
  const jenga_config& c = p->cfg;
  const jenga_plan_info_t& f = p->info;
  const int bh = c.batch * c.heads;
  const size_t half = (((size_t)bh * f.N_pad * D * 2) + 255) & ~(size_t)255;
  const u32x4* kp = (const u32x4*)ws;
  const u32x4* vp = (const u32x4*)((const char*)ws + half);
  const int chunk = (f.M_v + 7) / 8;                      // vision query blocks per XCD and head
  const int n_wg = bh * f.M_c + bh * 8 * chunk;           // text blocks first, then the vision runs
  const float log2e = 1.4426950408889634f;
  const float scale = log2e / sqrtf((float)D);
  if constexpr (BLK == 128) {
    if (c.flags & JENGA_FLAG_PACED_WALK) {
      // a workgroup spends about 6.3 us (D = 128; 3.6 us at D = 64) on a block of 128 keys when three share a CU
      uint32_t* params = (uint32_t*)((char*)ws + 2 * half);
      walk_pace_kernel<<<1, 1024, 0, st>>>(sel_count, bh * f.M, f.M, D == 128 ? 630.f : 360.f, params);
      attn_h_kernel<D, true><<<dim3(n_wg), 256, 0, st>>>((const uint16_t*)q, kp, vp, sel_count, sel_index,
                                                         p->d_blk_valid, (uint16_t*)out, lse, bh, f.M, f.M_v, f.N_pad,
                                                         chunk, f.pad_v, f.pad_c, scale, c.text_bias * log2e, params);
    } else {
      attn_h_kernel<D, false><<<dim3(n_wg), 256, 0, st>>>((const uint16_t*)q, kp, vp, sel_count, sel_index,
                                                          p->d_blk_valid, (uint16_t*)out, lse, bh, f.M, f.M_v,
                                                          f.N_pad, chunk, f.pad_v, f.pad_c, scale,
                                                          c.text_bias * log2e, nullptr);
    }
  }
  else
    attn_kernel<BLK, D><<<dim3(n_wg), AttnTraits<BLK, D>::NTHR, 0, st>>>(
        (const uint16_t*)q, kp, vp, sel_count, sel_index, p->d_blk_valid, (uint16_t*)out, lse, bh, f.M, f.M_v,
        f.N_pad, chunk, scale, c.text_bias * log2e);   // blocks of 32 or 64 tokens: in-order walk only
  return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_EHIP;
}

}  // namespace

namespace jenga {

#define JENGA_FOR_SHAPES(X) X(128, 128) X(64, 128) X(32, 128) X(128, 64) X(64, 64) X(32, 64)

int launch_pack(const jenga_plan* p, const void* k, const void* v, void* ws, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  const int blk = p->cfg.block, d = p->cfg.head_dim;
#define X(B, DD) \
  if (blk == B && d == DD) return run_pack<B, DD>(p, k, v, ws, st);
  JENGA_FOR_SHAPES(X)
#undef X
  return JENGA_EUNSUPPORTED;
}

int launch_attention(const jenga_plan* p, const void* q, void* ws, const int32_t* sel_count,
                     const int32_t* sel_index, void* out, float* lse, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  const int blk = p->cfg.block, d = p->cfg.head_dim;
#define X(B, DD) \
  if (blk == B && d == DD) return run_attention<B, DD>(p, q, ws, sel_count, sel_index, out, lse, st);
  JENGA_FOR_SHAPES(X)
#undef X
  return JENGA_EUNSUPPORTED;
}

}  // namespace jenga
