// The C ABI (see include/jenga.h): argument validation, plan life cycle, dispatch to the launchers.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <new>

#include "jenga_internal.h"

namespace {

bool config_ok(const jenga_config& c, int* why) {
  *why = JENGA_EINVAL;
  if (c.T < 1 || c.H < 1 || c.W < 1 || c.n_text < 0 || c.batch < 1 || c.heads < 1) return false;
  if (!(c.topk_ratio > 0.0 && c.topk_ratio <= 1.0)) return false;
  if (!(c.cum_prob >= 0.0 && c.cum_prob < 1.0)) return false;
  if (!std::isfinite(c.text_bias)) return false;   // NaN and +-inf: exp2(-inf + inf) would poison a row
  if (c.flags & ~7u) return false;
  *why = JENGA_EUNSUPPORTED;
  if (c.head_dim != 64 && c.head_dim != 128) return false;
  if (c.block != 32 && c.block != 64 && c.block != 128) return false;
  const long long nv = (long long)c.T * c.H * c.W;
  if (nv > (1ll << 24) || c.n_text > (1 << 20)) return false;
  const long long M = (nv + c.block - 1) / c.block + (c.n_text + c.block - 1) / c.block;
  if (M > 2048) return false;   // select keeps a row of M block probabilities in one wavefront
  if ((long long)c.batch * c.heads > 65535) return false;
  return true;
}

// The plan's tables live on the device that was current at creation; a hot call made with another
// device current would launch there with pointers that device cannot read.
bool on_plan_device(const jenga_plan* p) {
  int dev = -1;
  return hipGetDevice(&dev) == hipSuccess && dev == p->device;
}

template <typename T>
int to_device(const std::vector<T>& h, T** d) {
  *d = nullptr;
  const size_t bytes = (h.size() ? h.size() : 1) * sizeof(T);
  if (hipMalloc((void**)d, bytes) != hipSuccess) return JENGA_ENOMEM;
  if (!h.empty() && hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess)
    return JENGA_EHIP;
  return JENGA_OK;
}

}  // namespace

extern "C" {

int jenga_plan_create(const jenga_config* cfg, jenga_plan** out) {
  if (!cfg || !out) return JENGA_EINVAL;
  *out = nullptr;
  int why;
  if (!config_ok(*cfg, &why)) return why;
  jenga_plan* p = new (std::nothrow) jenga_plan();
  if (!p) return JENGA_ENOMEM;
  p->cfg = *cfg;
  p->d_src_of_pos = nullptr;
  p->d_blk_valid = nullptr;
  p->d_fixed_bits = nullptr;
  int rc = JENGA_OK;
  try {
    rc = jenga::build_host_tables(p);
  } catch (const std::bad_alloc&) {
    rc = JENGA_ENOMEM;
  }
  if (rc == JENGA_OK && hipGetDevice(&p->device) != hipSuccess) rc = JENGA_EHIP;
  if (rc == JENGA_OK) rc = to_device(p->src_of_pos, &p->d_src_of_pos);
  if (rc == JENGA_OK) rc = to_device(p->blk_valid, &p->d_blk_valid);
  if (rc == JENGA_OK) rc = to_device(p->fixed_bits, &p->d_fixed_bits);
  if (rc != JENGA_OK) {
    jenga_plan_destroy(p);
    return rc;
  }
  *out = p;
  return JENGA_OK;
}

int jenga_plan_destroy(jenga_plan* p) {
  if (!p) return JENGA_OK;
  int rc = JENGA_OK;
  if (p->d_src_of_pos && hipFree(p->d_src_of_pos) != hipSuccess) rc = JENGA_EHIP;
  if (p->d_blk_valid && hipFree(p->d_blk_valid) != hipSuccess) rc = JENGA_EHIP;
  if (p->d_fixed_bits && hipFree(p->d_fixed_bits) != hipSuccess) rc = JENGA_EHIP;
  delete p;
  return rc;
}

int jenga_plan_info(const jenga_plan* p, jenga_plan_info_t* info) {
  if (!p || !info) return JENGA_EINVAL;
  *info = p->info;
  return JENGA_OK;
}

int jenga_plan_export(const jenga_plan* p, int32_t* perm, int32_t* inv_perm, uint8_t* adja) {
  if (!p) return JENGA_EINVAL;
  const size_t nv = (size_t)p->info.N_v;
  if (perm) std::memcpy(perm, p->perm.data(), nv * sizeof(int32_t));
  if (inv_perm) std::memcpy(inv_perm, p->inv_perm.data(), nv * sizeof(int32_t));
  if (adja) {
    const int mv = p->info.M_v;
    const bool on = (p->cfg.flags & JENGA_FLAG_ADJACENCY) != 0;
    for (int i = 0; i < mv; ++i)
      for (int j = 0; j < mv; ++j)
        adja[(size_t)i * mv + j] =
            on ? (uint8_t)((p->fixed_bits[(size_t)i * p->nt64 + (j >> 6)] >> (j & 63)) & 1ull) : 0;
  }
  return JENGA_OK;
}

int jenga_plan_tables(const jenga_config* cfg, jenga_plan_info_t* info, int32_t* perm, int32_t* inv_perm,
                      uint8_t* adja) {
  if (!cfg || !info) return JENGA_EINVAL;
  int why;
  if (!config_ok(*cfg, &why)) return why;
  jenga_plan* p = new (std::nothrow) jenga_plan();
  if (!p) return JENGA_ENOMEM;
  p->cfg = *cfg;
  p->d_src_of_pos = nullptr;
  p->d_blk_valid = nullptr;
  p->d_fixed_bits = nullptr;
  int rc = JENGA_OK;
  try {
    rc = jenga::build_host_tables(p);
  } catch (const std::bad_alloc&) {
    rc = JENGA_ENOMEM;
  }
  if (rc == JENGA_OK) {
    *info = p->info;
    rc = jenga_plan_export(p, perm, inv_perm, adja);
  }
  delete p;
  return rc;
}

int jenga_curve_permute(const jenga_plan* p, const void* src_thw, void* dst_curve, void* stream) {
  if (!p || !src_thw || !dst_curve) return JENGA_EINVAL;
  if (!on_plan_device(p)) return JENGA_EINVAL;
  return jenga::launch_permute(p, src_thw, dst_curve, true, stream);
}

int jenga_curve_permute_rows(const jenga_plan* p, const void* src_rows, void* dst_rows, int32_t row_bytes,
                             void* stream) {
  if (!p || !src_rows || !dst_rows) return JENGA_EINVAL;
  if (!on_plan_device(p)) return JENGA_EINVAL;
  if (row_bytes < 16 || row_bytes > 4096 || (row_bytes & (row_bytes - 1)) != 0) return JENGA_EUNSUPPORTED;
  return jenga::launch_permute_rows(p, src_rows, dst_rows, row_bytes, stream);
}

int jenga_unpermute(const jenga_plan* p, const void* src_curve, void* dst_thw, void* stream) {
  if (!p || !src_curve || !dst_thw) return JENGA_EINVAL;
  if (!on_plan_device(p)) return JENGA_EINVAL;
  return jenga::launch_permute(p, src_curve, dst_thw, false, stream);
}

int jenga_select_blocks(const jenga_plan* p, const void* q_curve, const void* k_curve, int32_t* sel_count,
                        int32_t* sel_index, uint8_t* mask_or_null, void* workspace, size_t workspace_bytes,
                        void* stream) {
  if (!p || !q_curve || !k_curve || !sel_count || !sel_index || !workspace) return JENGA_EINVAL;
  if (!on_plan_device(p)) return JENGA_EINVAL;
  if (((uintptr_t)workspace & 255u) != 0) return JENGA_EINVAL;
  if (workspace_bytes < p->info.select_workspace_bytes) return JENGA_EWORKSPACE;
  return jenga::launch_select(p, q_curve, k_curve, sel_count, sel_index, mask_or_null, workspace, stream);
}

int jenga_block_sparse_attn(const jenga_plan* p, const void* q, const void* k, const void* v,
                            const int32_t* sel_count, const int32_t* sel_index, void* out_curve,
                            float* lse_or_null, void* workspace, size_t workspace_bytes, void* stream) {
  if (!p || !q || !k || !v || !sel_count || !sel_index || !out_curve || !workspace) return JENGA_EINVAL;
  if (!on_plan_device(p)) return JENGA_EINVAL;
  if (((uintptr_t)workspace & 255u) != 0) return JENGA_EINVAL;
  if (workspace_bytes < p->info.attn_workspace_bytes) return JENGA_EWORKSPACE;
  const int rc = jenga::launch_pack(p, k, v, workspace, stream);
  if (rc != JENGA_OK) return rc;
  return jenga::launch_attention(p, q, workspace, sel_count, sel_index, out_curve, lse_or_null, stream);
}

int jenga_pack_kv(const jenga_plan* p, const void* k, const void* v, void* workspace, size_t workspace_bytes,
                  void* stream) {
  if (!p || !k || !v || !workspace) return JENGA_EINVAL;
  if (!on_plan_device(p)) return JENGA_EINVAL;
  if (((uintptr_t)workspace & 255u) != 0) return JENGA_EINVAL;
  if (workspace_bytes < p->info.attn_workspace_bytes) return JENGA_EWORKSPACE;
  return jenga::launch_pack(p, k, v, workspace, stream);
}

int jenga_block_sparse_attn_packed(const jenga_plan* p, const void* q, const void* packed_kv_workspace,
                                   size_t workspace_bytes, const int32_t* sel_count, const int32_t* sel_index,
                                   void* out_curve, float* lse_or_null, void* stream) {
  if (!p || !q || !packed_kv_workspace || !sel_count || !sel_index || !out_curve) return JENGA_EINVAL;
  if (!on_plan_device(p)) return JENGA_EINVAL;
  if (((uintptr_t)packed_kv_workspace & 255u) != 0) return JENGA_EINVAL;
  if (workspace_bytes < p->info.attn_workspace_bytes) return JENGA_EWORKSPACE;
  return jenga::launch_attention(p, q, packed_kv_workspace, sel_count, sel_index, out_curve, lse_or_null, stream);
}

const char* jenga_strerror(int status) {
  switch (status) {
    case JENGA_OK: return "ok";
    case JENGA_EINVAL: return "invalid argument";
    case JENGA_EUNSUPPORTED: return "configuration not supported by this build";
    case JENGA_EWORKSPACE: return "workspace too small";
    case JENGA_EHIP: return "HIP runtime or kernel launch failure";
    case JENGA_ENOMEM: return "out of memory";
    default: return "unknown status";
  }
}

}  // extern "C"
