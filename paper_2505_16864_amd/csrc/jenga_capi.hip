// The device half of the C ABI (see include/jenga.h): plan life cycle on the device, argument validation of
// the hot calls, dispatch to the launchers.  The host-only entry points live in jenga_host.cpp.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>

#include "jenga_internal.h"

namespace {

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
  if (!jenga::config_ok(*cfg, &why)) return why;
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
  if (rc == JENGA_OK) rc = jenga::select_scratch_init(p->device);
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

int jenga_block_sparse_attn_packed(const jenga_plan* p, const void* q, void* packed_kv_workspace,
                                   size_t workspace_bytes, const int32_t* sel_count, const int32_t* sel_index,
                                   void* out_curve, float* lse_or_null, void* stream) {
  if (!p || !q || !packed_kv_workspace || !sel_count || !sel_index || !out_curve) return JENGA_EINVAL;
  if (!on_plan_device(p)) return JENGA_EINVAL;
  if (((uintptr_t)packed_kv_workspace & 255u) != 0) return JENGA_EINVAL;
  if (workspace_bytes < p->info.attn_workspace_bytes) return JENGA_EWORKSPACE;
  return jenga::launch_attention(p, q, packed_kv_workspace, sel_count, sel_index, out_curve, lse_or_null, stream);
}

}  // extern "C"
