// The host-only half of the C ABI (see include/jenga.h): configuration checks, plan tables without a
// device, table export, status strings.  No HIP in this file, so that it can be built and run under
// the host sanitizers together with jenga_plan.cpp.
#include <cmath>
#include <cstring>
#include <new>

#include "jenga_internal.h"

namespace jenga {

bool config_ok(const jenga_config& c, int* why) {
  *why = JENGA_EINVAL;
  if (c.T < 1 || c.H < 1 || c.W < 1 || c.n_text < 0 || c.batch < 1 || c.heads < 1) return false;
  if (!(c.topk_ratio > 0.0 && c.topk_ratio <= 1.0)) return false;
  if (!(c.cum_prob >= 0.0 && c.cum_prob < 1.0)) return false;
  if (!std::isfinite(c.text_bias)) return false;   // NaN and +-inf: exp2(-inf + inf) would poison a row
  if (c.flags & ~15u) return false;
  *why = JENGA_EUNSUPPORTED;
  if (c.head_dim != 64 && c.head_dim != 128) return false;
  if (c.block != 32 && c.block != 64 && c.block != 128) return false;
  // at most 2^24 vision tokens; multiply step by step so that no product can overflow
  const long long lim = 1ll << 24;
  if (c.T > lim || c.H > lim || c.W > lim || (long long)c.T * c.H > lim) return false;
  const long long nv = (long long)c.T * c.H * c.W;
  if (nv > lim || c.n_text > (1 << 20)) return false;
  const long long M = (nv + c.block - 1) / c.block + (c.n_text + c.block - 1) / c.block;
  if (M > 2048) return false;   // select keeps a row of M block probabilities in one wavefront
  if ((long long)c.batch * c.heads > 65535) return false;
  return true;
}

}  // namespace jenga

extern "C" {

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
  if (rc == JENGA_OK) {
    *info = p->info;
    rc = jenga_plan_export(p, perm, inv_perm, adja);
  }
  delete p;
  return rc;
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
