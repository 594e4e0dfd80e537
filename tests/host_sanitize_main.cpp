// Test driver for the host half of the library under AddressSanitizer and UndefinedBehaviorSanitizer
// (CPU only).  Reads configurations from stdin, one per line:
//     T H W n_text batch heads head_dim block topk_ratio cum_prob text_bias flags
// calls jenga_plan_tables for each and prints one line per configuration:
//     status N_v M_v M_c M N_pad pad_v pad_c K_top fnv(perm) fnv(inv_perm) fnv(adja)
// (64-bit FNV-1a hashes of the exported tables, 0 when the call fails).  Any sanitizer report aborts
// the process with a non-zero exit code.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "jenga.h"

static uint64_t fnv(const void* data, size_t bytes) {
  const unsigned char* p = (const unsigned char*)data;
  uint64_t h = 1469598103934665603ull;
  for (size_t i = 0; i < bytes; ++i) {
    h ^= p[i];
    h *= 1099511628211ull;
  }
  return h;
}

int main() {
  jenga_config c;
  double k, pr;
  float beta;
  unsigned flags;
  while (std::scanf("%d %d %d %d %d %d %d %d %lf %lf %f %u", &c.T, &c.H, &c.W, &c.n_text, &c.batch, &c.heads,
                    &c.head_dim, &c.block, &k, &pr, &beta, &flags) == 12) {
    c.topk_ratio = k;
    c.cum_prob = pr;
    c.text_bias = beta;
    c.flags = flags;
    jenga_plan_info_t info = {};
    // first without tables (also tells the sizes), then with exactly sized tables so that any
    // write past the end is caught by the sanitizer's red zones
    int rc = jenga_plan_tables(&c, &info, nullptr, nullptr, nullptr);
    uint64_t hp = 0, hi = 0, ha = 0;
    if (rc == JENGA_OK) {
      std::vector<int32_t> perm(info.N_v), inv(info.N_v);
      std::vector<uint8_t> adja((size_t)info.M_v * info.M_v);
      rc = jenga_plan_tables(&c, &info, perm.data(), inv.data(), adja.data());
      hp = fnv(perm.data(), perm.size() * 4);
      hi = fnv(inv.data(), inv.size() * 4);
      ha = fnv(adja.data(), adja.size());
    }
    std::printf("%d %d %d %d %d %d %d %d %d %llu %llu %llu\n", rc, info.N_v, info.M_v, info.M_c, info.M, info.N_pad,
                info.pad_v, info.pad_c, info.K_top, (unsigned long long)hp, (unsigned long long)hi,
                (unsigned long long)ha);
    std::printf("%s\n", jenga_strerror(rc));
  }
  // null-argument paths of the host entry points
  std::printf("null %d %d %d\n", jenga_plan_tables(nullptr, nullptr, nullptr, nullptr, nullptr),
              jenga_plan_info(nullptr, nullptr), jenga_plan_export(nullptr, nullptr, nullptr, nullptr));
  return 0;
}
