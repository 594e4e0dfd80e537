// Internal declarations shared by the host plan code and the HIP translation units.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>
#include "jenga.h"

struct jenga_plan {
  jenga_config cfg;
  jenga_plan_info_t info;
  int device;
  int nt64;  // 64-bit words per row of the fixed-mask table: ceil(M / 64)
  // host tables
  std::vector<int32_t> perm, inv_perm;
  std::vector<int32_t> src_of_pos;  // [N_pad] index into the thw-side sequence, -1 for a pad
  std::vector<int32_t> blk_valid;   // [M] valid tokens per block
  std::vector<uint64_t> fixed_bits; // [M_v][nt64] adjacency and condition bits per query block
  // device copies
  int32_t* d_src_of_pos;
  int32_t* d_blk_valid;
  uint64_t* d_fixed_bits;
};

namespace jenga {

// Validates a configuration; on failure *why is the jenga_status to return.
bool config_ok(const jenga_config& c, int* why);

// Curve order of a T x H x W grid: fills cells with the thw index of each curve position.
void curve_order(int T, int H, int W, bool use_curve, std::vector<int32_t>& perm);

// Host tables of a plan (no device work).  Returns a jenga_status.
int build_host_tables(jenga_plan* plan);

// Kernel launchers (defined in the .hip files).  All return a jenga_status.
int launch_permute(const jenga_plan* p, const void* src, void* dst, bool forward, void* stream);
int launch_permute_rows(const jenga_plan* p, const void* src, void* dst, int row_bytes, void* stream);
int launch_select(const jenga_plan* p, const void* q, const void* k, int32_t* sel_count,
                  int32_t* sel_index, uint8_t* mask, void* ws, void* stream);
// Looks up the address of the static selection scratch on `device` (the current device) once.
int select_scratch_init(int device);
int launch_pack(const jenga_plan* p, const void* k, const void* v, void* ws, void* stream);
int launch_attention(const jenga_plan* p, const void* q, void* packed_ws, const int32_t* sel_count,
                     const int32_t* sel_index, void* out, float* lse, void* stream);

}  // namespace jenga
