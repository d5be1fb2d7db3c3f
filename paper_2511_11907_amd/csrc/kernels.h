// Internal launch interface between the C-ABI layer (api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/kvswap_hip.h"

namespace kvs {

// Work granules of the streaming kernels (units = wave-wide 1 KiB loads).
constexpr int kPredictUnitsPerWgStep = 4 * 8;  // 4 waves x 8 loads in flight
constexpr int kAttnUnitsPerWgStep = 4 * 4;     // 4 waves x 4 (K,V) load pairs in flight

// Launch geometry derived from the params alone (the host computes it once per
// call; kvs_workspace_bytes uses the same numbers).
struct Plan {
  int problems;          // P = B * H_kv
  int n_groups;          // NG = N / G
  int q_per_kv;          // H_q / H_kv
  // predict
  int meta_lanes_per_row;   // lanes of 16 B that cover one K_lr row
  int meta_rows_per_unit;   // rows covered by one wave-wide 1 KiB load
  int predict_units;        // wave-loads per problem
  int predict_units_per_wg;
  int predict_chunks;       // workgroups per problem
  // attention
  int kv_lanes_per_tok;     // lanes of 16 B that cover one K (or V) row
  int kv_toks_per_unit;     // tokens covered by one wave-wide load
  int attn_units;           // wave-loads (of K, and as many of V) per problem
  int attn_units_per_split;
  int attn_splits;          // workgroups per problem
  // workspace layout (byte offsets, 256-byte aligned)
  size_t off_gs, off_part_ml, off_part_o, total_bytes;
};

Plan make_plan(const kvs_params& p);

hipError_t launch_build_metadata(const kvs_params& p, const Plan& pl, const void* K,
                                 const float* A, void* K_lr, hipStream_t st);
hipError_t launch_predict(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                          const float* A, float* gs, hipStream_t st);
hipError_t launch_topk(const kvs_params& p, const Plan& pl, const float* gs, int32_t* idx,
                       hipStream_t st);
hipError_t launch_attn(const kvs_params& p, const Plan& pl, const void* q, const void* K,
                       const void* V, const int32_t* idx, float* part_ml, float* part_o,
                       hipStream_t st);
hipError_t launch_combine(const kvs_params& p, const Plan& pl, const float* part_ml,
                          const float* part_o, void* out, hipStream_t st);

}  // namespace kvs
