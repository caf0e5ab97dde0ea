// Argument blocks and launchers shared by the C-ABI layer and the HIP kernels.
#pragma once
#include <cstdint>

#include <hip/hip_runtime_api.h>

namespace ellm {

constexpr int MAX_LAUNCH_REQ = 256;   // requests described by one launch's kernel arguments
constexpr int MAX_PATCH = 448;        // table entries patched by one launch

// what a kernel needs to turn (tensor, token) into an address
struct PoolView {
  char* base;                 // device pool
  const int32_t* table;       // device mirror of the chunk tables, [max_tensors][max_slots]
  uint32_t chunk_bytes;
  int32_t tokens_per_chunk;
  int32_t max_slots;
  int32_t n_q_heads, n_kv_heads, head_dim, group;
};

// one decode launch: requests [q_row0, q_row0 + n_req) of the caller's batch
struct BatchArgs {
  int32_t n_req, n_items;     // n_items = work items of these requests
  int32_t item_base;          // first workspace item of this launch
  int32_t q_row0;             // row of the first request in q / out
  int32_t tensor[MAX_LAUNCH_REQ];
  int32_t len[MAX_LAUNCH_REQ];
  int32_t item0[MAX_LAUNCH_REQ];   // first work item of request b, relative to this launch
};

struct AppendArgs {
  int32_t n_req, total_new;
  int32_t tensor[MAX_LAUNCH_REQ];
  int32_t len_before[MAX_LAUNCH_REQ];
  int32_t tok0[MAX_LAUNCH_REQ];    // first new-token row of request b, relative to this launch
};

struct PatchArgs {
  int32_t n;
  int32_t idx[MAX_PATCH];
  int32_t val[MAX_PATCH];
};

// each returns 0 or a hipError_t value
int launch_table_patch(int32_t* table, const PatchArgs& a, hipStream_t stream);
int launch_kv_append(const PoolView& pv, const void* k_new, const void* v_new, const AppendArgs& a,
                     hipStream_t stream);
int launch_decode(const PoolView& pv, const void* q, void* out, float* ws, float scale_log2, int32_t split_tokens,
                  const BatchArgs& a, hipStream_t stream);

}  // namespace ellm
