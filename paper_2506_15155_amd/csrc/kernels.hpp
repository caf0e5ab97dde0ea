// Argument blocks and launchers shared by the C-ABI layer and the HIP kernels.
#pragma once
#include <cstdint>

#include <hip/hip_runtime_api.h>

namespace ellm {

constexpr int MAX_LAUNCH_REQ = 128;   // requests described by one launch's kernel arguments (4 KB in all)
constexpr int MAX_PIECE_REQ = 512;    // pieces per kv head that the request lookup table covers
constexpr int MAX_PATCH = 448;        // table entries patched by one launch
constexpr int TILE_TOKENS = 64;       // rows of K (and V) one wave handles at a time
constexpr int WS_ROW_PAD = 4;         // a partial row is head_dim accumulators, m, l and 2 unused floats

// what a kernel needs to turn (tensor, token) into an address
struct PoolView {
  char* base;                 // device pool
  const int32_t* table;       // device mirror of the chunk tables, [max_tensors][max_slots]
  uint32_t chunk_bytes;
  int32_t tokens_per_chunk;
  int32_t tiles_per_chunk;    // ceil(tokens_per_chunk / TILE_TOKENS); a tile never straddles a chunk
  int32_t max_slots;
  int32_t n_q_heads, n_kv_heads, head_dim, group;
};

// One decode launch: requests [q_row0, q_row0 + n_req) of the caller's batch.
// The tiles of every (request, kv head) pair are cut into pieces, one wave and one partial result
// each: first n_big "big" pieces of tiles_big tiles, then the remaining tiles in "small" pieces of
// tiles_small tiles (the last one may be shorter). The grid runs all big pieces first, kv head
// major (index g * big_per_head + big_prefix[b] + j), then all small pieces in the same order: the
// big pieces fill the GPU once, and the small ones are handed out by the hardware dispatcher as
// waves finish, which evens out waves and compute units that run at different speeds. Partial j of
// a pair is big piece j, or small piece j - n_big; the cut is fixed by the plan, so results do not
// depend on which wave ran when.
struct BatchArgs {
  int32_t n_req;
  int32_t q_row0;             // row of the first request in q / out
  int32_t big_per_head;       // = big_prefix[n_req]
  int32_t small_per_head;     // = small_prefix[n_req]
  int32_t tiles_big, tiles_small;
  int32_t max_partials;       // partial slots per (request, kv head) = most pieces any request has
  int32_t ws_slot0;           // first partial slot of this launch in the workspace
  int32_t use_piece_req;      // piece_req is filled in (big_per_head + small_per_head <= MAX_PIECE_REQ)
  int32_t pad;
  // request of piece i of a kv head (big pieces first, then small ones), one byte each: lets a wave
  // find its request with one scalar load instead of a search through the prefix arrays
  uint32_t piece_req[MAX_PIECE_REQ / 4];
  // per request, one record, so that a wave gets all of it with one round of scalar loads
  struct Req {
    int32_t len, tensor;
    int32_t big_prefix, small_prefix;   // pieces of the requests before this one, per phase
    int32_t n_big, n_small;             // this request's pieces, per phase
  } req[MAX_LAUNCH_REQ];
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

// resident waves of the partial-pass kernel per compute unit (occupancy query), per (head_dim, group)
int partial_waves_per_cu(int head_dim, int group);

// each returns 0 or a hipError_t value
int launch_table_patch(int32_t* table, const PatchArgs& a, hipStream_t stream);
int launch_kv_append(const PoolView& pv, const void* k_new, const void* v_new, const AppendArgs& a,
                     hipStream_t stream);
// k_new / v_new non-NULL: fused append. a.len then counts one token per request whose K/V row
// ([request][kv head][dim], rows q_row0 .. of the caller's batch) is still in k_new / v_new; the
// kernel uses it from there and writes it into the chunk.
int launch_decode_partial(const PoolView& pv, const void* q, const void* k_new, const void* v_new, float* ws,
                          float scale_log2, const BatchArgs& a, hipStream_t stream);
int launch_decode_combine(const PoolView& pv, const float* ws, void* out, const BatchArgs& a, hipStream_t stream);

// calibration (measurement only)
int launch_copy(void* dst, const void* src, int64_t bytes, hipStream_t stream);
int launch_read(const void* src, int64_t bytes, uint32_t* sink, hipStream_t stream);
int launch_kv_stream(const PoolView& pv, uint32_t* sink, const BatchArgs& a, hipStream_t stream);

}  // namespace ellm
