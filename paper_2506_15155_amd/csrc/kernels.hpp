// Argument blocks and launchers shared by the C-ABI layer and the HIP kernels.
#pragma once
#include <cstddef>
#include <cstdint>

#include <hip/hip_runtime_api.h>

namespace ellm {

constexpr int MAX_LAUNCH_REQ = 128;   // requests described by one launch's kernel arguments (4 KB in all)
constexpr int MAX_WAVE_REQ = 512;     // waves per kv head that the request lookup table covers
constexpr int MAX_PATCH = 448;        // table entries patched by one launch
constexpr int TILE_TOKENS = 64;       // rows of K (and V) one wave handles at a time
constexpr int SIMDS_PER_CU = 4;       // a decode launch runs one wave on each SIMD
constexpr int WS_ML = 2;              // floats per partial and q head in the (m, l) region of the workspace
constexpr size_t STATIC_WS_BYTES = 16u << 20;   // the fixed workspace of the entry point that allocates nothing

// what a kernel needs to turn (tensor, token) into an address
struct PoolView {
  char* base;                 // device pool
  const int32_t* table;       // device mirror of the chunk tables, [max_tensors][max_slots]
  const uint64_t* vbase;      // NULL: kernels go through the table. Else: per tensor, the start of its virtual
                              // address range, into which the driver has mapped its chunks; kernels read that
  uint32_t chunk_bytes;
  int32_t tokens_per_chunk;
  int32_t tiles_per_chunk;    // ceil(tokens_per_chunk / TILE_TOKENS); a tile never straddles a chunk
  int32_t max_slots;
  int32_t n_q_heads, n_kv_heads, head_dim, group;
};

// One decode launch: requests [q_row0, q_row0 + n_req) of the caller's batch.
// For every kv head the tiles of all requests, laid end to end in request order, form one sequence
// of tiles_per_head tiles, which is dealt out evenly to waves_per_head waves: wave w takes
// tiles_each tiles, the first tiles_extra waves one more, each from where the wave before it
// stopped. A wave whose share runs from one request into the next finishes a result for each; so
// request b is covered by n_part waves per kv head, numbered from the wave that holds its first
// tile (wave_first). A request that lies wholly inside one wave's share (n_part == 1) needs no
// second pass: that wave normalises and writes the output row itself. Only the others ("split"
// requests) get partial results in the workspace, part0 + j for the j-th wave, and a combine pass.
// A launch has one wave for every SIMD of the GPU (a second wave on a SIMD is served markedly
// worse than the first and slows both down): all are resident at once and have the same amount to
// read, so none waits for a slot and none is left over at the end. The cut is fixed by the plan,
// so results do not depend on which wave ran when.
//
// Workspace of a launch, from the pointer the launch is given: accumulator rows
// [kv head][partial slot of the head][q head of the group][D] fp32 (ws_slots = n_kv_heads *
// parts_per_head slots in all), then the (m, l) pairs in the same order, WS_ML floats each.
struct BatchArgs {
  int32_t n_req;
  int32_t q_row0;             // row of the first request in q / out
  int32_t tiles_per_head;     // tiles of all requests of the launch, for one kv head
  int32_t waves_per_head;     // <= tiles_per_head
  int32_t tiles_each, tiles_extra;   // tiles_per_head = waves_per_head * tiles_each + tiles_extra
  int32_t parts_per_head;     // partial slots per kv head = sum of n_part over the split requests
  int32_t ws_slots;           // n_kv_heads * parts_per_head
  int32_t use_wave_req;       // wave_req is filled in (waves_per_head <= MAX_WAVE_REQ)
  int32_t n_split_req;        // requests with n_part > 1: the combine pass runs for these only
  // request that holds the first tile of wave w of a kv head, one byte each: lets a wave find its
  // request with one scalar load instead of a search through the prefix entries
  uint32_t wave_req[MAX_WAVE_REQ / 4];
  // the split requests in ascending order, one byte each
  uint32_t split_req[MAX_LAUNCH_REQ / 4];
  // per request, one record, so that a wave gets all of it with one round of scalar loads
  struct Req {
    int32_t len, tensor;
    int32_t tile_prefix;      // tiles of the requests before this one
    int32_t wave_first;       // wave that holds this request's first tile
    int32_t n_part;           // waves that hold tiles of this request
    int32_t part0;            // first partial slot of the request within a kv head's slots (split requests)
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

// chunks copied by one launch between the pool and the pinned host buffer: move i is device chunk
// chunk[i] <-> host slot host_slot[i]
constexpr int MAX_COPY = 480;
struct CopyArgs {
  int32_t n;
  int32_t chunk[MAX_COPY];
  int32_t host_slot[MAX_COPY];
};

// resident waves of the partial-pass kernel per compute unit (occupancy query), per (head_dim, group)
int partial_waves_per_cu(int head_dim, int group);

// each returns 0 or a hipError_t value
int launch_table_patch(int32_t* table, const PatchArgs& a, hipStream_t stream);
int launch_kv_append(const PoolView& pv, const void* k_new, const void* v_new, const AppendArgs& a,
                     hipStream_t stream);
// Whole chunks between the pool (chunk c at pool + c * chunk_bytes) and the host buffer as the GPU
// sees it (slot s at host + s * chunk_bytes); to_host: offload, else fetch.
int launch_chunk_copy(char* pool, char* host, uint32_t chunk_bytes, const CopyArgs& a, bool to_host, hipStream_t stream);
// k_new / v_new non-NULL: fused append. a.len then counts one token per request whose K/V row
// ([request][kv head][dim], rows q_row0 .. of the caller's batch) is still in k_new / v_new; the
// kernel uses it from there and writes it into the chunk.
// out: the caller's output rows; requests with n_part == 1 are finished by the partial pass itself.
// ev_start / ev_stop (may be NULL): events that receive the start time of the call's first attention
// kernel and the end time of its last one, taken from the kernels' own dispatches.
int launch_decode_partial(const PoolView& pv, const void* q, const void* k_new, const void* v_new, float* ws,
                          void* out, float scale_log2, const BatchArgs& a, hipStream_t stream,
                          hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
int launch_decode_combine(const PoolView& pv, const float* ws, void* out, const BatchArgs& a, hipStream_t stream);

// Device address and size of the library's fixed workspace on the current device (resolved once per
// device, kept afterwards). Allocates nothing. Returns 0 or a hipError_t value.
int static_workspace(float** ptr, size_t* bytes);

// calibration (measurement only)
int launch_copy(void* dst, const void* src, int64_t bytes, hipStream_t stream);
int launch_read(const void* src, int64_t bytes, uint32_t* sink, hipStream_t stream);
int launch_kv_stream(const PoolView& pv, uint32_t* sink, const BatchArgs& a, hipStream_t stream);

}  // namespace ellm
