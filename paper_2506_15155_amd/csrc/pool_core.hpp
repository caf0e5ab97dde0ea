// Host-side state of the unified chunk pool and the per-tensor chunk tables.
//
// No HIP dependency: this is the part of the library that decides, on the host and before any
// launch, whether a call is legal, and that owns the virtual-to-physical map the kernels read.
// It follows the eLLM paper (arXiv 2506.15155): one physical pool shared by a KV side and an
// activation side (Sec. 2.1), per-request virtual tensors whose chunk-aligned slots are bound on
// demand (Sec. 2.1.1), ownership transfer of idle chunks between the two sides (Sec. 2.2.1), and
// host slots that hold offloaded chunks (Sec. 2.2.2).
//
// Every mutating operation is split into check (returns an error code, changes nothing) and
// commit (cannot fail), so callers can enqueue device work between the two.
#pragma once
#include <cstdint>
#include <set>
#include <string>
#include <utility>
#include <vector>

namespace ellm {

enum : int {
  OK = 0, ERR_INVALID = -1, ERR_OOM = -2, ERR_OWNED = -3, ERR_UNMAPPED = -4, ERR_NOT_RESIDENT = -5,
  ERR_RANGE = -6, ERR_EMPTY = -7, ERR_HOST_FULL = -8, ERR_HIP = -9, ERR_NO_DEVICE = -10
};
enum : uint8_t { OWNER_KV = 0, OWNER_ACT = 1 };
enum : uint8_t { CHUNK_FREE = 0, CHUNK_MAPPED = 1, CHUNK_BUSY = 2 };
constexpr int32_t ENTRY_UNMAPPED = -1;
inline int32_t entry_from_host_slot(int32_t s) { return -s - 2; }
inline int32_t host_slot_of_entry(int32_t e) { return -e - 2; }

struct Geometry {
  int32_t n_chunks = 0, n_host_slots = 0, tokens_per_chunk = 0;
  uint32_t chunk_bytes = 0;
  int32_t n_q_heads = 0, n_kv_heads = 0, head_dim = 0, group = 0;
  int32_t max_tensors = 0, max_slots = 0;
  uint64_t bytes_per_token = 0;
};

struct TensorRec {
  bool used = false;
  bool released = false;   // mapped and available: waits for a new request (Sec. 2.1.2)
  int32_t run = 0;         // while released: leading slots that still have a device chunk
  int64_t max_tokens = 0, len = 0;
  int32_t n_slots = 0;
};

// a planned chunk move between a device chunk and a host slot
struct Move { int32_t slot, chunk, host_slot; };

class PoolCore {
 public:
  PoolCore(const Geometry& g, const uint8_t* initial_owner);

  const Geometry& geom() const { return g_; }
  std::string& err() { return err_; }

  int tensor_create(int64_t max_tokens, int32_t* out);
  int tensor_destroy(int32_t id);
  // request turnover (Sec. 2.1.2): release keeps the leading mapped slots and makes the tensor
  // available; acquire picks the best-fitting available tensor or maps a fresh one on demand
  int tensor_release(int32_t id);
  int tensor_acquire(int64_t need_tokens, int64_t max_tokens, uint32_t flags, int32_t* out);
  // logical host buffer (Sec. 2.3.2): offloads may fill at most this many host slots; shrinking it
  // evicts nothing
  int set_logical_host_slots(int32_t n);
  int32_t logical_host_slots() const { return logical_host_; }
  // SLO-aware scaling of the logical buffer (Sec. 2.3.2)
  int slo_configure(double ttft_slo, double tpot_slo, double alpha, int32_t window, int32_t threshold);
  int slo_observe(double ttft, double tpot, int32_t* logical_out);
  // speculative pre-mapping (Sec. 3.1): one chunk for every request whose next token opens an empty slot
  int premap_next(const int32_t* ids, int32_t batch, uint32_t flags, int32_t* n_mapped);
  int premap_ahead(const int32_t* ids, int32_t batch, int64_t tokens_ahead, uint32_t flags, int32_t* n_mapped);
  int map_chunks(int32_t id, int32_t first, int32_t n, const int32_t* chunk_ids, uint32_t flags);
  int unmap_chunks(int32_t id, int32_t first, int32_t n);
  int transfer(const int32_t* chunk_ids, int32_t n, int new_owner);
  int set_act_busy(const int32_t* chunk_ids, int32_t n, int busy);

  // append: check the whole batch; on success `n_eff[b]` holds the token counts. commit bumps lens.
  int append_check(const int32_t* ids, int32_t batch, const int32_t* n_new, std::vector<int32_t>& n_eff,
                   int64_t* total);
  void append_commit(const int32_t* ids, int32_t batch, const int32_t* n_eff);
  // extra: tokens a not yet committed append adds to every request (0 or 1)
  int decode_check(const int32_t* ids, int32_t batch, int32_t extra = 0);

  // offload / fetch: plan lists the moves in slot order; commit applies them
  int offload_plan(int32_t id, int32_t first, int32_t n, std::vector<Move>& moves);
  void offload_commit(int32_t id, const std::vector<Move>& moves);
  int fetch_plan(int32_t id, int32_t first, int32_t n, const int32_t* chunk_ids, std::vector<Move>& moves);
  void fetch_commit(int32_t id, const std::vector<Move>& moves);

  // a tensor that belongs to a request; released ones take no call but acquire, destroy and read-out
  const TensorRec* tensor(int32_t id) const {
    return (id >= 0 && id < g_.max_tensors && t_[id].used && !t_[id].released) ? &t_[id] : nullptr;
  }
  const TensorRec* tensor_any(int32_t id) const {
    return (id >= 0 && id < g_.max_tensors && t_[id].used) ? &t_[id] : nullptr;
  }
  const int32_t* row(int32_t id) const { return &table_[(size_t)id * g_.max_slots]; }
  const std::vector<int32_t>& table() const { return table_; }
  // bumped by every change of an entry of the tensor's row
  uint32_t row_version(int32_t id) const { return row_version_[id]; }

  // table entries changed since the last take_dirty(): flat index into table()
  std::vector<int64_t> take_dirty();
  bool has_dirty() const { return !dirty_.empty(); }
  // a second, independent record of changed entries for a consumer that mirrors the table elsewhere
  // (driver mappings); off unless asked for
  void log_map_changes(bool on) { map_log_ = on; }
  std::vector<int64_t> take_map_changes();

  const std::vector<uint8_t>& owner() const { return owner_; }
  const std::vector<uint8_t>& state() const { return state_; }
  const std::vector<int32_t>& map_tensor() const { return map_tensor_; }
  const std::vector<int32_t>& map_slot() const { return map_slot_; }
  const std::vector<int32_t>& host_tensor() const { return host_tensor_; }
  const std::vector<int32_t>& host_slot() const { return host_slot_; }

  // O(n) consistency scan (tables vs chunk records vs free lists); 0 = consistent
  int self_check() const;

 private:
  int fail(int code, const char* what);
  int32_t* row_mut(int32_t id) { return &table_[(size_t)id * g_.max_slots]; }
  void set_entry(int32_t id, int32_t slot, int32_t value);
  void release_entry(int32_t e);
  int pick_chunks(int32_t n, const int32_t* explicit_ids, bool inflate, std::vector<int32_t>& out);
  void take_chunk(int32_t c, int32_t id, int32_t slot);

  Geometry g_;
  std::vector<uint8_t> owner_, state_;
  std::vector<int32_t> map_tensor_, map_slot_, host_tensor_, host_slot_;
  std::set<int32_t> free_kv_, free_act_, free_host_, free_ids_;
  std::set<std::pair<int32_t, int32_t>> released_;   // (leading mapped slots, handle) of every released tensor
  std::vector<TensorRec> t_;
  std::vector<int32_t> table_;     // max_tensors x max_slots, row-major, ENTRY_UNMAPPED where empty
  std::vector<int64_t> dirty_, map_dirty_;
  bool map_log_ = false;
  std::vector<uint32_t> row_version_;
  int32_t logical_host_ = 0;
  struct Slo {
    bool on = false;
    double ttft = 0, tpot = 0, alpha = 2;
    int32_t window = 5, threshold = 3;
    std::vector<uint8_t> ttft_hits, tpot_hits;   // violation flags of the iterations since the last change, newest last
  } slo_;
  std::vector<uint32_t> stamp_;    // per-chunk / per-tensor marks for duplicate detection
  uint32_t stamp_now_ = 0;
  std::string err_;
};

}  // namespace ellm
