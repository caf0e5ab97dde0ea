// C-ABI layer of libellm: argument checks, host state machine calls, stream ordering, launches.
// The contract of every entry point is stated in include/ellm.h.
#include "ellm.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <string>
#include <map>
#include <vector>

#include "kernels.hpp"
#include "map_queue.hpp"
#include "pool_core.hpp"

namespace {

thread_local std::string g_last_error = "";

int set_err(int code, const std::string& text) {
  g_last_error = text;
  return code;
}

int hip_err(hipError_t e, const char* where) {
  char buf[256];
  snprintf(buf, sizeof buf, "%s: %s", where, hipGetErrorString(e));
  return set_err(ELLM_ERR_HIP, buf);
}

#define HIP_TRY(call, where)                          \
  do {                                                \
    hipError_t e_ = (call);                           \
    if (e_ != hipSuccess) return hip_err(e_, where);  \
  } while (0)

}  // namespace

// the driver calls of a driver-mapped pool, as the pool's mapper thread makes them
struct HipMapDriver {
  int device = 0;
  size_t chunk_bytes = 0;
  const char* call = "";
  void thread_begin() { (void)hipSetDevice(device); }
  int wait_event(void* ev) {
    const hipError_t e = hipEventSynchronize((hipEvent_t)ev);
    (void)hipEventDestroy((hipEvent_t)ev);
    call = "hipEventSynchronize(before unmap)";
    return (int)e;
  }
  int map(char* at, void* handle) {
    call = "hipMemMap(tensor slot)";
    hipError_t e = hipMemMap(at, chunk_bytes, 0, (hipMemGenericAllocationHandle_t)handle, 0);
    if (e != hipSuccess) return (int)e;
    hipMemAccessDesc acc = {};
    acc.location.type = hipMemLocationTypeDevice;
    acc.location.id = device;
    acc.flags = hipMemAccessFlagsProtReadWrite;
    call = "hipMemSetAccess(tensor slot)";
    return (int)hipMemSetAccess(at, chunk_bytes, &acc, 1);
  }
  int unmap(char* at) {
    call = "hipMemUnmap(tensor slot)";
    return (int)hipMemUnmap(at, chunk_bytes);
  }
  const char* last_call() const { return call; }
};

struct ellm_pool {
  ellm::Geometry geom;
  std::unique_ptr<ellm::PoolCore> core;
  char* device_base = nullptr;
  char* host_base = nullptr;
  bool metadata_only = false;

  // device-side metadata, created by the first call that needs the device
  bool dev_ready = false;
  int32_t* d_table = nullptr;
  float* d_ws = nullptr;               // partial results of one decode launch (see BatchArgs)
  int64_t ws_cap_slots = 0;            // partial slots it holds
  float* static_ws = nullptr;          // this device's copy of the library's fixed workspace
  int64_t static_ws_slots = 0;
  hipStream_t side_in = nullptr;       // fetches (host -> device)
  hipStream_t side_out = nullptr;      // offloads (device -> host): a stream of its own, so that the two
                                       // directions use their own copy engines and run at the same time
  bool one_allocation = false;         // the pool buffer lies inside one device allocation (asked once)
  char* host_dev = nullptr;            // the host buffer as the GPU addresses it (NULL: it cannot)
  bool copy_kernels = false;           // offload / fetch by the library's copy kernel (where host_dev is known)
                                       // instead of the runtime's copy engines: faster alone, but it takes
                                       // compute units from the kernels it is meant to run beside
  ellm::CopyArgs copy_args;            // staging for one launch's list of chunks
  hipStream_t last_stream = nullptr;   // last stream given to append / decode
  bool have_last_stream = false;
  hipEvent_t ev_switch = nullptr;      // orders a new compute stream behind the one used before

  // Ordering between the compute stream and the two side streams is kept per chunk and per host
  // slot, so that a copy waits only for the kernels and copies that touched its chunks and a
  // kernel only for the copies of its chunks: a fetch for the next layer runs under this layer's
  // attention. Every compute call, fetch call and offload call gets a sequence number of its kind
  // and records an event from that kind's ring after its work; a chunk (host slot) remembers the
  // last call of each kind that touched it. Pools without host slots never migrate and skip it.
  static constexpr int EV_RING = 256;
  struct Ring {
    std::vector<hipEvent_t> ev;
    int64_t seq = 0;                   // calls of this kind so far = seq of the newest event
    int64_t done = 0;                  // highest seq the host has seen finished
  };
  Ring r_compute, r_in, r_out;
  // Compute calls are numbered but not marked one by one: an event behind every kernel would cost the
  // caller's stream a few microseconds each. A mark is recorded, on the stream of the latest compute
  // call, only when a copy (or an unmap) has to wait for a compute call no mark covers yet; mark i
  // (event r_compute.ev[i % EV_RING]) covers every compute call up to compute_covers[i % EV_RING].
  std::vector<int64_t> compute_covers;
  int64_t compute_marks = 0, compute_covered = 0;
  std::vector<int64_t> chunk_compute, chunk_in, chunk_out;   // per chunk: seq of the last call of a kind, 0 = none
  std::vector<int64_t> host_in, host_out;                    // per host slot: last fetch that read it, last offload that wrote it
  // what each waiting stream already waits for, per ring (a stream is in order, so waiting for seq n covers all before)
  int64_t compute_waits_in = 0, compute_waits_out = 0;
  int64_t in_waits_compute = 0, in_waits_out = 0;
  int64_t out_waits_compute = 0, out_waits_in = 0;
  // Per tensor: the newest fetch / offload that touched one of its chunks, valid while its table
  // row is unchanged (a copy that touches a chunk of a tensor always changes that tensor's row), so
  // that a compute call walks a tensor's slots once per change and not once per call.
  struct CopySeen { uint32_t row_version = 0; bool valid = false; int64_t in = 0, out = 0; };
  std::vector<CopySeen> copy_seen;
  int32_t fail_launch_in = 0;          // debug: the n-th launch from now fails without launching (0 = off)

  // Driver-mapped pools (ELLM_POOL_DRIVER_MAPPED): the chunks are physical allocations of the
  // library's own, all mapped once, in id order, into one range (`window`, which is device_base:
  // copies and table-reading kernels address chunks there), and additionally, while they back a
  // slot, into the virtual range of that slot's tensor, which is what the attention kernel reads.
  bool vmm = false;
  bool vmm_table_kernels = false;      // debug: run the table-reading kernels (on the window) instead
  int vmm_device = 0;
  std::vector<hipMemGenericAllocationHandle_t> vmm_handles;   // per chunk
  size_t vmm_window_mapped = 0;        // chunks mapped into the window so far
  std::vector<char*> vbase;            // per tensor handle: start of its reserved range, nullptr = none yet
  std::vector<int32_t> vmm_mapped;     // per (tensor, slot): chunk the driver has mapped there, -1 = none
  uint64_t* d_vbase = nullptr;         // device copy of vbase
  std::vector<int32_t> vbase_dirty;    // tensor handles whose base the device copy does not have yet
  // The driver calls run on a thread of the pool's own, in the order they were asked for (paper
  // Sec. 3.1: mappings made ahead of time and unmappings both happen beside the computation).
  std::unique_ptr<ellm::MapQueue<HipMapDriver>> mapq;
  uint64_t vmm_last_map = 0;                 // newest map job
  bool vmm_async = true;                     // false: every call waits for the jobs it asked for
  std::vector<uint64_t> vmm_slot_job;        // per (tensor, slot): the map job that makes it readable
  std::vector<uint64_t> vmm_tensor_job;      // per tensor: the newest of those
  int32_t split_override = 0;
  int32_t wave_slots = 0;              // waves of a decode launch: one per SIMD of the GPU (0 = not asked yet)
  int32_t waves_percent = 100;         // waves of a launch, as a share of what the GPU holds at once
  int64_t plan_total_tiles = 0;        // of the launch planned last: tiles per kv head,
  int64_t plan_waves = 0, plan_slots = 0;   // waves per kv head, partial slots

  // optional timing of the partial (dominant) kernel with events on the caller's stream
  std::vector<hipEvent_t> prof_ev;     // 2 per record
  int32_t prof_used = 0;
  int32_t prof_stride = 1, prof_phase = 0;   // every prof_stride-th launch is timed

  // scratch reused across calls
  std::vector<int32_t> n_eff;
  std::vector<ellm::Move> moves;
  std::vector<ellm::BatchArgs> launches;
  std::vector<int32_t> tiles_tmp;
};

namespace {

using ellm::PoolCore;

int core_err(ellm_pool* p, int rc) {
  if (rc) g_last_error = p->core->err();
  return rc;
}

int vmm_sync(ellm_pool* p);
int vmm_wait_slots(ellm_pool* p, const int32_t* ids, int32_t batch, int32_t extra);

// result of a call into the host state machine that may have changed table entries: a failed call
// changed nothing; after a successful one a driver-mapped pool brings its mappings in line
int core_changed(ellm_pool* p, int rc) {
  if (rc) return core_err(p, rc);
  return p->vmm ? vmm_sync(p) : ELLM_OK;
}

ellm::PoolView view_of(const ellm_pool* p) {
  ellm::PoolView v;
  v.base = p->device_base;
  v.table = p->d_table;
  v.vbase = (p->vmm && !p->vmm_table_kernels) ? p->d_vbase : nullptr;
  v.chunk_bytes = p->geom.chunk_bytes;
  v.tokens_per_chunk = p->geom.tokens_per_chunk;
  v.tiles_per_chunk = (p->geom.tokens_per_chunk + ellm::TILE_TOKENS - 1) / ellm::TILE_TOKENS;
  v.max_slots = p->geom.max_slots;
  v.n_q_heads = p->geom.n_q_heads;
  v.n_kv_heads = p->geom.n_kv_heads;
  v.head_dim = p->geom.head_dim;
  v.group = p->geom.group;
  return v;
}

int32_t wave_slots(ellm_pool* p);

// SIMDs of the current device (4 per compute unit); without a device, those of a nominal MI355X
int32_t device_simds() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
    return cus * ellm::SIMDS_PER_CU;
  (void)hipGetLastError();
  return 256 * ellm::SIMDS_PER_CU;
}

// Partial slots one decode launch can need under the automatic partition: every wave writes one
// partial, and one more for every request boundary inside its share; the waves of all kv heads
// together are at most one per SIMD, and each kv head's sequence has n_req - 1 inner boundaries.
int64_t launch_slot_bound(int32_t simds, int32_t n_kv_heads, int32_t n_req) {
  return (int64_t)simds + (int64_t)n_kv_heads * (std::max(n_req, 1) - 1);
}

size_t slot_bytes(int32_t group, int32_t head_dim) { return (size_t)group * (head_dim + ellm::WS_ML) * sizeof(float); }

int ensure_device(ellm_pool* p) {
  if (p->dev_ready) return ELLM_OK;
  const size_t bytes = p->core->table().size() * sizeof(int32_t);
  HIP_TRY(hipMalloc((void**)&p->d_table, bytes), "hipMalloc(table mirror)");
  HIP_TRY(hipMemcpy(p->d_table, p->core->table().data(), bytes, hipMemcpyHostToDevice), "hipMemcpy(table mirror)");
  (void)p->core->take_dirty();   // the full upload covers everything so far
  // the workspace is sized once, for the largest launch the automatic partition can produce
  p->ws_cap_slots = launch_slot_bound(device_simds(), p->geom.n_kv_heads, std::min<int32_t>(p->geom.max_tensors, ellm::MAX_LAUNCH_REQ));
  HIP_TRY(hipMalloc((void**)&p->d_ws, (size_t)p->ws_cap_slots * slot_bytes(p->geom.group, p->geom.head_dim)), "hipMalloc(workspace)");
  if (p->vmm) {
    const size_t vb = (size_t)p->geom.max_tensors * sizeof(uint64_t);
    HIP_TRY(hipMalloc((void**)&p->d_vbase, vb), "hipMalloc(tensor bases)");
    HIP_TRY(hipMemset(p->d_vbase, 0, vb), "hipMemset(tensor bases)");
  }
  if (!p->vmm && p->device_base) {
    void* base = nullptr;
    size_t size = 0;
    const size_t pool_bytes = (size_t)p->geom.n_chunks * p->geom.chunk_bytes;
    if (hipMemGetAddressRange((hipDeviceptr_t*)&base, &size, (hipDeviceptr_t)p->device_base) == hipSuccess)
      p->one_allocation = (char*)base <= p->device_base && p->device_base + pool_bytes <= (char*)base + size;
    else
      (void)hipGetLastError();
  }
  if (p->host_base && p->geom.n_host_slots > 0) {
    void* seen = nullptr;
    if (hipHostGetDevicePointer(&seen, p->host_base, 0) == hipSuccess) p->host_dev = (char*)seen;
    else (void)hipGetLastError();
  }
  HIP_TRY(hipStreamCreateWithFlags(&p->side_in, hipStreamNonBlocking), "hipStreamCreate(side)");
  HIP_TRY(hipStreamCreateWithFlags(&p->side_out, hipStreamNonBlocking), "hipStreamCreate(side)");
  HIP_TRY(hipEventCreateWithFlags(&p->ev_switch, hipEventDisableTiming), "hipEventCreate");
  {
    // everything a later call that may not allocate will need is looked up now: the wave capacity
    // (an occupancy query) and this device's address of the library's fixed workspace
    (void)wave_slots(p);
    size_t bytes = 0;
    const int e = ellm::static_workspace(&p->static_ws, &bytes);
    if (e) return hip_err((hipError_t)e, "hipGetSymbolAddress(fixed workspace)");
    p->static_ws_slots = (int64_t)(bytes / slot_bytes(p->geom.group, p->geom.head_dim));
    p->launches.reserve(((size_t)p->geom.max_tensors + ellm::MAX_LAUNCH_REQ - 1) / ellm::MAX_LAUNCH_REQ);
    p->tiles_tmp.reserve(ellm::MAX_LAUNCH_REQ);
  }
  if (p->geom.n_host_slots > 0 || p->vmm) {
    p->chunk_compute.assign(p->geom.n_chunks, 0);
    p->chunk_in.assign(p->geom.n_chunks, 0);
    p->chunk_out.assign(p->geom.n_chunks, 0);
    p->host_in.assign(p->geom.n_host_slots, 0);
    p->host_out.assign(p->geom.n_host_slots, 0);
    p->copy_seen.assign(p->geom.max_tensors, ellm_pool::CopySeen());
    p->compute_covers.assign(ellm_pool::EV_RING, 0);
    for (ellm_pool::Ring* r : {&p->r_compute, &p->r_in, &p->r_out})
      for (int i = 0; i < ellm_pool::EV_RING; i++) {
        hipEvent_t e;
        HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming), "hipEventCreate");
        r->ev.push_back(e);
      }
  }
  p->dev_ready = true;
  return ELLM_OK;
}

// push host-side table changes to the device mirror, ordered on `stream`: the changed entries
// travel in the arguments of small patch kernels, MAX_PATCH per launch, so nothing here waits for
// the device and no staging buffer has to outlive the call
int flush_table(ellm_pool* p, hipStream_t stream) {
  if (!p->vbase_dirty.empty()) {
    // new tensor ranges: their 64-bit bases go to the device as pairs of 32-bit words
    ellm::PatchArgs a;
    a.n = 0;
    for (size_t i = 0; i < p->vbase_dirty.size(); i++) {
      const int32_t id = p->vbase_dirty[i];
      const uint64_t v = (uint64_t)(uintptr_t)p->vbase[id];
      a.idx[a.n] = 2 * id;     a.val[a.n++] = (int32_t)(uint32_t)v;
      a.idx[a.n] = 2 * id + 1; a.val[a.n++] = (int32_t)(uint32_t)(v >> 32);
      if (a.n + 2 > ellm::MAX_PATCH || i + 1 == p->vbase_dirty.size()) {
        int e = ellm::launch_table_patch((int32_t*)p->d_vbase, a, stream);
        if (e) return hip_err((hipError_t)e, "tensor base patch launch");
        a.n = 0;
      }
    }
    p->vbase_dirty.clear();
  }
  if (!p->core->has_dirty()) return ELLM_OK;
  std::vector<int64_t> dirty = p->core->take_dirty();
  const std::vector<int32_t>& tab = p->core->table();
  ellm::PatchArgs a;
  size_t i = 0;
  while (i < dirty.size()) {
    a.n = 0;
    for (; i < dirty.size() && a.n < ellm::MAX_PATCH; i++, a.n++) {
      a.idx[a.n] = (int32_t)dirty[i];
      a.val[a.n] = tab[dirty[i]];
    }
    int e = ellm::launch_table_patch(p->d_table, a, stream);
    if (e) return hip_err((hipError_t)e, "table patch launch");
  }
  return ELLM_OK;
}

// chunks are tracked where something besides the kernels touches them: copies to and from host
// slots, or the driver unmapping them from a tensor's range
bool tracks_chunks(const ellm_pool* p) { return p->geom.n_host_slots > 0 || p->vmm; }

// the event that covers call `need` of ring r: its own, or, once the ring has gone round, the
// newest one of the same (in-order) stream
hipEvent_t event_of(const ellm_pool::Ring& r, int64_t& need) {
  if (need <= r.seq - ellm_pool::EV_RING) need = r.seq;
  return r.ev[need % ellm_pool::EV_RING];
}

// `waiter` waits for call `need` of ring r unless it already waits for that much
int wait_for(hipStream_t waiter, const ellm_pool::Ring& r, int64_t need, int64_t& waited) {
  if (need <= waited || need <= r.done) return ELLM_OK;
  HIP_TRY(hipStreamWaitEvent(waiter, event_of(r, need), 0), "hipStreamWaitEvent");
  waited = need;
  return ELLM_OK;
}

// the host waits until call `need` of ring r has finished
int host_wait(ellm_pool::Ring& r, int64_t need) {
  if (need <= r.done) return ELLM_OK;
  HIP_TRY(hipEventSynchronize(event_of(r, need)), "hipEventSynchronize");
  r.done = need;
  return ELLM_OK;
}

// The event behind compute call `need` of this pool, recorded now if no mark covers that call yet
// (then it covers everything enqueued so far on the compute stream, which is in order). *covers
// receives the newest call the event stands behind.
int compute_mark(ellm_pool* p, int64_t need, hipEvent_t* ev, int64_t* covers) {
  ellm_pool::Ring& r = p->r_compute;
  if (need > p->compute_covered) {
    const int64_t i = p->compute_marks % ellm_pool::EV_RING;
    HIP_TRY(hipEventRecord(r.ev[i], p->last_stream), "hipEventRecord(compute mark)");
    p->compute_covers[i] = p->compute_covered = r.seq;
    p->compute_marks++;
    *ev = r.ev[i];
    *covers = r.seq;
    return ELLM_OK;
  }
  // the oldest mark still in the ring that covers the call (marks are in ascending order of cover)
  int64_t pick = p->compute_marks - 1;
  for (int64_t i = p->compute_marks - 2; i >= 0 && i > p->compute_marks - 1 - ellm_pool::EV_RING; i--) {
    if (p->compute_covers[i % ellm_pool::EV_RING] < need) break;
    pick = i;
  }
  *ev = r.ev[pick % ellm_pool::EV_RING];
  *covers = p->compute_covers[pick % ellm_pool::EV_RING];
  return ELLM_OK;
}

// `waiter` (a side stream) waits for compute call `need`
int wait_for_compute(ellm_pool* p, hipStream_t waiter, int64_t need, int64_t& waited) {
  if (need <= waited || need <= p->r_compute.done) return ELLM_OK;
  hipEvent_t ev;
  int64_t covers;
  int rc = compute_mark(p, need, &ev, &covers);
  if (rc) return rc;
  HIP_TRY(hipStreamWaitEvent(waiter, ev, 0), "hipStreamWaitEvent(compute mark)");
  waited = covers;
  return ELLM_OK;
}

// a call of ring r's kind has enqueued its work on `stream`: number it and mark its end
int record_on(ellm_pool::Ring& r, hipStream_t stream, int64_t* seq) {
  *seq = ++r.seq;
  HIP_TRY(hipEventRecord(r.ev[*seq % ellm_pool::EV_RING], stream), "hipEventRecord");
  return ELLM_OK;
}

// Things every compute call does before launching on `stream`: wait for the copies that touched
// the chunks of the tensors it works on (and, in a driver-mapped pool, for the mapper thread to have
// mapped the slots the call reaches with `extra` more tokens per tensor), bring the device table up to date. The ordering state
// treats the compute calls as one in-order sequence; a call on another stream than the one before
// is therefore first put behind that one.
int enter_compute(ellm_pool* p, hipStream_t stream, const int32_t* ids, int32_t batch, int32_t extra) {
  int rc = ensure_device(p);
  if (rc) return rc;
  if (p->vmm && (rc = vmm_wait_slots(p, ids, batch, extra))) return rc;
  if (p->have_last_stream && stream != p->last_stream) {
    HIP_TRY(hipEventRecord(p->ev_switch, p->last_stream), "hipEventRecord(stream change)");
    HIP_TRY(hipStreamWaitEvent(stream, p->ev_switch, 0), "hipStreamWaitEvent(stream change)");
    p->compute_waits_in = p->compute_waits_out = 0;   // what the old stream waited for, the new one has yet to
  }
  if (tracks_chunks(p) && (p->r_in.seq > p->compute_waits_in || p->r_out.seq > p->compute_waits_out)) {
    int64_t need_in = 0, need_out = 0;
    for (int32_t b = 0; b < batch; b++) {
      ellm_pool::CopySeen& cs = p->copy_seen[ids[b]];
      const uint32_t ver = p->core->row_version(ids[b]);
      if (!cs.valid || cs.row_version != ver) {
        const ellm::TensorRec* t = p->core->tensor(ids[b]);
        const int32_t* r = p->core->row(ids[b]);
        cs.in = cs.out = 0;
        for (int32_t s = 0; s < t->n_slots; s++)
          if (r[s] >= 0) {
            cs.in = std::max(cs.in, p->chunk_in[r[s]]);
            cs.out = std::max(cs.out, p->chunk_out[r[s]]);
          }
        cs.row_version = ver;
        cs.valid = true;
      }
      need_in = std::max(need_in, cs.in);
      need_out = std::max(need_out, cs.out);
    }
    if ((rc = wait_for(stream, p->r_in, need_in, p->compute_waits_in))) return rc;
    if ((rc = wait_for(stream, p->r_out, need_out, p->compute_waits_out))) return rc;
  }
  rc = flush_table(p, stream);
  if (rc) return rc;
  p->last_stream = stream;
  p->have_last_stream = true;
  return ELLM_OK;
}

// after a compute call's launches: remember which chunks it touches and mark its end on the stream
int leave_compute(ellm_pool* p, hipStream_t stream, const int32_t* ids, int32_t batch) {
  if (!tracks_chunks(p)) return ELLM_OK;
  (void)stream;                        // == p->last_stream: where a mark for this call would be recorded
  const int64_t seq = ++p->r_compute.seq;
  for (int32_t b = 0; b < batch; b++) {
    const ellm::TensorRec* t = p->core->tensor(ids[b]);
    const int32_t* r = p->core->row(ids[b]);
    for (int32_t s = 0; s < t->n_slots; s++)
      if (r[s] >= 0) p->chunk_compute[r[s]] = seq;
  }
  return ELLM_OK;
}

// An offload reads device chunks and writes host slots; a fetch reads host slots and overwrites
// device chunks. Its stream waits for the kernels that touched those chunks (the last reader of
// a chunk about to be overwritten may still run) and for the copies of the other direction that
// touched the same chunks or host slots.
int enter_migration(ellm_pool* p, const std::vector<ellm::Move>& moves, bool fetch) {
  int rc = ensure_device(p);
  if (rc) return rc;
  int64_t need_compute = 0, need_other = 0;
  for (const ellm::Move& m : moves) {
    need_compute = std::max(need_compute, p->chunk_compute[m.chunk]);
    if (fetch) need_other = std::max({need_other, p->chunk_out[m.chunk], p->host_out[m.host_slot]});
    else need_other = std::max({need_other, p->chunk_in[m.chunk], p->host_in[m.host_slot]});
  }
  if (fetch) {
    if ((rc = wait_for_compute(p, p->side_in, need_compute, p->in_waits_compute))) return rc;
    return wait_for(p->side_in, p->r_out, need_other, p->in_waits_out);
  }
  if ((rc = wait_for_compute(p, p->side_out, need_compute, p->out_waits_compute))) return rc;
  return wait_for(p->side_out, p->r_in, need_other, p->out_waits_in);
}

// Moves i, i + 1, ... whose chunks and whose host slots are both consecutive are one contiguous piece
// of the pool and one of the host buffer: they travel as one copy (a 2 MiB copy reaches 44 GB/s on
// this machine, a large one 57). Returns how many moves from i on form such a run. Only where the
// pool is known to lie inside one device allocation: a pool whose chunks are mappings of their own
// (a driver-mapped pool's window, a caller's buffer built the same way) is copied chunk by chunk.
size_t move_run(const ellm_pool* p, const std::vector<ellm::Move>& moves, size_t i) {
  size_t n = 1;
  if (!p->one_allocation) return n;
  while (i + n < moves.size() && moves[i + n].chunk == moves[i].chunk + (int32_t)n &&
         moves[i + n].host_slot == moves[i].host_slot + (int32_t)n)
    n++;
  return n;
}

// Enqueues the copies of an offload (device chunk -> host slot) or a fetch on that direction's side
// stream: copy calls of the runtime, one per run of neighbouring chunks, which the copy engines carry
// out beside the kernels; or, if asked for and the GPU can address the host buffer, one launch of the
// library's copy kernel for all of them. Measured on the 8B-shaped elastic step (3.56 GB each way):
// the kernel moves 49 / 54 GB/s out / in against 46 / 46, but an attention kernel that runs beside it
// takes 205-224 us instead of 69-83 (62 alone), and the layer-wise overlapped step is no shorter
// (114-117 against 109-123 ms); so the copy engines are the default.
int copy_chunks(ellm_pool* p, const std::vector<ellm::Move>& moves, bool fetch) {
  const size_t cb = p->geom.chunk_bytes;
  hipStream_t side = fetch ? p->side_in : p->side_out;
  if (p->host_dev && p->copy_kernels) {
    for (size_t i = 0; i < moves.size(); i += ellm::MAX_COPY) {
      ellm::CopyArgs& a = p->copy_args;
      a.n = (int32_t)std::min<size_t>(ellm::MAX_COPY, moves.size() - i);
      for (int32_t k = 0; k < a.n; k++) {
        a.chunk[k] = moves[i + k].chunk;
        a.host_slot[k] = moves[i + k].host_slot;
      }
      const int e = ellm::launch_chunk_copy(p->device_base, p->host_dev, (uint32_t)cb, a, !fetch, side);
      if (e) return hip_err((hipError_t)e, fetch ? "copy kernel launch (fetch)" : "copy kernel launch (offload)");
    }
    return ELLM_OK;
  }
  for (size_t i = 0; i < moves.size();) {
    const size_t n = move_run(p, moves, i);
    const ellm::Move& m = moves[i];
    char* dev = p->device_base + (size_t)m.chunk * cb;
    char* host = p->host_base + (size_t)m.host_slot * cb;
    if (fetch) HIP_TRY(hipMemcpyAsync(dev, host, n * cb, hipMemcpyHostToDevice, side), "hipMemcpyAsync(fetch)");
    else HIP_TRY(hipMemcpyAsync(host, dev, n * cb, hipMemcpyDeviceToHost, side), "hipMemcpyAsync(offload)");
    i += n;
  }
  return ELLM_OK;
}

int leave_migration(ellm_pool* p, const std::vector<ellm::Move>& moves, bool fetch) {
  int64_t seq;
  int rc = fetch ? record_on(p->r_in, p->side_in, &seq) : record_on(p->r_out, p->side_out, &seq);
  if (rc) return rc;
  for (const ellm::Move& m : moves) {
    (fetch ? p->chunk_in : p->chunk_out)[m.chunk] = seq;
    (fetch ? p->host_in : p->host_out)[m.host_slot] = seq;
  }
  return ELLM_OK;
}

// Chunks are about to leave the KV side's care (handed to the activation side, or marked busy
// there): copies of this library that still read or write them must have finished first, because
// whoever uses the chunks next runs on streams the library does not see. The host waits.
int settle_copies(ellm_pool* p, const int32_t* chunk_ids, int32_t n) {
  if (!p->dev_ready || !tracks_chunks(p)) return ELLM_OK;
  int64_t need_in = 0, need_out = 0;
  for (int32_t i = 0; i < n; i++) {
    need_in = std::max(need_in, p->chunk_in[chunk_ids[i]]);
    need_out = std::max(need_out, p->chunk_out[chunk_ids[i]]);
  }
  int rc = host_wait(p->r_out, need_out);
  if (rc) return rc;
  return host_wait(p->r_in, need_in);
}

// ---- driver-mapped pools --------------------------------------------------------------------
// The paper's mechanism (Sec. 2.1.1, Sec. 3.2): a tensor is a reserved virtual address range and a
// chunk that backs one of its slots is mapped there by the driver. The host table stays the
// source of truth; after every call that changed table entries the driver mappings are brought in
// line with it, entry by entry: what left a slot is unmapped (once the kernels that may still
// read it there have finished), what came is mapped and made accessible.
//   A driver call takes tens of microseconds on an idle GPU and a few hundred while kernels run, so
// the calls are not made by the thread that changed the table: they are queued, in order, for a
// thread of the pool's own (paper Sec. 3.1: chunks are mapped ahead of their first use, and
// unmapping is taken off the critical path). A compute call waits only for the map jobs of the
// slots it is about to touch; a slot mapped one step ahead is ready by then. An unmap job first
// waits, on its own thread, for an event recorded behind the kernels launched so far.
hipMemAllocationProp vmm_prop(int dev) {
  hipMemAllocationProp prop = {};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = dev;
  return prop;
}

// the caller waits until the mapper thread has finished job `seq`; reports what went wrong there
int vmm_wait(ellm_pool* p, uint64_t seq) {
  std::string where;
  const int e = p->mapq->wait(seq, &where);
  if (!e) return ELLM_OK;
  if (e < 0) return set_err(ELLM_ERR_HIP, where);       // the test hook's refusal
  return hip_err((hipError_t)e, where.c_str());
}

int vmm_drain(ellm_pool* p) { return p->vmm && p->mapq && p->mapq->running() ? vmm_wait(p, p->mapq->last()) : ELLM_OK; }

// A compute call is about to touch the first ceil((len + extra) / tokens per chunk) slots of these
// tensors: the map jobs of those slots must have finished. Slots mapped further ahead are not
// waited for.
int vmm_wait_slots(ellm_pool* p, const int32_t* ids, int32_t batch, int32_t extra) {
  const uint64_t done = p->mapq->done();
  // after a driver error some slot may be without its chunk: nothing is launched on this pool again
  // (the thread sets the flag before it counts the job as done, so it is read after the count)
  if (p->mapq->failed()) return vmm_wait(p, 0);
  if (done >= p->vmm_last_map) return ELLM_OK;
  uint64_t need = 0;
  for (int32_t b = 0; b < batch; b++) {
    if (p->vmm_tensor_job[ids[b]] <= done) continue;
    const ellm::TensorRec* t = p->core->tensor(ids[b]);
    const int64_t slots = std::min<int64_t>(t->n_slots, (t->len + extra + p->geom.tokens_per_chunk - 1) / p->geom.tokens_per_chunk);
    const uint64_t* j = &p->vmm_slot_job[(size_t)ids[b] * p->geom.max_slots];
    for (int64_t s_ = 0; s_ < slots; s_++) need = std::max(need, j[s_]);
  }
  return need > done ? vmm_wait(p, need) : ELLM_OK;
}

int vmm_sync(ellm_pool* p) {
  if (!p->vmm) return ELLM_OK;
  const std::vector<int64_t> changed = p->core->take_map_changes();
  if (changed.empty()) return ELLM_OK;
  const size_t cb = p->geom.chunk_bytes;
  const std::vector<int32_t>& tab = p->core->table();
  std::vector<ellm::MapJob> jobs;
  bool kernels_may_read = false;             // an unmapped chunk may still be read by a kernel in flight
  for (int64_t flat : changed) {
    const int32_t id = (int32_t)(flat / p->geom.max_slots), slot = (int32_t)(flat % p->geom.max_slots);
    const int32_t want = tab[flat] >= 0 ? tab[flat] : -1, have = p->vmm_mapped[flat];
    if (want == have) continue;
    if (!p->vbase[id]) {
      // a tensor handle's range is reserved once, for the largest tensor the pool allows, and kept
      // for the handle's later lives
      void* va = nullptr;
      const hipError_t e = hipMemAddressReserve(&va, (size_t)p->geom.max_slots * cb, 0, nullptr, 0);
      if (e != hipSuccess) {
        // the table already names chunks that will never be mapped: no kernel may run on this pool again
        p->mapq->fail_now((int)e, "hipMemAddressReserve(tensor)");
        if (!jobs.empty()) p->mapq->push(jobs);
        return hip_err(e, "hipMemAddressReserve(tensor)");
      }
      p->vbase[id] = (char*)va;
      p->vbase_dirty.push_back(id);
    }
    char* at = p->vbase[id] + (size_t)slot * cb;
    if (have >= 0) {
      if (p->dev_ready && p->chunk_compute[have] > p->r_compute.done) kernels_may_read = true;
      jobs.push_back({at, nullptr, true, nullptr});
      p->vmm_mapped[flat] = -1;
    }
    if (want >= 0) {
      jobs.push_back({at, (void*)p->vmm_handles[want], false, nullptr});
      p->vmm_mapped[flat] = want;
      p->vmm_slot_job[flat] = p->vmm_tensor_job[id] = p->vmm_last_map = p->mapq->last() + jobs.size();
    }
  }
  if (jobs.empty()) return ELLM_OK;
  if (kernels_may_read && p->have_last_stream) {
    // one event behind everything launched so far covers every unmap of this call: the first of
    // them waits for it, the others run after that one
    hipEvent_t ev = nullptr;
    hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e == hipSuccess && (e = hipEventRecord(ev, p->last_stream)) != hipSuccess) {
      (void)hipEventDestroy(ev);
      ev = nullptr;
    }
    if (ev) {
      for (ellm::MapJob& j : jobs)
        if (j.unmap) { j.after = (void*)ev; break; }
    } else {
      // no event to be had: the jobs are already decided, so this thread waits for the kernels itself
      (void)hipGetLastError();
      if (hipStreamSynchronize(p->last_stream) != hipSuccess) {
        p->mapq->fail_now((int)e, "hipEventRecord(before unmap)");
        return hip_err(e, "hipEventRecord(before unmap)");
      }
    }
  }
  p->mapq->push(jobs);
  return p->vmm_async ? ELLM_OK : vmm_drain(p);
}

// creates the chunks and the window; on failure everything created so far is released by vmm_teardown
int vmm_setup(ellm_pool* p) {
  HIP_TRY(hipGetDevice(&p->vmm_device), "hipGetDevice");
  hipMemAllocationProp prop = vmm_prop(p->vmm_device);
  size_t gran = 0;
  HIP_TRY(hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityMinimum), "hipMemGetAllocationGranularity");
  if (gran == 0 || p->geom.chunk_bytes % gran)
    return set_err(ELLM_ERR_INVALID, "pool_create: chunk_bytes must be a multiple of the driver's allocation granularity");
  const size_t cb = p->geom.chunk_bytes, n = (size_t)p->geom.n_chunks;
  void* va = nullptr;
  HIP_TRY(hipMemAddressReserve(&va, cb * n, 0, nullptr, 0), "hipMemAddressReserve(window)");
  p->device_base = (char*)va;
  p->vmm_handles.reserve(n);
  for (size_t c = 0; c < n; c++) {
    hipMemGenericAllocationHandle_t h;
    HIP_TRY(hipMemCreate(&h, cb, &prop, 0), "hipMemCreate(chunk)");
    p->vmm_handles.push_back(h);
  }
  for (; p->vmm_window_mapped < n; p->vmm_window_mapped++)
    HIP_TRY(hipMemMap(p->device_base + p->vmm_window_mapped * cb, cb, 0, p->vmm_handles[p->vmm_window_mapped], 0), "hipMemMap(window)");
  hipMemAccessDesc acc = {};
  acc.location = prop.location;
  acc.flags = hipMemAccessFlagsProtReadWrite;
  HIP_TRY(hipMemSetAccess(p->device_base, cb * n, &acc, 1), "hipMemSetAccess(window)");
  p->vbase.assign(p->geom.max_tensors, nullptr);
  p->vmm_mapped.assign((size_t)p->geom.max_tensors * p->geom.max_slots, -1);
  p->vmm_slot_job.assign((size_t)p->geom.max_tensors * p->geom.max_slots, 0);
  p->vmm_tensor_job.assign(p->geom.max_tensors, 0);
  p->core->log_map_changes(true);
  HipMapDriver drv;
  drv.device = p->vmm_device;
  drv.chunk_bytes = cb;
  p->mapq.reset(new ellm::MapQueue<HipMapDriver>(drv));
  p->mapq->start();
  return ELLM_OK;
}

void vmm_teardown(ellm_pool* p) {
  if (p->mapq) p->mapq->stop();        // the thread works off what is queued, then ends
  const size_t cb = p->geom.chunk_bytes;
  for (size_t flat = 0; flat < p->vmm_mapped.size(); flat++)
    if (p->vmm_mapped[flat] >= 0) {
      const size_t id = flat / p->geom.max_slots, slot = flat % p->geom.max_slots;
      (void)hipMemUnmap(p->vbase[id] + slot * cb, cb);
    }
  for (char* va : p->vbase)
    if (va) (void)hipMemAddressFree(va, (size_t)p->geom.max_slots * cb);
  for (size_t c = 0; c < p->vmm_window_mapped; c++) (void)hipMemUnmap(p->device_base + c * cb, cb);
  for (hipMemGenericAllocationHandle_t h : p->vmm_handles) (void)hipMemRelease(h);
  if (p->device_base) (void)hipMemAddressFree(p->device_base, cb * (size_t)p->geom.n_chunks);
  p->device_base = nullptr;
  // after a driver error some slots recorded as mapped never were, and unmapping those fails: that is
  // expected here and must not be left behind as the calling thread's last error
  (void)hipGetLastError();
}

// Under the automatic partition a launch never needs more partial slots than the workspace was
// sized for. With a partition override in force (tests and measurements) it may: then, and only
// then, the workspace is replaced by a larger one, which waits for the device.
int ensure_workspace(ellm_pool* p, int64_t n_slots) {
  if (n_slots <= p->ws_cap_slots) return ELLM_OK;
  if (p->split_override <= 0 && p->waves_percent == 100)
    return set_err(ELLM_ERR_RANGE, "decode_attention: launch needs more partial slots than ellm_workspace_bytes allows for");
  HIP_TRY(hipDeviceSynchronize(), "hipDeviceSynchronize(workspace growth)");
  HIP_TRY(hipFree(p->d_ws), "hipFree(workspace)");
  p->d_ws = nullptr;
  p->ws_cap_slots = 0;
  const int64_t grow = n_slots + n_slots / 4;
  HIP_TRY(hipMalloc((void**)&p->d_ws, (size_t)grow * slot_bytes(p->geom.group, p->geom.head_dim)), "hipMalloc(workspace)");
  p->ws_cap_slots = grow;
  return ELLM_OK;
}

// Waves of a decode launch: one for every SIMD of the GPU (fewer if the kernel's resources allow
// fewer). Two waves per SIMD, which the kernel's registers and LDS would allow, measured slower on
// every workload: the second wave of a SIMD gets its loads served 15 to 50 % more slowly than the
// first, and it takes bandwidth from it. Without a device (metadata-only pools, planning calls on
// a host without GPU) a nominal MI355X figure is used: 256 compute units x 4 SIMDs.
int32_t wave_slots(ellm_pool* p) {
  if (p->wave_slots > 0) return p->wave_slots;
  int32_t slots = 256 * ellm::SIMDS_PER_CU;
  if (!p->metadata_only) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      slots = cus * std::min(ellm::SIMDS_PER_CU, ellm::partial_waves_per_cu(p->geom.head_dim, p->geom.group));
    else
      (void)hipGetLastError();
  }
  p->wave_slots = slots;
  return slots;
}

// The partition of one launch (at most MAX_LAUNCH_REQ requests). For each kv head the tiles of all
// requests form one sequence, dealt out evenly to as many waves as the GPU has SIMDs (all kv
// heads together): every wave reads the same amount, all are resident from the start, and a wave
// whose share crosses from one request into the next finishes a result for each. The cut
// depends only on the batch's lengths, the pool geometry and the device's wave capacity, never on
// physical chunk ids or on which wave runs when: every rounding is reproducible and invariant
// under remapping.
// With an override (tests) every wave gets the given number of tokens' worth of tiles.
void plan_launch(ellm_pool* p, const int32_t* ids, int32_t n_req, int32_t q_row0, ellm::BatchArgs& a, int32_t extra = 0) {
  const int32_t Tc = p->geom.tokens_per_chunk;
  const int32_t tpc = (Tc + ellm::TILE_TOKENS - 1) / ellm::TILE_TOKENS;
  int64_t total = 0;
  std::vector<int32_t>& tiles = p->tiles_tmp;
  tiles.resize(n_req);
  for (int32_t i = 0; i < n_req; i++) {
    const int64_t len = p->core->tensor(ids[i])->len + extra;   // extra: tokens of a fused append
    const int64_t full = len / Tc, rem = len - full * Tc;
    tiles[i] = (int32_t)(full * tpc + (rem + ellm::TILE_TOKENS - 1) / ellm::TILE_TOKENS);
    a.req[i].tensor = ids[i];
    a.req[i].len = (int32_t)len;
    a.req[i].tile_prefix = (int32_t)std::min<int64_t>(total, 0x7fffffff);
    total += tiles[i];
  }
  int64_t waves;
  if (p->split_override > 0) {
    const int64_t per = std::max<int64_t>(1, p->split_override / ellm::TILE_TOKENS);
    waves = (total + per - 1) / per;
  } else {
    waves = (int64_t)wave_slots(p) * p->waves_percent / 100 / p->geom.n_kv_heads;
  }
  waves = std::max<int64_t>(1, std::min<int64_t>(waves, total));
  const int64_t each = total / waves, more = total - each * waves;
  // wave that holds tile x: the first `more` waves hold each + 1 tiles, the others each
  auto wave_of = [&](int64_t x) { return x < more * (each + 1) ? x / (each + 1) : more + (x - more * (each + 1)) / each; };
  std::memset(a.split_req, 0, sizeof(a.split_req));
  int64_t at = 0, parts = 0;
  int32_t n_split = 0;
  for (int32_t i = 0; i < n_req; i++) {
    const int64_t w0 = wave_of(at), w1 = wave_of(at + tiles[i] - 1);
    a.req[i].wave_first = (int32_t)w0;
    a.req[i].n_part = (int32_t)(w1 - w0 + 1);
    a.req[i].part0 = 0;
    if (w1 > w0) {               // a request shared by several waves: partial results and a combine pass
      a.req[i].part0 = (int32_t)std::min<int64_t>(parts, 0x7fffffff);
      parts += w1 - w0 + 1;
      a.split_req[n_split >> 2] |= (uint32_t)i << ((n_split & 3) * 8);
      n_split++;
    }
    at += tiles[i];
  }
  a.n_req = n_req;
  a.q_row0 = q_row0;
  a.tiles_per_head = (int32_t)std::min<int64_t>(total, 0x7fffffff);
  a.waves_per_head = (int32_t)std::min<int64_t>(waves, 0x7fffffff);
  a.tiles_each = (int32_t)each;
  a.tiles_extra = (int32_t)more;
  a.parts_per_head = (int32_t)std::min<int64_t>(parts, 0x7fffffff);
  a.ws_slots = (int32_t)std::min<int64_t>(parts * p->geom.n_kv_heads, 0x7fffffff);
  a.n_split_req = n_split;
  a.use_wave_req = waves <= ellm::MAX_WAVE_REQ ? 1 : 0;
  if (a.use_wave_req) {
    std::memset(a.wave_req, 0, sizeof(a.wave_req));
    int32_t i = 0;
    for (int64_t w = 0; w < waves; w++) {
      const int64_t lo = w * each + std::min<int64_t>(w, more);
      while (a.req[i].tile_prefix + (int64_t)tiles[i] <= lo) i++;
      a.wave_req[w >> 2] |= (uint32_t)i << ((w & 3) * 8);
    }
  }
  p->plan_total_tiles = total;
  p->plan_waves = waves;
  p->plan_slots = parts * p->geom.n_kv_heads;
}

// a debug hook can make the n-th launch from now fail as if the runtime had refused it
bool launch_refused(ellm_pool* p) { return p->fail_launch_in > 0 && --p->fail_launch_in == 0; }

}  // namespace

// ------------------------------------------------------------------------------------------------
extern "C" {

const char* ellm_last_error(void) { return g_last_error.c_str(); }

int ellm_pool_create(const ellm_pool_desc* d, ellm_pool** out) {
  if (!d || !out) return set_err(ELLM_ERR_INVALID, "pool_create: NULL argument");
  *out = nullptr;
  const bool meta = (d->flags & ELLM_POOL_METADATA_ONLY) != 0, vmm = (d->flags & ELLM_POOL_DRIVER_MAPPED) != 0;
  if (d->flags & ~(ELLM_POOL_METADATA_ONLY | ELLM_POOL_DRIVER_MAPPED) || d->reserved || (meta && vmm))
    return set_err(ELLM_ERR_INVALID, "pool_create: unknown flags");
  if (vmm && d->device_base) return set_err(ELLM_ERR_INVALID, "pool_create: a driver-mapped pool creates its own chunks; device_base must be NULL");
  if (d->dtype != ELLM_BF16) return set_err(ELLM_ERR_INVALID, "pool_create: dtype must be ELLM_BF16");
  if (d->head_dim != 64 && d->head_dim != 128) return set_err(ELLM_ERR_INVALID, "pool_create: head_dim must be 64 or 128");
  if (!d->n_kv_heads || !d->n_q_heads || d->n_q_heads % d->n_kv_heads || d->n_q_heads / d->n_kv_heads > 64)
    return set_err(ELLM_ERR_INVALID, "pool_create: n_q_heads must be a multiple (<= 64x) of n_kv_heads");
  if (!d->chunk_bytes || d->chunk_bytes % 256) return set_err(ELLM_ERR_INVALID, "pool_create: chunk_bytes must be a positive multiple of 256");
  const uint64_t bpt = 2ull * d->n_kv_heads * d->head_dim * 2ull;
  if (d->chunk_bytes < bpt) return set_err(ELLM_ERR_INVALID, "pool_create: a chunk must hold at least one token");
  const uint64_t n_chunks = d->device_bytes / d->chunk_bytes;
  const uint64_t n_host = d->host_bytes / d->chunk_bytes;
  if (n_chunks < 1 || n_chunks > 0x7ffffff0ull || n_host > 0x7ffffff0ull)
    return set_err(ELLM_ERR_INVALID, "pool_create: pool must hold between 1 and 2^31 chunks");
  if (!meta && !vmm && (!d->device_base || ((uintptr_t)d->device_base & 255)))
    return set_err(ELLM_ERR_INVALID, "pool_create: device_base must be a 256-byte aligned device pointer");
  if (!meta && n_host > 0 && !d->host_base) return set_err(ELLM_ERR_INVALID, "pool_create: host_base missing");
  if (!d->max_tensors || !d->max_slots_per_tensor ||
      (uint64_t)d->max_tensors * d->max_slots_per_tensor > 0x7fffffffull)
    return set_err(ELLM_ERR_INVALID, "pool_create: max_tensors * max_slots_per_tensor must be in 1 .. 2^31-1");
  if (d->initial_owner)
    for (uint64_t c = 0; c < n_chunks; c++)
      if (d->initial_owner[c] > ELLM_OWNER_ACT) return set_err(ELLM_ERR_INVALID, "pool_create: bad initial owner");

  ellm_pool* p = new ellm_pool();
  p->geom.n_chunks = (int32_t)n_chunks;
  p->geom.n_host_slots = (int32_t)n_host;
  p->geom.chunk_bytes = d->chunk_bytes;
  p->geom.bytes_per_token = bpt;
  p->geom.tokens_per_chunk = (int32_t)(d->chunk_bytes / bpt);
  p->geom.n_q_heads = d->n_q_heads;
  p->geom.n_kv_heads = d->n_kv_heads;
  p->geom.head_dim = d->head_dim;
  p->geom.group = d->n_q_heads / d->n_kv_heads;
  p->geom.max_tensors = (int32_t)d->max_tensors;
  p->geom.max_slots = (int32_t)d->max_slots_per_tensor;
  p->core.reset(new PoolCore(p->geom, d->initial_owner));
  p->device_base = (char*)d->device_base;
  p->host_base = (char*)d->host_base;
  p->metadata_only = meta;
  p->vmm = vmm;
  if (vmm) {
    const int rc = vmm_setup(p);
    if (rc) {
      vmm_teardown(p);
      delete p;
      return rc;
    }
  }
  *out = p;
  return ELLM_OK;
}

int ellm_pool_destroy(ellm_pool* p) {
  if (!p) return set_err(ELLM_ERR_INVALID, "pool_destroy: NULL pool");
  int rc = ELLM_OK;
  if (p->dev_ready) {
    if (hipStreamSynchronize(p->side_in) != hipSuccess) rc = ELLM_ERR_HIP;
    if (hipStreamSynchronize(p->side_out) != hipSuccess) rc = ELLM_ERR_HIP;
    if (p->have_last_stream && hipStreamSynchronize(p->last_stream) != hipSuccess) rc = ELLM_ERR_HIP;
    (void)hipStreamDestroy(p->side_in);
    (void)hipStreamDestroy(p->side_out);
    for (ellm_pool::Ring* r : {&p->r_compute, &p->r_in, &p->r_out})
      for (hipEvent_t e : r->ev) (void)hipEventDestroy(e);
    (void)hipFree(p->d_table);
    if (p->ev_switch) (void)hipEventDestroy(p->ev_switch);
    for (hipEvent_t e : p->prof_ev) (void)hipEventDestroy(e);
    if (p->d_ws) (void)hipFree(p->d_ws);
    if (p->d_vbase) (void)hipFree(p->d_vbase);
  }
  if (p->vmm) {
    if (hipDeviceSynchronize() != hipSuccess) rc = ELLM_ERR_HIP;
    vmm_teardown(p);
  }
  delete p;
  return rc;
}

int ellm_tensor_create(ellm_pool* p, int64_t max_tokens, ellm_tensor_id* out) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  return core_err(p, p->core->tensor_create(max_tokens, out));
}

int ellm_tensor_destroy(ellm_pool* p, ellm_tensor_id id) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  return core_changed(p, p->core->tensor_destroy(id));
}

int ellm_tensor_map_chunks(ellm_pool* p, ellm_tensor_id id, int32_t first_slot, int32_t n_slots,
                           const int32_t* chunk_ids, uint32_t flags) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  return core_changed(p, p->core->map_chunks(id, first_slot, n_slots, chunk_ids, flags));
}

int ellm_tensor_unmap_chunks(ellm_pool* p, ellm_tensor_id id, int32_t first_slot, int32_t n_slots) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  return core_changed(p, p->core->unmap_chunks(id, first_slot, n_slots));
}

int ellm_pool_transfer(ellm_pool* p, const int32_t* chunk_ids, int32_t n, int new_owner) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  int rc = core_err(p, p->core->transfer(chunk_ids, n, new_owner));
  if (rc || new_owner != ELLM_OWNER_ACT) return rc;
  return settle_copies(p, chunk_ids, n);     // an offload may still be reading a chunk it has just freed
}

int ellm_pool_set_act_busy(ellm_pool* p, const int32_t* chunk_ids, int32_t n, int busy) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  int rc = core_err(p, p->core->set_act_busy(chunk_ids, n, busy));
  if (rc || !busy) return rc;
  return settle_copies(p, chunk_ids, n);
}

int ellm_kv_append(ellm_pool* p, const ellm_tensor_id* ids, int32_t batch, const int32_t* n_new,
                   const void* k_new, const void* v_new, void* stream_) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  int64_t total = 0;
  int rc = core_err(p, p->core->append_check(ids, batch, n_new, p->n_eff, &total));
  if (rc) return rc;
  if (total > 0 && (!k_new || !v_new)) return set_err(ELLM_ERR_INVALID, "kv_append: NULL k_new / v_new");
  if (total > 0x7fffffffll / (2 * p->geom.n_kv_heads)) return set_err(ELLM_ERR_RANGE, "kv_append: too many tokens in one call");
  if (total == 0) return ELLM_OK;
  hipStream_t stream = (hipStream_t)stream_;
  int32_t most_new = 0;
  for (int32_t b = 0; b < batch; b++) most_new = std::max(most_new, n_new ? n_new[b] : 1);
  if (!p->metadata_only && (rc = enter_compute(p, stream, ids, batch, most_new))) return rc;
  // One launch per group of MAX_LAUNCH_REQ requests; a group's lengths advance as soon as its launch
  // has been accepted, so rows written and lengths agree at every point, also when the runtime
  // refuses a later launch.
  const size_t tok_bytes = (size_t)p->geom.n_kv_heads * p->geom.head_dim * 2;
  ellm::AppendArgs a;
  int64_t row0 = 0;
  int err = ELLM_OK;
  int32_t done = 0;
  for (int32_t b0 = 0; b0 < batch && !err; b0 += ellm::MAX_LAUNCH_REQ) {
    const int32_t nb = std::min<int32_t>(ellm::MAX_LAUNCH_REQ, batch - b0);
    a.n_req = nb;
    int32_t t = 0;
    for (int32_t i = 0; i < nb; i++) {
      a.tensor[i] = ids[b0 + i];
      a.len_before[i] = (int32_t)p->core->tensor(ids[b0 + i])->len;
      a.tok0[i] = t;
      t += p->n_eff[b0 + i];
    }
    a.total_new = t;
    if (t > 0 && launch_refused(p)) err = set_err(ELLM_ERR_HIP, "kv_append launch: refused (debug hook)");
    else if (t > 0 && !p->metadata_only) {
      const int e = ellm::launch_kv_append(view_of(p), (const char*)k_new + row0 * tok_bytes,
                                           (const char*)v_new + row0 * tok_bytes, a, stream);
      if (e) err = hip_err((hipError_t)e, "kv_append launch");
    }
    if (err) break;
    p->core->append_commit(ids + b0, nb, p->n_eff.data() + b0);
    done = b0 + nb;
    row0 += t;
  }
  if (!p->metadata_only && done > 0 && (rc = leave_compute(p, stream, ids, done))) return rc;
  return err;
}

int ellm_tensor_release(ellm_pool* p, ellm_tensor_id id) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  return core_changed(p, p->core->tensor_release(id));
}

int ellm_tensor_acquire(ellm_pool* p, int64_t need_tokens, int64_t max_tokens, uint32_t flags, ellm_tensor_id* out) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  if (flags & ~ELLM_MAP_ALLOW_INFLATE) return set_err(ELLM_ERR_INVALID, "tensor_acquire: unknown flags");
  return core_changed(p, p->core->tensor_acquire(need_tokens, max_tokens, flags, out));
}

int ellm_tensor_is_released(ellm_pool* p, ellm_tensor_id id) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  const ellm::TensorRec* t = p->core->tensor_any(id);
  if (!t) return set_err(ELLM_ERR_INVALID, "is_released: bad tensor handle");
  return t->released ? 1 : 0;
}

int ellm_kv_premap_next(ellm_pool* p, const ellm_tensor_id* ids, int32_t batch, uint32_t flags, int32_t* n_mapped) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  if (flags & ~ELLM_MAP_ALLOW_INFLATE) return set_err(ELLM_ERR_INVALID, "premap_next: unknown flags");
  return core_changed(p, p->core->premap_next(ids, batch, flags, n_mapped));
}

int ellm_kv_premap_ahead(ellm_pool* p, const ellm_tensor_id* ids, int32_t batch, int64_t tokens_ahead, uint32_t flags,
                         int32_t* n_mapped) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  if (flags & ~ELLM_MAP_ALLOW_INFLATE) return set_err(ELLM_ERR_INVALID, "premap_ahead: unknown flags");
  return core_changed(p, p->core->premap_ahead(ids, batch, tokens_ahead, flags, n_mapped));
}

int ellm_pool_flush_tables(ellm_pool* p, void* stream) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  if (p->metadata_only) return ELLM_OK;
  int rc = ensure_device(p);
  if (rc) return rc;
  return flush_table(p, (hipStream_t)stream);
}

int ellm_pool_set_logical_host_slots(ellm_pool* p, int32_t n) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  return core_err(p, p->core->set_logical_host_slots(n));
}

int ellm_pool_get_logical_host_slots(ellm_pool* p, int32_t* n) {
  if (!p || !n) return set_err(ELLM_ERR_INVALID, "get_logical_host_slots: NULL argument");
  *n = p->core->logical_host_slots();
  return ELLM_OK;
}

int ellm_pool_slo_configure(ellm_pool* p, double ttft_slo, double tpot_slo, double alpha, int32_t window, int32_t threshold) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  return core_err(p, p->core->slo_configure(ttft_slo, tpot_slo, alpha, window, threshold));
}

int ellm_pool_slo_observe(ellm_pool* p, double ttft, double tpot, int32_t* logical_host_slots) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  return core_err(p, p->core->slo_observe(ttft, tpot, logical_host_slots));
}

int ellm_decode_plan(ellm_pool* p, const ellm_tensor_id* ids, int32_t batch, int32_t* n_split, int32_t* split_tokens) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  int rc = core_err(p, p->core->decode_check(ids, batch));
  if (rc) return rc;
  ellm::BatchArgs a;
  int32_t per_wave = 0;
  for (int32_t b0 = 0; b0 < batch; b0 += ellm::MAX_LAUNCH_REQ) {
    const int32_t nb = std::min<int32_t>(ellm::MAX_LAUNCH_REQ, batch - b0);
    plan_launch(p, ids + b0, nb, b0, a);
    per_wave = std::max(per_wave, a.tiles_each + (a.tiles_extra > 0 ? 1 : 0));
    if (n_split)
      for (int32_t i = 0; i < nb; i++)
        n_split[b0 + i] = a.req[i].n_part;
  }
  if (split_tokens) *split_tokens = per_wave * ellm::TILE_TOKENS;
  return ELLM_OK;
}

int ellm_pool_set_split_tokens(ellm_pool* p, int32_t split_tokens) {
  if (!p || split_tokens < 0) return set_err(ELLM_ERR_INVALID, "set_split_tokens: bad argument");
  p->split_override = split_tokens;
  return ELLM_OK;
}

// decode over `ids`; with k_new / v_new the one-token append is fused into the same launches.
// ws / ws_cap_slots: where the partial results go. The launches of a call run one after the other
// on one stream, each followed by its combine pass, so all of them use the same workspace.
static int decode_impl(ellm_pool* p, const ellm_tensor_id* ids, int32_t batch, const void* q, const void* k_new,
                       const void* v_new, void* out, float scale, hipStream_t stream, int32_t* n_launched,
                       float* ws_fixed = nullptr, int64_t ws_fixed_slots = 0) {
  const int32_t extra = k_new ? 1 : 0;
  *n_launched = 0;               // requests whose launches the runtime has accepted
  // plan every launch first: a call that cannot run must not have launched anything
  std::vector<ellm::BatchArgs>& launches = p->launches;
  launches.clear();
  int64_t most_slots = 0;
  for (int32_t b0 = 0; b0 < batch; b0 += ellm::MAX_LAUNCH_REQ) {
    const int32_t nb = std::min<int32_t>(ellm::MAX_LAUNCH_REQ, batch - b0);
    launches.emplace_back();
    plan_launch(p, ids + b0, nb, b0, launches.back(), extra);
    if (p->plan_total_tiles > 0x7fffffffll || p->plan_waves * p->geom.n_kv_heads > 0x7fffffffll || p->plan_slots > 0x7fffffffll)
      return set_err(ELLM_ERR_RANGE, "decode_attention: too much work for one call");
    most_slots = std::max(most_slots, p->plan_slots);
  }
  if (ws_fixed && most_slots > ws_fixed_slots)
    return set_err(ELLM_ERR_RANGE, "decode_attention_noalloc: the batch needs more partial results than the fixed "
                                   "workspace of ELLM_NOALLOC_WORKSPACE_BYTES holds");
  int rc = enter_compute(p, stream, ids, batch, extra);
  if (rc) return rc;
  if (!ws_fixed && (rc = ensure_workspace(p, most_slots))) return rc;
  float* ws = ws_fixed ? ws_fixed : p->d_ws;
  if (scale == 0.f) scale = 1.0f / std::sqrt((float)p->geom.head_dim);
  const float scale_log2 = scale * 1.4426950408889634f;

  const ellm::PoolView pv = view_of(p);
  int err = ELLM_OK;
  for (const ellm::BatchArgs& a : launches) {
    bool prof = (size_t)(p->prof_used + 1) * 2 <= p->prof_ev.size();
    if (prof && p->prof_stride > 1) {
      prof = p->prof_phase == 0;
      p->prof_phase = (p->prof_phase + 1) % p->prof_stride;
    }
    if (launch_refused(p)) { err = set_err(ELLM_ERR_HIP, "decode partial launch: refused (debug hook)"); break; }
    int e = ellm::launch_decode_partial(pv, q, k_new, v_new, ws, out, scale_log2, a, stream,
                                        prof ? p->prof_ev[2 * p->prof_used] : nullptr,
                                        prof ? p->prof_ev[2 * p->prof_used + 1] : nullptr);
    if (e) { err = hip_err((hipError_t)e, "decode partial launch"); break; }
    *n_launched += a.n_req;
    if (prof) p->prof_used++;
    e = ellm::launch_decode_combine(pv, ws, out, a, stream);
    if (e) { err = hip_err((hipError_t)e, "decode combine launch"); break; }
  }
  // also after a refused launch: the chunks of the requests already launched are in use on the stream
  if (*n_launched > 0 && (rc = leave_compute(p, stream, ids, *n_launched)) && !err) err = rc;
  return err;
}

int ellm_decode_attention(ellm_pool* p, const ellm_tensor_id* ids, int32_t batch, const void* q, void* out,
                          float scale, void* stream_) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  if (batch < 0 || !q || !out || !std::isfinite(scale)) return set_err(ELLM_ERR_INVALID, "decode_attention: bad argument");
  int rc = core_err(p, p->core->decode_check(ids, batch));
  if (rc) return rc;
  if (batch == 0) return ELLM_OK;
  if (p->metadata_only) return set_err(ELLM_ERR_NO_DEVICE, "decode_attention: pool has no device");
  int32_t n_launched = 0;
  return decode_impl(p, ids, batch, q, nullptr, nullptr, out, scale, (hipStream_t)stream_, &n_launched);
}

int ellm_decode_attention_noalloc(ellm_pool* p, const ellm_tensor_id* ids, int32_t batch, const void* q, void* out,
                                  float scale, void* stream_) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  if (batch < 0 || !q || !out || !std::isfinite(scale)) return set_err(ELLM_ERR_INVALID, "decode_attention_noalloc: bad argument");
  int rc = core_err(p, p->core->decode_check(ids, batch));
  if (rc) return rc;
  if (batch == 0) return ELLM_OK;
  if (p->metadata_only) return set_err(ELLM_ERR_NO_DEVICE, "decode_attention_noalloc: pool has no device");
  if (!p->dev_ready)
    return set_err(ELLM_ERR_INVALID, "decode_attention_noalloc: the pool's device-side metadata does not exist yet and "
                                     "creating it allocates: call ellm_pool_prepare first");
  int32_t n_launched = 0;
  return decode_impl(p, ids, batch, q, nullptr, nullptr, out, scale, (hipStream_t)stream_, &n_launched, p->static_ws,
                     p->static_ws_slots);
}

int ellm_kv_append_decode(ellm_pool* p, const ellm_tensor_id* ids, int32_t batch, const void* k_new, const void* v_new,
                          const void* q, void* out, float scale, void* stream_) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  if (batch < 0 || !q || !out || !std::isfinite(scale)) return set_err(ELLM_ERR_INVALID, "kv_append_decode: bad argument");
  int rc = core_err(p, p->core->append_check(ids, batch, nullptr, p->n_eff, nullptr));
  if (rc) return rc;
  if (batch > 0 && (!k_new || !v_new)) return set_err(ELLM_ERR_INVALID, "kv_append_decode: NULL k_new / v_new");
  rc = core_err(p, p->core->decode_check(ids, batch, 1));
  if (rc) return rc;
  if (batch == 0) return ELLM_OK;
  if (p->metadata_only) return set_err(ELLM_ERR_NO_DEVICE, "kv_append_decode: pool has no device");
  // the kernels of a launch write the new rows, so the lengths of its requests advance with it
  int32_t n_launched = 0;
  rc = decode_impl(p, ids, batch, q, k_new, v_new, out, scale, (hipStream_t)stream_, &n_launched);
  p->core->append_commit(ids, n_launched, p->n_eff.data());
  return rc;
}

int ellm_chunk_deflate_to_host(ellm_pool* p, ellm_tensor_id id, int32_t first_slot, int32_t n_slots) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  int rc = core_err(p, p->core->offload_plan(id, first_slot, n_slots, p->moves));
  if (rc) return rc;
  if (!p->moves.empty() && !p->metadata_only) {
    rc = enter_migration(p, p->moves, false);
    if (rc) return rc;
    if ((rc = copy_chunks(p, p->moves, false))) return rc;
    rc = leave_migration(p, p->moves, false);
    if (rc) return rc;
  }
  p->core->offload_commit(id, p->moves);
  return core_changed(p, ELLM_OK);
}

int ellm_chunk_inflate_from_host(ellm_pool* p, ellm_tensor_id id, int32_t first_slot, int32_t n_slots,
                                 const int32_t* chunk_ids) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  int rc = core_err(p, p->core->fetch_plan(id, first_slot, n_slots, chunk_ids, p->moves));
  if (rc) return rc;
  if (!p->moves.empty() && !p->metadata_only) {
    rc = enter_migration(p, p->moves, true);
    if (rc) return rc;
    if ((rc = copy_chunks(p, p->moves, true))) return rc;
    rc = leave_migration(p, p->moves, true);
    if (rc) return rc;
  }
  p->core->fetch_commit(id, p->moves);
  return core_changed(p, ELLM_OK);
}

uint64_t ellm_workspace_bytes(const ellm_pool_desc* d, int32_t max_batch) {
  if (!d || max_batch < 1 || !d->n_kv_heads || !d->n_q_heads || d->n_q_heads % d->n_kv_heads ||
      (d->head_dim != 64 && d->head_dim != 128))
    return 0;
  const int32_t n_req = std::min<int32_t>(max_batch, ellm::MAX_LAUNCH_REQ);
  return (uint64_t)launch_slot_bound(device_simds(), d->n_kv_heads, n_req) *
         slot_bytes(d->n_q_heads / d->n_kv_heads, d->head_dim);
}

int ellm_pool_prepare(ellm_pool* p, void* stream) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  if (p->metadata_only) return ELLM_OK;
  int rc = ensure_device(p);
  if (rc) return rc;
  return flush_table(p, (hipStream_t)stream);
}

int ellm_pool_get_device_base(ellm_pool* p, void** base) {
  if (!p || !base) return set_err(ELLM_ERR_INVALID, "get_device_base: NULL argument");
  *base = p->device_base;
  return ELLM_OK;
}

int ellm_pool_get_mapping_stats(ellm_pool* p, int64_t* n_map, double* us_map, int64_t* n_unmap, double* us_unmap) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  int rc = vmm_drain(p);           // the figures are the mapper thread's: complete once it has nothing left to do
  if (rc) return rc;
  if (n_map) *n_map = p->mapq ? p->mapq->maps : 0;
  if (us_map) *us_map = p->mapq ? p->mapq->map_us : 0.0;
  if (n_unmap) *n_unmap = p->mapq ? p->mapq->unmaps : 0;
  if (us_unmap) *us_unmap = p->mapq ? p->mapq->unmap_us : 0.0;
  return ELLM_OK;
}

int ellm_pool_get_mapping_wait(ellm_pool* p, double* us_waited) {
  if (!p || !us_waited) return set_err(ELLM_ERR_INVALID, "get_mapping_wait: NULL argument");
  *us_waited = p->mapq ? p->mapq->waited_us() : 0.0;
  return ELLM_OK;
}

int ellm_debug_set_async_mapping(ellm_pool* p, int on) {
  if (!p || !p->vmm) return set_err(ELLM_ERR_INVALID, "set_async_mapping: not a driver-mapped pool");
  p->vmm_async = on != 0;
  return p->vmm_async ? ELLM_OK : vmm_drain(p);
}

int ellm_debug_fail_mapping(ellm_pool* p, int32_t nth) {
  if (!p || !p->vmm || nth < 0) return set_err(ELLM_ERR_INVALID, "fail_mapping: bad argument");
  p->mapq->fail_map_in(nth);
  return ELLM_OK;
}

int ellm_debug_set_copy_kernels(ellm_pool* p, int on) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  p->copy_kernels = on != 0;
  return ELLM_OK;
}

int ellm_debug_set_table_kernels(ellm_pool* p, int on) {
  if (!p || !p->vmm) return set_err(ELLM_ERR_INVALID, "set_table_kernels: not a driver-mapped pool");
  p->vmm_table_kernels = on != 0;
  return ELLM_OK;
}

int ellm_debug_fail_launch(ellm_pool* p, int32_t nth) {
  if (!p || nth < 0) return set_err(ELLM_ERR_INVALID, "debug_fail_launch: bad argument");
  p->fail_launch_in = nth;
  return ELLM_OK;
}

int ellm_pool_sync(ellm_pool* p) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  int rc = vmm_drain(p);
  if (rc) return rc;
  if (!p->dev_ready) return ELLM_OK;
  HIP_TRY(hipStreamSynchronize(p->side_in), "hipStreamSynchronize(side)");
  p->r_in.done = p->r_in.seq;
  HIP_TRY(hipStreamSynchronize(p->side_out), "hipStreamSynchronize(side)");
  p->r_out.done = p->r_out.seq;
  return ELLM_OK;
}

int ellm_pool_get_geometry(ellm_pool* p, int32_t* n_chunks, int32_t* tokens_per_chunk, int32_t* n_host_slots,
                           uint64_t* bytes_per_token) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  if (n_chunks) *n_chunks = p->geom.n_chunks;
  if (tokens_per_chunk) *tokens_per_chunk = p->geom.tokens_per_chunk;
  if (n_host_slots) *n_host_slots = p->geom.n_host_slots;
  if (bytes_per_token) *bytes_per_token = p->geom.bytes_per_token;
  return ELLM_OK;
}

int ellm_tensor_get_table(ellm_pool* p, ellm_tensor_id id, int32_t* out, int32_t cap, int32_t* n_slots, int64_t* len) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  const ellm::TensorRec* t = p->core->tensor_any(id);
  if (!t) return set_err(ELLM_ERR_INVALID, "get_table: bad tensor handle");
  if (out && cap > 0) std::memcpy(out, p->core->row(id), sizeof(int32_t) * (size_t)std::min(cap, t->n_slots));
  if (n_slots) *n_slots = t->n_slots;
  if (len) *len = t->len;
  return ELLM_OK;
}

int ellm_pool_get_owner_state(ellm_pool* p, uint8_t* owner, uint8_t* state, int32_t* mapped_tensor, int32_t* mapped_slot) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  const size_t n = (size_t)p->geom.n_chunks;
  if (owner) std::memcpy(owner, p->core->owner().data(), n);
  if (state) std::memcpy(state, p->core->state().data(), n);
  if (mapped_tensor) std::memcpy(mapped_tensor, p->core->map_tensor().data(), n * sizeof(int32_t));
  if (mapped_slot) std::memcpy(mapped_slot, p->core->map_slot().data(), n * sizeof(int32_t));
  return ELLM_OK;
}

int ellm_pool_get_host_slots(ellm_pool* p, int32_t* tensor, int32_t* slot) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  const size_t n = (size_t)p->geom.n_host_slots;
  if (tensor && n) std::memcpy(tensor, p->core->host_tensor().data(), n * sizeof(int32_t));
  if (slot && n) std::memcpy(slot, p->core->host_slot().data(), n * sizeof(int32_t));
  return ELLM_OK;
}

int ellm_pool_profile_enable(ellm_pool* p, int32_t max_records) {
  if (!p || max_records < 0) return set_err(ELLM_ERR_INVALID, "profile_enable: bad argument");
  if (p->metadata_only) return set_err(ELLM_ERR_NO_DEVICE, "profile_enable: pool has no device");
  for (hipEvent_t e : p->prof_ev) (void)hipEventDestroy(e);
  p->prof_ev.clear();
  p->prof_used = 0;
  for (int32_t i = 0; i < 2 * max_records; i++) {
    hipEvent_t e;
    HIP_TRY(hipEventCreate(&e), "hipEventCreate(profile)");
    p->prof_ev.push_back(e);
  }
  return ELLM_OK;
}

int ellm_pool_profile_stride(ellm_pool* p, int32_t stride) {
  if (!p || stride < 1) return set_err(ELLM_ERR_INVALID, "profile_stride: bad argument");
  p->prof_stride = stride;
  p->prof_phase = 0;
  return ELLM_OK;
}

int ellm_pool_profile_collect(ellm_pool* p, float* ms, int32_t cap, int32_t* n) {
  if (!p || cap < 0 || (cap > 0 && !ms)) return set_err(ELLM_ERR_INVALID, "profile_collect: bad argument");
  const int32_t m = std::min(cap, p->prof_used);
  for (int32_t i = 0; i < m; i++) {
    HIP_TRY(hipEventSynchronize(p->prof_ev[2 * i + 1]), "hipEventSynchronize(profile)");
    HIP_TRY(hipEventElapsedTime(&ms[i], p->prof_ev[2 * i], p->prof_ev[2 * i + 1]), "hipEventElapsedTime(profile)");
  }
  if (n) *n = p->prof_used;
  p->prof_used = 0;
  return ELLM_OK;
}

int ellm_debug_copy(void* dst, const void* src, uint64_t bytes, void* stream) {
  if (!dst || !src || bytes % 16) return set_err(ELLM_ERR_INVALID, "debug_copy: bad argument");
  int e = ellm::launch_copy(dst, src, (int64_t)bytes, (hipStream_t)stream);
  if (e) return hip_err((hipError_t)e, "copy launch");
  return ELLM_OK;
}

int ellm_debug_stream_read(const void* src, uint64_t bytes, void* sink, void* stream) {
  if (!src || !sink || bytes % 16) return set_err(ELLM_ERR_INVALID, "debug_stream_read: bad argument");
  int e = ellm::launch_read(src, (int64_t)bytes, (uint32_t*)sink, (hipStream_t)stream);
  if (e) return hip_err((hipError_t)e, "read launch");
  return ELLM_OK;
}

int ellm_debug_kv_stream_read(ellm_pool* p, const ellm_tensor_id* ids, int32_t batch, void* sink, void* stream_) {
  if (!p || !sink) return set_err(ELLM_ERR_INVALID, "debug_kv_stream_read: bad argument");
  int rc = core_err(p, p->core->decode_check(ids, batch));
  if (rc) return rc;
  if (batch == 0) return ELLM_OK;
  if (p->metadata_only) return set_err(ELLM_ERR_NO_DEVICE, "debug_kv_stream_read: pool has no device");
  hipStream_t stream = (hipStream_t)stream_;
  rc = enter_compute(p, stream, ids, batch, 0);
  if (rc) return rc;
  const ellm::PoolView pv = view_of(p);
  ellm::BatchArgs a;
  for (int32_t b0 = 0; b0 < batch; b0 += ellm::MAX_LAUNCH_REQ) {
    const int32_t nb = std::min<int32_t>(ellm::MAX_LAUNCH_REQ, batch - b0);
    plan_launch(p, ids + b0, nb, b0, a);
    int e = ellm::launch_kv_stream(pv, (uint32_t*)sink, a, stream);
    if (e) return hip_err((hipError_t)e, "kv stream launch");
  }
  return leave_compute(p, stream, ids, batch);
}

int ellm_debug_set_waves(ellm_pool* p, int32_t percent) {
  if (!p || percent < 1 || percent > 1600) return set_err(ELLM_ERR_INVALID, "set_waves: bad argument");
  p->waves_percent = percent;
  return ELLM_OK;
}

// The paper's own mechanism, measured for comparison: chunks created as physical allocations and
// mapped into a reserved virtual range with the driver's virtual-memory calls.
int ellm_debug_vmm_latency(uint64_t chunk_bytes, int32_t n_chunks, double* us) {
  if (!us || n_chunks < 1 || n_chunks > 4096 || chunk_bytes == 0) return set_err(ELLM_ERR_INVALID, "vmm_latency: bad argument");
  using clk = std::chrono::steady_clock;
  auto since = [](clk::time_point t0) { return std::chrono::duration<double, std::micro>(clk::now() - t0).count(); };
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
  hipMemAllocationProp prop = {};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = dev;
  size_t gran = 0;
  HIP_TRY(hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityMinimum), "hipMemGetAllocationGranularity");
  const size_t cb = ((size_t)chunk_bytes + gran - 1) / gran * gran;
  void* va = nullptr;
  HIP_TRY(hipMemAddressReserve(&va, cb * n_chunks, 0, nullptr, 0), "hipMemAddressReserve");
  std::vector<hipMemGenericAllocationHandle_t> h(n_chunks);
  hipMemAccessDesc acc = {};
  acc.location = prop.location;
  acc.flags = hipMemAccessFlagsProtReadWrite;
  int created = 0, mapped = 0, rc = ELLM_OK;
  hipError_t e = hipSuccess;
  auto t0 = clk::now();
  for (; created < n_chunks; created++)
    if ((e = hipMemCreate(&h[created], cb, &prop, 0)) != hipSuccess) break;
  us[0] = since(t0) / std::max(created, 1);
  if (e == hipSuccess) {
    t0 = clk::now();
    for (; mapped < n_chunks; mapped++) {
      if ((e = hipMemMap((char*)va + (size_t)mapped * cb, cb, 0, h[mapped], 0)) != hipSuccess) break;
      if ((e = hipMemSetAccess((char*)va + (size_t)mapped * cb, cb, &acc, 1)) != hipSuccess) { mapped++; break; }
    }
    us[1] = since(t0) / std::max(mapped, 1);
  }
  if (e == hipSuccess) e = hipMemset(va, 0, cb * n_chunks);       // the mapping is usable
  if (e == hipSuccess) e = hipDeviceSynchronize();
  t0 = clk::now();
  for (int i = 0; i < mapped; i++) (void)hipMemUnmap((char*)va + (size_t)i * cb, cb);
  us[2] = since(t0) / std::max(mapped, 1);
  t0 = clk::now();
  for (int i = 0; i < created; i++) (void)hipMemRelease(h[i]);
  us[3] = since(t0) / std::max(created, 1);
  (void)hipMemAddressFree(va, cb * n_chunks);
  if (e != hipSuccess) rc = hip_err(e, "virtual-memory call");
  return rc;
}

// A buffer whose 2 MiB (or chunk-sized) pieces are separate physical allocations mapped into one
// reserved virtual range by the driver, in a shuffled order: what a pool looks like under the
// paper's mechanism (Sec. 2.1.1, Sec. 3.2) once chunks have been mapped and unmapped for a while.
namespace {
struct VmmBuffer {
  size_t piece = 0;
  std::vector<hipMemGenericAllocationHandle_t> handles;
  int mapped = 0;
};
std::map<void*, VmmBuffer> g_vmm_buffers;
}  // namespace

int ellm_debug_vmm_buffer_create(uint64_t chunk_bytes, int32_t n_chunks, uint32_t seed, uint16_t fill16, void** base,
                                 uint64_t* bytes) {
  if (!base || !bytes || n_chunks < 1 || n_chunks > (1 << 20) || chunk_bytes == 0)
    return set_err(ELLM_ERR_INVALID, "vmm_buffer_create: bad argument");
  *base = nullptr;
  *bytes = 0;
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
  hipMemAllocationProp prop = {};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = dev;
  size_t gran = 0;
  HIP_TRY(hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityMinimum), "hipMemGetAllocationGranularity");
  if (chunk_bytes % gran)
    return set_err(ELLM_ERR_INVALID, "vmm_buffer_create: chunk_bytes must be a multiple of the driver's allocation granularity");
  const size_t cb = (size_t)chunk_bytes;
  void* va = nullptr;
  HIP_TRY(hipMemAddressReserve(&va, cb * n_chunks, 0, nullptr, 0), "hipMemAddressReserve");
  VmmBuffer buf;
  buf.piece = cb;
  buf.handles.resize(n_chunks);
  hipError_t e = hipSuccess;
  int created = 0;
  for (; created < n_chunks; created++)
    if ((e = hipMemCreate(&buf.handles[created], cb, &prop, 0)) != hipSuccess) break;
  // physical piece order[i] backs virtual piece i
  std::vector<int32_t> order(n_chunks);
  for (int32_t i = 0; i < n_chunks; i++) order[i] = i;
  uint64_t x = 0x9E3779B97F4A7C15ull ^ seed;
  for (int32_t i = n_chunks - 1; i > 0; i--) {
    x = x * 6364136223846793005ull + 1442695040888963407ull;
    std::swap(order[i], order[(int32_t)((x >> 33) % (uint64_t)(i + 1))]);
  }
  hipMemAccessDesc acc = {};
  acc.location = prop.location;
  acc.flags = hipMemAccessFlagsProtReadWrite;
  if (e == hipSuccess)
    for (; buf.mapped < n_chunks; buf.mapped++)
      if ((e = hipMemMap((char*)va + (size_t)buf.mapped * cb, cb, 0, buf.handles[order[buf.mapped]], 0)) != hipSuccess) break;
  if (e == hipSuccess) e = hipMemSetAccess(va, cb * n_chunks, &acc, 1);
  if (e == hipSuccess) e = hipMemsetD16(va, fill16, cb * n_chunks / 2);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    for (int i = 0; i < buf.mapped; i++) (void)hipMemUnmap((char*)va + (size_t)i * cb, cb);
    for (int i = 0; i < created; i++) (void)hipMemRelease(buf.handles[i]);
    (void)hipMemAddressFree(va, cb * n_chunks);
    return hip_err(e, "virtual-memory call");
  }
  g_vmm_buffers[va] = std::move(buf);
  *base = va;
  *bytes = cb * n_chunks;
  return ELLM_OK;
}

int ellm_debug_vmm_buffer_destroy(void* base) {
  auto it = g_vmm_buffers.find(base);
  if (it == g_vmm_buffers.end()) return set_err(ELLM_ERR_INVALID, "vmm_buffer_destroy: not a buffer of vmm_buffer_create");
  HIP_TRY(hipDeviceSynchronize(), "hipDeviceSynchronize");
  VmmBuffer& b = it->second;
  const size_t n = b.handles.size();
  for (int i = 0; i < b.mapped; i++) (void)hipMemUnmap((char*)base + (size_t)i * b.piece, b.piece);
  for (size_t i = 0; i < n; i++) (void)hipMemRelease(b.handles[i]);
  (void)hipMemAddressFree(base, b.piece * n);
  g_vmm_buffers.erase(it);
  return ELLM_OK;
}

int ellm_pool_self_check(ellm_pool* p) {
  if (!p) return set_err(ELLM_ERR_INVALID, "NULL pool");
  return p->core->self_check();
}

}  // extern "C"
