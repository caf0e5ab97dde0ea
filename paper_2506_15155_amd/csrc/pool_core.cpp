// Host-side pool and chunk-table state machine. See pool_core.hpp.
#include "pool_core.hpp"

#include <algorithm>
#include <cmath>
#include <cstdio>

namespace ellm {

PoolCore::PoolCore(const Geometry& g, const uint8_t* initial_owner) : g_(g) {
  owner_.assign(g.n_chunks, OWNER_KV);
  state_.assign(g.n_chunks, CHUNK_FREE);
  map_tensor_.assign(g.n_chunks, -1);
  map_slot_.assign(g.n_chunks, -1);
  host_tensor_.assign(g.n_host_slots, -1);
  host_slot_.assign(g.n_host_slots, -1);
  for (int32_t c = 0; c < g.n_chunks; c++) {
    if (initial_owner && initial_owner[c] == OWNER_ACT) { owner_[c] = OWNER_ACT; free_act_.insert(free_act_.end(), c); }
    else free_kv_.insert(free_kv_.end(), c);
  }
  for (int32_t s = 0; s < g.n_host_slots; s++) free_host_.insert(free_host_.end(), s);
  logical_host_ = g.n_host_slots;
  for (int32_t i = 0; i < g.max_tensors; i++) free_ids_.insert(free_ids_.end(), i);
  t_.resize(g.max_tensors);
  table_.assign((size_t)g.max_tensors * g.max_slots, ENTRY_UNMAPPED);
  row_version_.assign(g.max_tensors, 0u);
  stamp_.assign((size_t)std::max(g.n_chunks, g.max_tensors), 0u);
}

int PoolCore::fail(int code, const char* what) {
  err_ = what;
  return code;
}

void PoolCore::set_entry(int32_t id, int32_t slot, int32_t value) {
  int64_t flat = (int64_t)id * g_.max_slots + slot;
  if (table_[flat] != value) {
    table_[flat] = value;
    dirty_.push_back(flat);
    if (map_log_) map_dirty_.push_back(flat);
    row_version_[id]++;
  }
}

std::vector<int64_t> PoolCore::take_dirty() {
  std::sort(dirty_.begin(), dirty_.end());
  dirty_.erase(std::unique(dirty_.begin(), dirty_.end()), dirty_.end());
  std::vector<int64_t> out;
  out.swap(dirty_);
  return out;
}

std::vector<int64_t> PoolCore::take_map_changes() {
  std::sort(map_dirty_.begin(), map_dirty_.end());
  map_dirty_.erase(std::unique(map_dirty_.begin(), map_dirty_.end()), map_dirty_.end());
  std::vector<int64_t> out;
  out.swap(map_dirty_);
  return out;
}

void PoolCore::release_entry(int32_t e) {
  if (e >= 0) {
    state_[e] = CHUNK_FREE;
    map_tensor_[e] = map_slot_[e] = -1;
    (owner_[e] == OWNER_KV ? free_kv_ : free_act_).insert(e);
  } else if (e <= -2) {
    int32_t hs = host_slot_of_entry(e);
    host_tensor_[hs] = host_slot_[hs] = -1;
    free_host_.insert(hs);
  }
}

void PoolCore::take_chunk(int32_t c, int32_t id, int32_t slot) {
  (owner_[c] == OWNER_KV ? free_kv_ : free_act_).erase(c);
  owner_[c] = OWNER_KV;            // a borrowed activation chunk changes sides (Sec. 2.2.1 step 3)
  state_[c] = CHUNK_MAPPED;
  map_tensor_[c] = id;
  map_slot_[c] = slot;
  set_entry(id, slot, c);
}

int PoolCore::tensor_create(int64_t max_tokens, int32_t* out) {
  if (!out || max_tokens < 1) return fail(ERR_INVALID, "tensor_create: max_tokens must be >= 1");
  int64_t ns = (max_tokens + g_.tokens_per_chunk - 1) / g_.tokens_per_chunk;
  if (ns > g_.max_slots) return fail(ERR_RANGE, "tensor_create: max_tokens needs more slots than max_slots_per_tensor");
  if (free_ids_.empty()) return fail(ERR_OOM, "tensor_create: no free tensor handle");
  int32_t id = *free_ids_.begin();
  free_ids_.erase(free_ids_.begin());
  TensorRec& t = t_[id];
  t.used = true; t.max_tokens = max_tokens; t.len = 0; t.n_slots = (int32_t)ns;
  *out = id;
  return OK;
}

int PoolCore::tensor_destroy(int32_t id) {
  if (!tensor_any(id)) return fail(ERR_INVALID, "tensor_destroy: bad tensor handle");
  TensorRec& t = t_[id];
  if (t.released) released_.erase({t.run, id});
  for (int32_t s = 0; s < t.n_slots; s++) {
    release_entry(row(id)[s]);
    set_entry(id, s, ENTRY_UNMAPPED);
  }
  t = TensorRec();
  free_ids_.insert(id);
  return OK;
}

int PoolCore::tensor_release(int32_t id) {
  if (!tensor(id)) return fail(ERR_INVALID, "tensor_release: bad or already released tensor handle");
  TensorRec& t = t_[id];
  int32_t run = 0;
  while (run < t.n_slots && row(id)[run] >= 0) run++;
  for (int32_t s = run; s < t.n_slots; s++) {
    if (row(id)[s] == ENTRY_UNMAPPED) continue;
    release_entry(row(id)[s]);
    set_entry(id, s, ENTRY_UNMAPPED);
  }
  t.len = 0;
  t.released = true;
  t.run = run;
  released_.insert({run, id});
  return OK;
}

int PoolCore::tensor_acquire(int64_t need, int64_t max_tokens, uint32_t flags, int32_t* out) {
  const int64_t Tc = g_.tokens_per_chunk;
  if (!out || need < 0 || max_tokens < 1 || need > max_tokens)
    return fail(ERR_INVALID, "tensor_acquire: need_tokens must be in 0 .. max_tokens, max_tokens >= 1");
  if ((max_tokens + Tc - 1) / Tc > g_.max_slots)
    return fail(ERR_RANGE, "tensor_acquire: max_tokens needs more slots than max_slots_per_tensor");
  const int32_t n = (int32_t)((need + Tc - 1) / Tc);
  // best fit: released_ is ordered by (mapped slots, handle), so the first entry at or above n whose
  // virtual range suffices has the smallest sufficient size and, among equals, the lowest handle
  for (auto it = released_.lower_bound({n, -1}); it != released_.end(); ++it) {
    TensorRec& t = t_[it->second];
    if (t.max_tokens < max_tokens) continue;
    *out = it->second;
    released_.erase(it);
    t.released = false;
    t.run = 0;
    t.len = 0;
    return OK;
  }
  // on-demand mapping of a fresh tensor: plan first, change nothing on failure
  if (free_ids_.empty()) return fail(ERR_OOM, "tensor_acquire: no fitting available tensor and no free tensor handle");
  std::vector<int32_t> pick;
  pick.reserve(n);
  for (auto it = free_kv_.begin(); it != free_kv_.end() && (int32_t)pick.size() < n; ++it) pick.push_back(*it);
  std::vector<std::pair<int32_t, int32_t>> donors;   // (handle, slots taken back from its tail)
  for (auto it = released_.begin(); it != released_.end() && (int32_t)pick.size() < n; ++it) {
    if (it->first == 0) continue;
    int32_t left = it->first, took = 0;
    while ((int32_t)pick.size() < n && left > 0) {
      pick.push_back(row(it->second)[left - 1]);
      left--;
      took++;
    }
    donors.push_back({it->second, took});
  }
  if ((int32_t)pick.size() < n && (flags & 1u))
    for (auto it = free_act_.begin(); it != free_act_.end() && (int32_t)pick.size() < n; ++it) pick.push_back(*it);
  if ((int32_t)pick.size() < n) return fail(ERR_OOM, "tensor_acquire: not enough chunks for on-demand mapping");
  for (const auto& d : donors) {
    TensorRec& t = t_[d.first];
    released_.erase({t.run, d.first});
    for (int32_t s = t.run - d.second; s < t.run; s++) {
      release_entry(row(d.first)[s]);
      set_entry(d.first, s, ENTRY_UNMAPPED);
    }
    t.run -= d.second;
    released_.insert({t.run, d.first});
  }
  int32_t id = -1;
  int rc = tensor_create(max_tokens, &id);
  if (rc) return rc;
  for (int32_t i = 0; i < n; i++) take_chunk(pick[i], id, i);
  *out = id;
  return OK;
}

int PoolCore::set_logical_host_slots(int32_t n) {
  if (n < 0 || n > g_.n_host_slots) return fail(ERR_RANGE, "set_logical_host_slots: outside 0 .. host slots");
  logical_host_ = n;
  return OK;
}

int PoolCore::slo_configure(double ttft_slo, double tpot_slo, double alpha, int32_t window, int32_t threshold) {
  if (!(ttft_slo > 0) || !(tpot_slo > 0) || !(alpha > 1) || window < 1 || threshold < 1 || threshold > window)
    return fail(ERR_INVALID, "slo_configure: need positive thresholds, alpha > 1, 1 <= threshold <= window");
  slo_ = Slo();
  slo_.on = true;
  slo_.ttft = ttft_slo; slo_.tpot = tpot_slo; slo_.alpha = alpha;
  slo_.window = window; slo_.threshold = threshold;
  return OK;
}

// One scheduling iteration's latencies (a negative value: none measured in this iteration). A
// violation event is `threshold` iterations over the SLO among the last `window`; time per output
// token over -> the buffer shrinks by alpha, time to first token over -> it grows by alpha; both at
// once -> it shrinks. After a change the count starts again.
int PoolCore::slo_observe(double ttft, double tpot, int32_t* logical_out) {
  if (!slo_.on) return fail(ERR_INVALID, "slo_observe: not configured");
  if (ttft != ttft || tpot != tpot) return fail(ERR_INVALID, "slo_observe: NaN latency");
  slo_.ttft_hits.push_back(ttft > slo_.ttft ? 1 : 0);
  slo_.tpot_hits.push_back(tpot > slo_.tpot ? 1 : 0);
  if ((int32_t)slo_.ttft_hits.size() > slo_.window) {
    slo_.ttft_hits.erase(slo_.ttft_hits.begin());
    slo_.tpot_hits.erase(slo_.tpot_hits.begin());
  }
  int32_t n_ttft = 0, n_tpot = 0;
  for (uint8_t h : slo_.ttft_hits) n_ttft += h;
  for (uint8_t h : slo_.tpot_hits) n_tpot += h;
  if (n_tpot >= slo_.threshold) {
    logical_host_ = (int32_t)std::floor((double)logical_host_ / slo_.alpha);
    slo_.ttft_hits.clear(); slo_.tpot_hits.clear();
  } else if (n_ttft >= slo_.threshold) {
    const double grown = std::ceil(std::max(1.0, (double)logical_host_) * slo_.alpha);
    logical_host_ = (int32_t)std::min<double>(g_.n_host_slots, grown);
    slo_.ttft_hits.clear(); slo_.tpot_hits.clear();
  }
  if (logical_out) *logical_out = logical_host_;
  return OK;
}

int PoolCore::premap_next(const int32_t* ids, int32_t batch, uint32_t flags, int32_t* n_mapped) {
  if (batch < 0 || (batch > 0 && !ids)) return fail(ERR_INVALID, "premap_next: bad batch");
  const int64_t Tc = g_.tokens_per_chunk;
  ++stamp_now_;
  int32_t need = 0;
  auto opens_slot = [&](int32_t id) {
    const TensorRec& t = t_[id];
    return t.len < t.max_tokens && t.len % Tc == 0 && row(id)[t.len / Tc] == ENTRY_UNMAPPED;
  };
  for (int32_t b = 0; b < batch; b++) {
    if (!tensor(ids[b])) return fail(ERR_INVALID, "premap_next: bad tensor handle");
    if (stamp_[ids[b]] == stamp_now_) return fail(ERR_INVALID, "premap_next: tensor handle given twice");
    stamp_[ids[b]] = stamp_now_;
    if (opens_slot(ids[b])) need++;
  }
  std::vector<int32_t> pick;
  int rc = pick_chunks(need, nullptr, (flags & 1u) != 0, pick);
  if (rc) return rc;
  int32_t k = 0;
  for (int32_t b = 0; b < batch; b++)
    if (opens_slot(ids[b])) {
      take_chunk(pick[k], ids[b], (int32_t)(t_[ids[b]].len / Tc));
      k++;
    }
  if (n_mapped) *n_mapped = need;
  return OK;
}

int PoolCore::premap_ahead(const int32_t* ids, int32_t batch, int64_t tokens_ahead, uint32_t flags, int32_t* n_mapped) {
  if (batch < 0 || (batch > 0 && !ids)) return fail(ERR_INVALID, "premap_ahead: bad batch");
  if (tokens_ahead < 1) return fail(ERR_INVALID, "premap_ahead: tokens_ahead must be at least 1");
  const int64_t Tc = g_.tokens_per_chunk;
  ++stamp_now_;
  // slots [first, last) of a tensor are the ones its next tokens_ahead tokens are written to
  auto span = [&](int32_t id, int64_t* first, int64_t* last) {
    const TensorRec& t = t_[id];
    const int64_t until = std::min<int64_t>(t.len + tokens_ahead, t.max_tokens);
    *first = t.len / Tc;
    *last = until > t.len ? (until + Tc - 1) / Tc : *first;
  };
  int64_t need = 0;
  for (int32_t b = 0; b < batch; b++) {
    if (!tensor(ids[b])) return fail(ERR_INVALID, "premap_ahead: bad tensor handle");
    if (stamp_[ids[b]] == stamp_now_) return fail(ERR_INVALID, "premap_ahead: tensor handle given twice");
    stamp_[ids[b]] = stamp_now_;
    int64_t first, last;
    span(ids[b], &first, &last);
    const int32_t* r = row(ids[b]);
    for (int64_t s = first; s < last; s++)
      if (r[s] == ENTRY_UNMAPPED) need++;
  }
  if (need > 0x7fffffffll) return fail(ERR_OOM, "not enough free chunks");
  std::vector<int32_t> pick;
  int rc = pick_chunks((int32_t)need, nullptr, (flags & 1u) != 0, pick);
  if (rc) return rc;
  int32_t k = 0;
  for (int32_t b = 0; b < batch; b++) {
    int64_t first, last;
    span(ids[b], &first, &last);
    for (int64_t s = first; s < last; s++)
      if (row(ids[b])[s] == ENTRY_UNMAPPED) take_chunk(pick[k++], ids[b], (int32_t)s);
  }
  if (n_mapped) *n_mapped = (int32_t)need;
  return OK;
}

int PoolCore::pick_chunks(int32_t n, const int32_t* ids, bool inflate, std::vector<int32_t>& out) {
  out.clear();
  out.reserve(n);
  if (ids) {
    ++stamp_now_;
    for (int32_t i = 0; i < n; i++) {
      int32_t c = ids[i];
      if (c < 0 || c >= g_.n_chunks) return fail(ERR_RANGE, "chunk id outside the pool");
      if (state_[c] != CHUNK_FREE) return fail(ERR_OWNED, "chunk is mapped or busy");
      if (stamp_[c] == stamp_now_) return fail(ERR_OWNED, "chunk id given twice");
      if (owner_[c] == OWNER_ACT && !inflate) return fail(ERR_OWNED, "chunk belongs to the activation side");
      stamp_[c] = stamp_now_;
      out.push_back(c);
    }
    return OK;
  }
  for (auto it = free_kv_.begin(); it != free_kv_.end() && (int32_t)out.size() < n; ++it) out.push_back(*it);
  if ((int32_t)out.size() < n && inflate)
    for (auto it = free_act_.begin(); it != free_act_.end() && (int32_t)out.size() < n; ++it) out.push_back(*it);
  if ((int32_t)out.size() < n) return fail(ERR_OOM, "not enough free chunks");
  return OK;
}

int PoolCore::map_chunks(int32_t id, int32_t first, int32_t n, const int32_t* chunk_ids, uint32_t flags) {
  const TensorRec* t = tensor(id);
  if (!t || n < 0) return fail(ERR_INVALID, "map_chunks: bad tensor handle or negative count");
  if (n == 0) return OK;
  if (first < 0 || (int64_t)first + n > t->n_slots) return fail(ERR_RANGE, "map_chunks: slot range outside the tensor");
  for (int32_t i = 0; i < n; i++)
    if (row(id)[first + i] != ENTRY_UNMAPPED) return fail(ERR_INVALID, "map_chunks: slot already has a chunk");
  std::vector<int32_t> pick;
  int rc = pick_chunks(n, chunk_ids, (flags & 1u) != 0, pick);
  if (rc) return rc;
  for (int32_t i = 0; i < n; i++) take_chunk(pick[i], id, first + i);
  return OK;
}

int PoolCore::unmap_chunks(int32_t id, int32_t first, int32_t n) {
  const TensorRec* t = tensor(id);
  if (!t || n < 0) return fail(ERR_INVALID, "unmap_chunks: bad tensor handle or negative count");
  if (n == 0) return OK;
  if (first < 0 || (int64_t)first + n > t->n_slots) return fail(ERR_RANGE, "unmap_chunks: slot range outside the tensor");
  int64_t live = (t->len + g_.tokens_per_chunk - 1) / g_.tokens_per_chunk;
  if (first < live) return fail(ERR_INVALID, "unmap_chunks: slot holds live tokens");
  for (int32_t i = 0; i < n; i++)
    if (row(id)[first + i] == ENTRY_UNMAPPED) return fail(ERR_UNMAPPED, "unmap_chunks: slot has no chunk");
  for (int32_t i = 0; i < n; i++) {
    release_entry(row(id)[first + i]);
    set_entry(id, first + i, ENTRY_UNMAPPED);
  }
  return OK;
}

int PoolCore::transfer(const int32_t* ids, int32_t n, int new_owner) {
  if (n < 0 || (new_owner != OWNER_KV && new_owner != OWNER_ACT) || (n > 0 && !ids))
    return fail(ERR_INVALID, "transfer: bad count or owner");
  ++stamp_now_;
  for (int32_t i = 0; i < n; i++) {
    int32_t c = ids[i];
    if (c < 0 || c >= g_.n_chunks) return fail(ERR_RANGE, "transfer: chunk id outside the pool");
    if (state_[c] != CHUNK_FREE) return fail(ERR_OWNED, "transfer: chunk is mapped or busy");
    if (stamp_[c] == stamp_now_) return fail(ERR_INVALID, "transfer: chunk id given twice");
    stamp_[c] = stamp_now_;
  }
  for (int32_t i = 0; i < n; i++) {
    int32_t c = ids[i];
    if (owner_[c] == new_owner) continue;
    (owner_[c] == OWNER_KV ? free_kv_ : free_act_).erase(c);
    owner_[c] = (uint8_t)new_owner;
    (new_owner == OWNER_KV ? free_kv_ : free_act_).insert(c);
  }
  return OK;
}

int PoolCore::set_act_busy(const int32_t* ids, int32_t n, int busy) {
  if (n < 0 || (n > 0 && !ids)) return fail(ERR_INVALID, "set_act_busy: bad count");
  ++stamp_now_;
  for (int32_t i = 0; i < n; i++) {
    int32_t c = ids[i];
    if (c < 0 || c >= g_.n_chunks) return fail(ERR_RANGE, "set_act_busy: chunk id outside the pool");
    if (owner_[c] != OWNER_ACT) return fail(ERR_OWNED, "set_act_busy: chunk is not on the activation side");
    if (busy) { if (state_[c] != CHUNK_FREE) return fail(ERR_OWNED, "set_act_busy: chunk is not free"); }
    else { if (state_[c] != CHUNK_BUSY) return fail(ERR_INVALID, "set_act_busy: chunk is not busy"); }
    if (stamp_[c] == stamp_now_) return fail(ERR_INVALID, "set_act_busy: chunk id given twice");
    stamp_[c] = stamp_now_;
  }
  for (int32_t i = 0; i < n; i++) {
    int32_t c = ids[i];
    if (busy) { state_[c] = CHUNK_BUSY; free_act_.erase(c); }
    else { state_[c] = CHUNK_FREE; free_act_.insert(c); }
  }
  return OK;
}

int PoolCore::append_check(const int32_t* ids, int32_t batch, const int32_t* n_new, std::vector<int32_t>& n_eff,
                           int64_t* total) {
  if (batch < 0 || (batch > 0 && !ids)) return fail(ERR_INVALID, "kv_append: bad batch");
  n_eff.resize(batch);
  const int64_t Tc = g_.tokens_per_chunk;
  int64_t sum = 0;
  ++stamp_now_;
  for (int32_t b = 0; b < batch; b++) {
    const TensorRec* t = tensor(ids[b]);
    if (!t) return fail(ERR_INVALID, "kv_append: bad tensor handle");
    if (stamp_[ids[b]] == stamp_now_) return fail(ERR_INVALID, "kv_append: tensor handle given twice");
    stamp_[ids[b]] = stamp_now_;
    int64_t n = n_new ? n_new[b] : 1;
    if (n < 0) return fail(ERR_INVALID, "kv_append: negative token count");
    if (t->len + n > t->max_tokens) return fail(ERR_RANGE, "kv_append: tensor would exceed max_tokens");
    if (n > 0) {
      const int32_t* r = row(ids[b]);
      for (int64_t s = t->len / Tc; s <= (t->len + n - 1) / Tc; s++) {
        if (r[s] == ENTRY_UNMAPPED) return fail(ERR_UNMAPPED, "kv_append: target slot has no chunk");
        if (r[s] <= -2) return fail(ERR_NOT_RESIDENT, "kv_append: target slot is in host memory");
      }
    }
    n_eff[b] = (int32_t)n;
    sum += n;
  }
  if (total) *total = sum;
  return OK;
}

void PoolCore::append_commit(const int32_t* ids, int32_t batch, const int32_t* n_eff) {
  for (int32_t b = 0; b < batch; b++) t_[ids[b]].len += n_eff[b];
}

int PoolCore::decode_check(const int32_t* ids, int32_t batch, int32_t extra) {
  if (batch < 0 || (batch > 0 && !ids)) return fail(ERR_INVALID, "decode_attention: bad batch");
  const int64_t Tc = g_.tokens_per_chunk;
  for (int32_t b = 0; b < batch; b++) {
    const TensorRec* t = tensor(ids[b]);
    if (!t) return fail(ERR_INVALID, "decode_attention: bad tensor handle");
    if (t->len + extra == 0) return fail(ERR_EMPTY, "decode_attention: tensor holds no token");
    const int32_t* r = row(ids[b]);
    for (int64_t s = 0; s <= (t->len + extra - 1) / Tc; s++) {
      if (r[s] == ENTRY_UNMAPPED) return fail(ERR_UNMAPPED, "decode_attention: slot has no chunk");
      if (r[s] <= -2) return fail(ERR_NOT_RESIDENT, "decode_attention: slot is in host memory");
    }
  }
  return OK;
}

int PoolCore::offload_plan(int32_t id, int32_t first, int32_t n, std::vector<Move>& moves) {
  moves.clear();
  const TensorRec* t = tensor(id);
  if (!t || n < 0) return fail(ERR_INVALID, "deflate_to_host: bad tensor handle or negative count");
  if (n == 0) return OK;
  if (first < 0 || (int64_t)first + n > t->n_slots) return fail(ERR_RANGE, "deflate_to_host: slot range outside the tensor");
  for (int32_t i = 0; i < n; i++) {
    int32_t e = row(id)[first + i];
    if (e == ENTRY_UNMAPPED) return fail(ERR_UNMAPPED, "deflate_to_host: slot has no chunk");
    if (e <= -2) return fail(ERR_NOT_RESIDENT, "deflate_to_host: slot is already in host memory");
  }
  if ((int32_t)free_host_.size() < n) return fail(ERR_HOST_FULL, "deflate_to_host: not enough free host slots");
  if (g_.n_host_slots - (int32_t)free_host_.size() + n > logical_host_)
    return fail(ERR_HOST_FULL, "deflate_to_host: the logical host buffer is full");
  auto it = free_host_.begin();
  for (int32_t i = 0; i < n; i++, ++it) moves.push_back(Move{first + i, row(id)[first + i], *it});
  return OK;
}

void PoolCore::offload_commit(int32_t id, const std::vector<Move>& moves) {
  for (const Move& m : moves) {
    free_host_.erase(m.host_slot);
    host_tensor_[m.host_slot] = id;
    host_slot_[m.host_slot] = m.slot;
    state_[m.chunk] = CHUNK_FREE;
    map_tensor_[m.chunk] = map_slot_[m.chunk] = -1;
    free_kv_.insert(m.chunk);
    set_entry(id, m.slot, entry_from_host_slot(m.host_slot));
  }
}

int PoolCore::fetch_plan(int32_t id, int32_t first, int32_t n, const int32_t* chunk_ids, std::vector<Move>& moves) {
  moves.clear();
  const TensorRec* t = tensor(id);
  if (!t || n < 0) return fail(ERR_INVALID, "inflate_from_host: bad tensor handle or negative count");
  if (n == 0) return OK;
  if (first < 0 || (int64_t)first + n > t->n_slots) return fail(ERR_RANGE, "inflate_from_host: slot range outside the tensor");
  for (int32_t i = 0; i < n; i++) {
    int32_t e = row(id)[first + i];
    if (e == ENTRY_UNMAPPED) return fail(ERR_UNMAPPED, "inflate_from_host: slot has no chunk");
    if (e >= 0) return fail(ERR_INVALID, "inflate_from_host: slot is already on the device");
  }
  std::vector<int32_t> pick;
  int rc = pick_chunks(n, chunk_ids, false, pick);
  if (rc) return rc;
  for (int32_t i = 0; i < n; i++)
    moves.push_back(Move{first + i, pick[i], host_slot_of_entry(row(id)[first + i])});
  return OK;
}

void PoolCore::fetch_commit(int32_t id, const std::vector<Move>& moves) {
  for (const Move& m : moves) {
    host_tensor_[m.host_slot] = host_slot_[m.host_slot] = -1;
    free_host_.insert(m.host_slot);
    take_chunk(m.chunk, id, m.slot);
  }
}

int PoolCore::self_check() const {
  std::vector<int32_t> seen(g_.n_chunks, 0), hseen(g_.n_host_slots, 0);
  for (int32_t id = 0; id < g_.max_tensors; id++) {
    const TensorRec& t = t_[id];
    const int32_t* r = row(id);
    for (int32_t s = 0; s < g_.max_slots; s++) {
      int32_t e = r[s];
      if (!t.used || s >= t.n_slots) { if (e != ENTRY_UNMAPPED) return 1; continue; }
      if (e >= 0) {
        if (e >= g_.n_chunks || seen[e]++) return 2;
        if (state_[e] != CHUNK_MAPPED || map_tensor_[e] != id || map_slot_[e] != s || owner_[e] != OWNER_KV) return 3;
      } else if (e <= -2) {
        int32_t hs = host_slot_of_entry(e);
        if (hs >= g_.n_host_slots || hseen[hs]++) return 4;
        if (host_tensor_[hs] != id || host_slot_[hs] != s) return 5;
      }
    }
  }
  for (int32_t c = 0; c < g_.n_chunks; c++) {
    bool in_kv = free_kv_.count(c) != 0, in_act = free_act_.count(c) != 0;
    if (state_[c] == CHUNK_FREE) {
      if (in_kv != (owner_[c] == OWNER_KV) || in_act != (owner_[c] == OWNER_ACT)) return 6;
    } else if (in_kv || in_act) return 7;
    if (state_[c] == CHUNK_MAPPED && !seen[c]) return 8;
    if (state_[c] == CHUNK_BUSY && owner_[c] != OWNER_ACT) return 9;
  }
  for (int32_t s = 0; s < g_.n_host_slots; s++) {
    bool is_free = free_host_.count(s) != 0;
    if (is_free != (host_tensor_[s] < 0)) return 10;
    if (!is_free && !hseen[s]) return 11;
  }
  // released tensors: empty, mapped only in a leading run, and listed under that run
  size_t n_released = 0;
  for (int32_t id = 0; id < g_.max_tensors; id++) {
    const TensorRec& t = t_[id];
    if (!t.used || !t.released) continue;
    n_released++;
    if (t.len != 0 || !released_.count({t.run, id})) return 12;
    for (int32_t s = 0; s < t.n_slots; s++)
      if ((s < t.run) != (row(id)[s] >= 0) || (s >= t.run && row(id)[s] != ENTRY_UNMAPPED)) return 13;
  }
  if (n_released != released_.size()) return 14;
  return 0;
}

}  // namespace ellm
