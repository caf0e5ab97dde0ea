// Sanitizer run of the two host state machines, side by side.
//
// Built by tests/test_sanitizers.py with -fsanitize=address,undefined from the library's host pool
// (pool_core.cpp, C++) and the oracle (ellm_oracle.c, C), which share no code. A seeded random walk
// feeds both the same calls, many of them illegal on purpose (bad handles, ranges past the table,
// duplicate chunk ids, negative counts), and after every call compares return codes, chunk tables,
// owner / state arrays and host-slot maps, and runs both sides' own consistency scans. Any memory
// error or undefined behaviour on either side aborts the run; any disagreement exits non-zero.
//
// usage: sanitize_walk <seed> <steps> [oracle decode threads]
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "pool_core.hpp"

extern "C" {
struct orc_pool;
orc_pool* orc_pool_create(int32_t n_chunks, uint32_t chunk_bytes, int32_t n_host, int Hq, int Hkv, int D,
                          int32_t max_tensors, int32_t max_slots, const uint8_t* initial_owner, int keep_twin);
void orc_pool_destroy(orc_pool* p);
int orc_tensor_create(orc_pool* p, int64_t max_tokens, int32_t* out);
int orc_tensor_destroy(orc_pool* p, int32_t id);
int orc_tensor_map_chunks(orc_pool* p, int32_t id, int32_t first, int32_t n, const int32_t* ids, uint32_t flags);
int orc_tensor_unmap_chunks(orc_pool* p, int32_t id, int32_t first, int32_t n);
int orc_pool_set_logical_host_slots(orc_pool* p, int32_t n);
int32_t orc_pool_get_logical_host_slots(orc_pool* p);
int orc_pool_slo_configure(orc_pool* p, double ttft_slo, double tpot_slo, double alpha, int32_t window, int32_t threshold);
int orc_pool_slo_observe(orc_pool* p, double ttft, double tpot, int32_t* logical_out);
int orc_tensor_release(orc_pool* p, int32_t id);
int orc_tensor_is_released(orc_pool* p, int32_t id);
int orc_tensor_acquire(orc_pool* p, int64_t need, int64_t max_tokens, uint32_t flags, int32_t* out);
int orc_kv_premap_next(orc_pool* p, const int32_t* ids, int32_t batch, uint32_t flags, int32_t* n_mapped);
int orc_kv_premap_ahead(orc_pool* p, const int32_t* ids, int32_t batch, int64_t tokens_ahead, uint32_t flags, int32_t* n_mapped);
int orc_pool_transfer(orc_pool* p, const int32_t* ids, int32_t n, int new_owner);
int orc_pool_set_act_busy(orc_pool* p, const int32_t* ids, int32_t n, int busy);
int orc_kv_append(orc_pool* p, const int32_t* ids, int32_t batch, const int32_t* n_new, const uint16_t* k_new,
                  const uint16_t* v_new);
int orc_chunk_offload(orc_pool* p, int32_t id, int32_t first, int32_t n);
int orc_chunk_fetch(orc_pool* p, int32_t id, int32_t first, int32_t n, const int32_t* ids);
int orc_tensor_get_table(orc_pool* p, int32_t id, int32_t* out, int32_t cap, int32_t* n_slots, int64_t* len);
void orc_pool_get_owner_state(orc_pool* p, uint8_t* owner, uint8_t* state, int32_t* mt, int32_t* ms);
void orc_pool_get_host_slots(orc_pool* p, int32_t* tensor, int32_t* slot);
int orc_check_invariants(orc_pool* p);
int orc_decode_attention(orc_pool* p, const int32_t* ids, int32_t batch, const uint16_t* q, double scale, int mode,
                         int n_threads, double* out);
}

namespace {

struct Rng {   // splitmix64
  uint64_t s;
  uint64_t next() {
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
  int32_t range(int32_t lo, int32_t hi) { return lo + (int32_t)(next() % (uint64_t)(hi - lo)); }   // [lo, hi)
  bool chance(int percent) { return (int)(next() % 100) < percent; }
};

[[noreturn]] void die(uint64_t seed, int step, const char* op, const char* what, long a = 0, long b = 0) {
  std::fprintf(stderr, "sanitize_walk: seed %llu step %d op %s: %s (%ld vs %ld)\n", (unsigned long long)seed, step, op,
               what, a, b);
  std::exit(1);
}

}  // namespace

int main(int argc, char** argv) {
  const uint64_t seed = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 1;
  const int steps = argc > 2 ? std::atoi(argv[2]) : 2000;
  const int threads = argc > 3 ? std::atoi(argv[3]) : 1;
  Rng rng{seed * 0x2545F4914F6CDD1Dull + 7};

  const int32_t n_chunks = 40 + (int32_t)(seed % 3) * 9, n_host = (seed % 2) ? 3 : 9;
  const int32_t Hq = 8, Hkv = 4, D = 64, Tc = (seed % 4 == 0) ? 13 : 16, max_tensors = 6, max_slots = 12;
  const uint32_t chunk_bytes = (uint32_t)Tc * 2 * Hkv * D * 2 + ((seed % 4 == 0) ? 100u : 0u);   // slack leaves Tc unchanged
  std::vector<uint8_t> owner0(n_chunks);
  for (auto& o : owner0) o = rng.chance(35) ? 1 : 0;

  ellm::Geometry g;
  g.n_chunks = n_chunks; g.n_host_slots = n_host; g.tokens_per_chunk = Tc; g.chunk_bytes = chunk_bytes;
  g.n_q_heads = Hq; g.n_kv_heads = Hkv; g.head_dim = D; g.group = Hq / Hkv;
  g.max_tensors = max_tensors; g.max_slots = max_slots; g.bytes_per_token = 2ull * Hkv * D * 2;
  ellm::PoolCore lib(g, owner0.data());
  orc_pool* orc = orc_pool_create(n_chunks, chunk_bytes, n_host, Hq, Hkv, D, max_tensors, max_slots, owner0.data(), 0);
  if (!orc) die(seed, -1, "create", "oracle refused the geometry");
  if (seed % 2) {
    int a = lib.slo_configure(100.0, 5.0, 2.0, 5, 3), b = orc_pool_slo_configure(orc, 100.0, 5.0, 2.0, 5, 3);
    if (a != b) die(seed, -1, "slo_configure", "return codes differ", a, b);
  }

  std::vector<uint16_t> kv((size_t)200 * Hkv * D, 0x3c00), q((size_t)4 * Hq * D, 0x3f80);
  std::vector<double> out((size_t)4 * Hq * D);
  std::vector<int32_t> tab(max_slots), ids, tids, nn;
  std::vector<uint8_t> oo(n_chunks), os(n_chunks);
  std::vector<int32_t> omt(n_chunks), oms(n_chunks), oht(n_host), ohs(n_host);
  long n_ok = 0;

  for (int step = 0; step < steps; step++) {
    std::vector<int32_t> alive;
    for (int32_t t = 0; t < max_tensors; t++) if (lib.tensor_any(t)) alive.push_back(t);
    int32_t tid, first, n;
    if (!alive.empty() && rng.chance(80)) {
      tid = alive[rng.range(0, (int32_t)alive.size())];
      int32_t ns = lib.tensor_any(tid)->n_slots;
      first = rng.range(0, ns);
      n = rng.range(0, std::min(5, ns - first) + 1);
    } else {
      tid = rng.range(-1, max_tensors + 1);
      first = rng.range(-1, 13);
      n = rng.range(-1, 6);
    }
    ids.assign(n > 0 ? n : 0, 0);
    for (auto& c : ids) c = rng.range(-1, n_chunks + 1);
    const int32_t* idp = n > 0 ? ids.data() : nullptr;
    const uint32_t fl = (uint32_t)rng.range(0, 2);
    auto pick_batch = [&](bool distinct_alive) {
      int32_t nb = rng.range(0, 4);
      tids.assign(nb, 0);
      for (auto& t : tids) t = rng.range(-1, max_tensors);
      if (distinct_alive && !alive.empty() && rng.chance(80)) {
        std::vector<int32_t> pool = alive;
        tids.clear();
        while ((int32_t)tids.size() < nb && !pool.empty()) {
          int32_t k = rng.range(0, (int32_t)pool.size());
          tids.push_back(pool[k]);
          pool.erase(pool.begin() + k);
        }
      }
    };

    int a = 0, b = 0;
    const char* op = "";
    switch (rng.range(0, 100) / 6) {
      case 0: {
        op = "create";
        int64_t mt = rng.range(0, Tc * 13);
        int32_t ia = -1, ib = -1;
        a = lib.tensor_create(mt, &ia); b = orc_tensor_create(orc, mt, &ib);
        if (a == 0 && b == 0 && ia != ib) die(seed, step, op, "handles differ", ia, ib);
      } break;
      case 1:
        if (rng.chance(50)) { op = "destroy"; a = lib.tensor_destroy(tid); b = orc_tensor_destroy(orc, tid); }
        else { op = "unmap"; a = lib.unmap_chunks(tid, first, n); b = orc_tensor_unmap_chunks(orc, tid, first, n); }
        break;
      case 2: case 3:
        op = "map"; a = lib.map_chunks(tid, first, n, nullptr, fl); b = orc_tensor_map_chunks(orc, tid, first, n, nullptr, fl);
        break;
      case 4:
        op = "map_ids"; a = lib.map_chunks(tid, first, n, idp, fl); b = orc_tensor_map_chunks(orc, tid, first, n, idp, fl);
        break;
      case 5: {
        op = "transfer";
        int own = rng.range(0, 3);
        a = lib.transfer(ids.data(), (int32_t)ids.size(), own); b = orc_pool_transfer(orc, ids.data(), (int32_t)ids.size(), own);
      } break;
      case 6: {
        op = "busy";
        int busy = rng.range(0, 2);
        a = lib.set_act_busy(ids.data(), (int32_t)ids.size(), busy);
        b = orc_pool_set_act_busy(orc, ids.data(), (int32_t)ids.size(), busy);
      } break;
      case 7: case 8: case 9: {
        op = "append";
        pick_batch(true);
        nn.assign(tids.size(), 0);
        for (auto& x : nn) x = rng.range(-1, 40);
        const int32_t* np_ = (!tids.empty() && rng.chance(30)) ? nullptr : nn.data();
        std::vector<int32_t> n_eff;
        int64_t total = 0;
        a = lib.append_check(tids.data(), (int32_t)tids.size(), np_, n_eff, &total);
        if (a == 0) lib.append_commit(tids.data(), (int32_t)tids.size(), n_eff.data());
        b = orc_kv_append(orc, tids.data(), (int32_t)tids.size(), np_, kv.data(), kv.data());
      } break;
      case 10: {
        op = "decode";
        pick_batch(rng.chance(50));
        a = lib.decode_check(tids.data(), (int32_t)tids.size(), 0);
        b = orc_decode_attention(orc, tids.data(), (int32_t)tids.size(), q.data(), 0.0, 0, threads, out.data());
      } break;
      case 11: {
        op = "offload";
        std::vector<ellm::Move> mv;
        a = lib.offload_plan(tid, first, n, mv);
        if (a == 0) lib.offload_commit(tid, mv);
        b = orc_chunk_offload(orc, tid, first, n);
      } break;
      case 12: {
        op = "fetch";
        const int32_t* use = rng.chance(35) ? idp : nullptr;
        std::vector<ellm::Move> mv;
        a = lib.fetch_plan(tid, first, n, use, mv);
        if (a == 0) lib.fetch_commit(tid, mv);
        b = orc_chunk_fetch(orc, tid, first, n, use);
      } break;
      case 13:
        op = "release"; a = lib.tensor_release(tid); b = orc_tensor_release(orc, tid);
        break;
      case 14: {
        op = "acquire";
        int64_t need = rng.range(-1, Tc * 8), mt = rng.range(0, Tc * 13);
        int32_t ia = -1, ib = -1;
        a = lib.tensor_acquire(need, mt, fl, &ia); b = orc_tensor_acquire(orc, need, mt, fl, &ib);
        if (a == 0 && b == 0 && ia != ib) die(seed, step, op, "handles differ", ia, ib);
      } break;
      case 15: {
        op = "premap";
        pick_batch(true);
        int32_t na = -1, nb2 = -1;
        if (rng.chance(50)) {
          a = lib.premap_next(tids.data(), (int32_t)tids.size(), fl, &na);
          b = orc_kv_premap_next(orc, tids.data(), (int32_t)tids.size(), fl, &nb2);
        } else {
          const int64_t ahead = rng.range(0, 40);
          a = lib.premap_ahead(tids.data(), (int32_t)tids.size(), ahead, fl, &na);
          b = orc_kv_premap_ahead(orc, tids.data(), (int32_t)tids.size(), ahead, fl, &nb2);
        }
        if (a == 0 && b == 0 && na != nb2) die(seed, step, op, "mapped counts differ", na, nb2);
      } break;
      default:
        if (rng.chance(30)) {
          op = "logical";
          int32_t nl = rng.range(-1, n_host + 2);
          a = lib.set_logical_host_slots(nl); b = orc_pool_set_logical_host_slots(orc, nl);
        } else {
          op = "slo";
          static const double T1[3] = {-1.0, 10.0, 200.0}, T2[3] = {-1.0, 1.0, 9.0};
          double t1 = T1[rng.range(0, 3)], t2 = T2[rng.range(0, 3)];
          int32_t la = -1, lb = -1;
          a = lib.slo_observe(t1, t2, &la); b = orc_pool_slo_observe(orc, t1, t2, &lb);
          if (a == 0 && b == 0 && la != lb) die(seed, step, op, "logical sizes differ", la, lb);
        }
        break;
    }
    if (a != b) die(seed, step, op, "return codes differ", a, b);
    n_ok += a == 0;

    // state comparison
    orc_pool_get_owner_state(orc, oo.data(), os.data(), omt.data(), oms.data());
    orc_pool_get_host_slots(orc, oht.data(), ohs.data());
    for (int32_t c = 0; c < n_chunks; c++) {
      if (oo[c] != lib.owner()[c]) die(seed, step, op, "owner differs at chunk", c);
      if (os[c] != lib.state()[c]) die(seed, step, op, "state differs at chunk", c);
      if (omt[c] != lib.map_tensor()[c] || oms[c] != lib.map_slot()[c]) die(seed, step, op, "chunk record differs", c);
    }
    for (int32_t s = 0; s < n_host; s++)
      if (oht[s] != lib.host_tensor()[s] || ohs[s] != lib.host_slot()[s]) die(seed, step, op, "host slot record differs", s);
    if (orc_pool_get_logical_host_slots(orc) != lib.logical_host_slots()) die(seed, step, op, "logical host size differs");
    for (int32_t t = 0; t < max_tensors; t++) {
      int32_t ns = 0;
      int64_t len = 0;
      int rc = orc_tensor_get_table(orc, t, tab.data(), max_slots, &ns, &len);
      const ellm::TensorRec* r = lib.tensor_any(t);
      if ((rc == 0) != (r != nullptr)) die(seed, step, op, "tensor liveness differs", t);
      if (!r) continue;
      if (ns != r->n_slots || len != r->len) die(seed, step, op, "tensor shape differs", t);
      if ((orc_tensor_is_released(orc, t) != 0) != r->released) die(seed, step, op, "released flag differs", t);
      for (int32_t s = 0; s < ns; s++)
        if (tab[s] != lib.row(t)[s]) die(seed, step, op, "table entry differs", t, s);
    }
    if (int bad = lib.self_check()) die(seed, step, op, "library self_check rule broken", bad);
    if (int bad = orc_check_invariants(orc)) die(seed, step, op, "oracle invariant broken", bad);
    if (step % 64 == 0) (void)lib.take_dirty();
  }
  orc_pool_destroy(orc);
  std::printf("sanitize_walk: seed %llu, %d calls (%ld accepted), states equal throughout\n", (unsigned long long)seed,
              steps, n_ok);
  return 0;
}
