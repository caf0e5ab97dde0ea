/*
 * ellm_oracle.c — TEST INFRASTRUCTURE ONLY. A plain, slow CPU model of chunk-backed virtual KV
 * tensors with fp64 softmax attention, written from the eLLM paper (arXiv 2506.15155) and from the
 * published C-ABI contract of the GPU library. It shares no code, header, table or helper with the
 * GPU path and must never be linked into or called from it. Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may use it.
 *
 * What it models, and the passage each part follows:
 *   pool        one set of fixed-size physical chunks shared by a KV side and an activation side,
 *               every chunk with exactly one owner at a time (Sec. 2.1, unified pool; Sec. 2.2.1
 *               step 3, ownership transfer)
 *   tensor      a per-request virtual range of max_tokens tokens split into chunk-sized slots,
 *               chunks bound to slots on demand (Sec. 2.1.1)
 *   map         bind free chunks to slots; when the KV side has none left and the caller allows
 *               it, borrow free activation-side chunks, which change owner (Sec. 2.2.1 steps 1,3,4)
 *   transfer    hand free chunks to the other side (Sec. 2.2.1 step 3 and its reverse, deflation)
 *   offload     move chunk contents to a CPU-memory slot and free the chunk (Sec. 2.2.2)
 *   fetch       bring them back into (generally different) free chunks (Sec. 2.2.2)
 *   append      write the new tokens of every request at its current length (Sec. 3.1: one token
 *               per sequence per decode iteration)
 *   attention   one query token per request attends over all cached tokens with standard softmax
 *               attention; grouped-query (q head h uses kv head h / G) or multi-head (Sec. 4.1
 *               "Models"). The paper gives no formula; this is the textbook definition
 *                   s_t = scale * <q_h, K_t>,  w_t = exp(s_t - max s) / sum exp(s - max s),
 *                   o_h = sum_t w_t V_t
 *               evaluated in fp64, two passes, no mask, no blocking or reordering.
 *
 * Readings where the paper is silent (chunk layout, which free chunk is taken, error order) are
 * the C-ABI contract's; they are restated at each function. Parity status: every function here
 * has a pin in tests/oracle_pins.py (the attention arithmetic against closed forms and a library
 * routine, the pool rules against brute force and hand-worked sequences); the allocator order,
 * the in-chunk layout and the tie and rounding rules of reuse and buffer scaling are conventions
 * of this build, "parity unpinned" by the paper, which is silent on them.
 *
 * Build: gcc -O2 -shared -fPIC -pthread ellm_oracle.c -o libellm_oracle.so -lm
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* return codes, numerically as published by the C-ABI contract */
enum {
  ORC_OK = 0, ORC_INVALID = -1, ORC_OOM = -2, ORC_OWNED = -3, ORC_UNMAPPED = -4,
  ORC_NOT_RESIDENT = -5, ORC_RANGE = -6, ORC_EMPTY = -7, ORC_HOST_FULL = -8
};
enum { OWNER_KV = 0, OWNER_ACT = 1 };
enum { ST_FREE = 0, ST_MAPPED = 1, ST_BUSY = 2 };
#define ENTRY_NONE (-1)

/* ORC_MUTANT != 0 builds a deliberately WRONG oracle (one planted mistake per number). Tests
 * build these on the CPU to show that the pins catch each mistake; nothing else may use them. */
#ifndef ORC_MUTANT
#define ORC_MUTANT 0
#endif

typedef struct {
  int used;
  int released;        /* mapped and available: waits for a new request (Sec. 2.1.2) */
  int64_t max_tokens, len;
  int32_t n_slots;
  int32_t* table;      /* n_slots entries                                     */
  uint16_t* twin_k;    /* dense twin [len][Hkv][D], straight from the appends */
  uint16_t* twin_v;
  int64_t twin_cap;
} orc_tensor;

typedef struct {
  int32_t n_chunks, n_host, tokens_per_chunk, max_tensors, max_slots;
  uint32_t chunk_bytes;
  int Hq, Hkv, D, G;
  int keep_twin;
  uint8_t *owner, *state;
  int32_t *map_tensor, *map_slot;      /* per chunk  */
  int32_t *host_tensor, *host_slot;    /* per host slot, -1 = free */
  uint8_t** chunk_img;                 /* per chunk byte image, allocated on first touch (zeros) */
  uint8_t** host_img;                  /* per host slot byte image */
  orc_tensor* t;
  /* logical host buffer and its SLO-aware scaling (Sec. 2.3.2) */
  int32_t logical_host;
  int slo_on;
  double slo_ttft, slo_tpot, slo_alpha;
  int32_t slo_window, slo_threshold;
  double* hist_ttft;                   /* every observation ever made, in order */
  double* hist_tpot;
  int64_t hist_n, hist_cap, hist_start;  /* hist_start: first observation after the last size change */
} orc_pool;

static double bf16_to_f64(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* byte offset of (kv head h, plane p, row r, dim 0) inside a chunk: head-major, then plane,
 * then token row, then dim */
static size_t row_offset(const orc_pool* p, int h, int plane, int r) {
#if ORC_MUTANT == 6
  return (((size_t)plane * (size_t)p->Hkv + (size_t)h) * (size_t)p->tokens_per_chunk + (size_t)r) * (size_t)p->D * 2;
#endif
  return (((size_t)h * 2 + (size_t)plane) * (size_t)p->tokens_per_chunk + (size_t)r) * (size_t)p->D * 2;
}

static uint8_t* chunk_bytes_of(orc_pool* p, int32_t c) {
  if (!p->chunk_img[c]) p->chunk_img[c] = (uint8_t*)calloc(p->chunk_bytes, 1);
  return p->chunk_img[c];
}
static uint8_t* host_bytes_of(orc_pool* p, int32_t s) {
  if (!p->host_img[s]) p->host_img[s] = (uint8_t*)calloc(p->chunk_bytes, 1);
  return p->host_img[s];
}

orc_pool* orc_pool_create(int32_t n_chunks, uint32_t chunk_bytes, int32_t n_host, int Hq, int Hkv, int D,
                          int32_t max_tensors, int32_t max_slots, const uint8_t* initial_owner,
                          int keep_twin) {
  if (n_chunks < 1 || Hkv < 1 || Hq % Hkv || (D != 64 && D != 128) || max_tensors < 1 || max_slots < 1)
    return NULL;
  uint64_t bpt = 2ull * (uint64_t)Hkv * (uint64_t)D * 2ull;
  if (chunk_bytes < bpt) return NULL;
  orc_pool* p = (orc_pool*)calloc(1, sizeof *p);
  p->n_chunks = n_chunks; p->n_host = n_host; p->chunk_bytes = chunk_bytes;
  p->tokens_per_chunk = (int32_t)(chunk_bytes / bpt);
  p->Hq = Hq; p->Hkv = Hkv; p->D = D; p->G = Hq / Hkv;
  p->max_tensors = max_tensors; p->max_slots = max_slots; p->keep_twin = keep_twin;
  p->logical_host = n_host;
  p->owner = (uint8_t*)calloc(n_chunks, 1);
  p->state = (uint8_t*)calloc(n_chunks, 1);
  p->map_tensor = (int32_t*)malloc(sizeof(int32_t) * n_chunks);
  p->map_slot = (int32_t*)malloc(sizeof(int32_t) * n_chunks);
  for (int32_t c = 0; c < n_chunks; c++) {
    p->owner[c] = initial_owner ? initial_owner[c] : OWNER_KV;
    p->map_tensor[c] = p->map_slot[c] = -1;
  }
  p->host_tensor = (int32_t*)malloc(sizeof(int32_t) * (n_host > 0 ? n_host : 1));
  p->host_slot = (int32_t*)malloc(sizeof(int32_t) * (n_host > 0 ? n_host : 1));
  for (int32_t s = 0; s < n_host; s++) p->host_tensor[s] = p->host_slot[s] = -1;
  p->chunk_img = (uint8_t**)calloc(n_chunks, sizeof(uint8_t*));
  p->host_img = (uint8_t**)calloc(n_host > 0 ? n_host : 1, sizeof(uint8_t*));
  p->t = (orc_tensor*)calloc(max_tensors, sizeof(orc_tensor));
  return p;
}

void orc_pool_destroy(orc_pool* p) {
  if (!p) return;
  for (int32_t c = 0; c < p->n_chunks; c++) free(p->chunk_img[c]);
  for (int32_t s = 0; s < p->n_host; s++) free(p->host_img[s]);
  for (int32_t i = 0; i < p->max_tensors; i++) {
    free(p->t[i].table); free(p->t[i].twin_k); free(p->t[i].twin_v);
  }
  free(p->hist_ttft); free(p->hist_tpot);
  free(p->chunk_img); free(p->host_img); free(p->t);
  free(p->owner); free(p->state); free(p->map_tensor); free(p->map_slot);
  free(p->host_tensor); free(p->host_slot);
  free(p);
}

int32_t orc_tokens_per_chunk(const orc_pool* p) { return p->tokens_per_chunk; }

/* any tensor record in use, released or not */
static orc_tensor* tensor_any(orc_pool* p, int32_t id) {
  if (id < 0 || id >= p->max_tensors || !p->t[id].used) return NULL;
  return &p->t[id];
}

/* a tensor that belongs to a request: released ones take no call but acquire / destroy / read-out */
static orc_tensor* tensor_of(orc_pool* p, int32_t id) {
  orc_tensor* t = tensor_any(p, id);
  return (t && !t->released) ? t : NULL;
}

/* reserve a virtual range; lowest unused handle */
int orc_tensor_create(orc_pool* p, int64_t max_tokens, int32_t* out) {
  if (max_tokens < 1) return ORC_INVALID;
  int64_t ns = (max_tokens + p->tokens_per_chunk - 1) / p->tokens_per_chunk;
  if (ns > p->max_slots) return ORC_RANGE;
  for (int32_t i = 0; i < p->max_tensors; i++) {
    if (p->t[i].used) continue;
    orc_tensor* t = &p->t[i];
    memset(t, 0, sizeof *t);
    t->used = 1; t->max_tokens = max_tokens; t->n_slots = (int32_t)ns;
    t->table = (int32_t*)malloc(sizeof(int32_t) * (size_t)ns);
    for (int64_t s = 0; s < ns; s++) t->table[s] = ENTRY_NONE;
    *out = i;
    return ORC_OK;
  }
  return ORC_OOM;
}

static void release_entry(orc_pool* p, int32_t e) {
  if (e >= 0) {
    p->state[e] = ST_FREE; p->map_tensor[e] = p->map_slot[e] = -1;
  } else if (e <= -2) {
    int32_t hs = -e - 2;
    p->host_tensor[hs] = p->host_slot[hs] = -1;
  }
}

int orc_tensor_destroy(orc_pool* p, int32_t id) {
  orc_tensor* t = tensor_any(p, id);
  if (!t) return ORC_INVALID;
  for (int32_t s = 0; s < t->n_slots; s++) release_entry(p, t->table[s]);
  free(t->table); free(t->twin_k); free(t->twin_v);
  memset(t, 0, sizeof *t);
  return ORC_OK;
}

/* check explicit chunk ids for map / fetch; inflate says whether activation-owned chunks are ok */
static int check_explicit(const orc_pool* p, const int32_t* ids, int32_t n, int inflate) {
  for (int32_t i = 0; i < n; i++) {
    int32_t c = ids[i];
    if (c < 0 || c >= p->n_chunks) return ORC_RANGE;
    if (p->state[c] != ST_FREE) return ORC_OWNED;
    for (int32_t j = 0; j < i; j++) if (ids[j] == c) return ORC_OWNED;
    if (p->owner[c] == OWNER_ACT && !inflate) return ORC_OWNED;
  }
  return ORC_OK;
}

/* pool-chosen chunks: lowest free KV-owned ids first; then, if allowed, lowest free ACT-owned */
static int choose_chunks(const orc_pool* p, int32_t n, int inflate, int32_t* out) {
  int32_t k = 0;
#if ORC_MUTANT == 8
  for (int32_t c = p->n_chunks - 1; c >= 0 && k < n; c--)
    if (p->owner[c] == OWNER_KV && p->state[c] == ST_FREE) out[k++] = c;
#endif
  for (int32_t c = 0; c < p->n_chunks && k < n; c++)
    if (p->owner[c] == OWNER_KV && p->state[c] == ST_FREE) out[k++] = c;
  if (k < n && inflate)
    for (int32_t c = 0; c < p->n_chunks && k < n; c++)
      if (p->owner[c] == OWNER_ACT && p->state[c] == ST_FREE) out[k++] = c;
  return k == n ? ORC_OK : ORC_OOM;
}

int orc_tensor_map_chunks(orc_pool* p, int32_t id, int32_t first, int32_t n, const int32_t* ids, uint32_t flags) {
  orc_tensor* t = tensor_of(p, id);
  if (!t || n < 0) return ORC_INVALID;
  if (n == 0) return ORC_OK;
  if (first < 0 || (int64_t)first + n > t->n_slots) return ORC_RANGE;
  for (int32_t i = 0; i < n; i++) if (t->table[first + i] != ENTRY_NONE) return ORC_INVALID;
  int inflate = (flags & 1u) != 0;
  int32_t* pick = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
  int rc;
  if (ids) { rc = check_explicit(p, ids, n, inflate); if (!rc) memcpy(pick, ids, sizeof(int32_t) * (size_t)n); }
  else rc = choose_chunks(p, n, inflate, pick);
  if (rc) { free(pick); return rc; }
  for (int32_t i = 0; i < n; i++) {
    int32_t c = pick[i];
    p->owner[c] = OWNER_KV; p->state[c] = ST_MAPPED;
    p->map_tensor[c] = id; p->map_slot[c] = first + i;
    t->table[first + i] = c;
  }
  free(pick);
  return ORC_OK;
}

int orc_tensor_unmap_chunks(orc_pool* p, int32_t id, int32_t first, int32_t n) {
  orc_tensor* t = tensor_of(p, id);
  if (!t || n < 0) return ORC_INVALID;
  if (n == 0) return ORC_OK;
  if (first < 0 || (int64_t)first + n > t->n_slots) return ORC_RANGE;
  int64_t live = (t->len + p->tokens_per_chunk - 1) / p->tokens_per_chunk;
#if ORC_MUTANT == 14
  live = t->len / p->tokens_per_chunk;                                       /* partly filled slot not counted */
#endif
  if (first < live) return ORC_INVALID;
  for (int32_t i = 0; i < n; i++) if (t->table[first + i] == ENTRY_NONE) return ORC_UNMAPPED;
  for (int32_t i = 0; i < n; i++) {
#if ORC_MUTANT != 15
    release_entry(p, t->table[first + i]);
#endif
    t->table[first + i] = ENTRY_NONE;
  }
  return ORC_OK;
}

/* ---- logical host buffer (Sec. 2.3.2 "SLO-aware Buffer Scaling Policy") ------------------------ */

int orc_pool_set_logical_host_slots(orc_pool* p, int32_t n) {
  if (n < 0 || n > p->n_host) return ORC_RANGE;
  p->logical_host = n;
  return ORC_OK;
}

int32_t orc_pool_get_logical_host_slots(orc_pool* p) { return p->logical_host; }

int orc_pool_slo_configure(orc_pool* p, double ttft_slo, double tpot_slo, double alpha, int32_t window, int32_t threshold) {
  if (!(ttft_slo > 0) || !(tpot_slo > 0) || !(alpha > 1) || window < 1 || threshold < 1 || threshold > window)
    return ORC_INVALID;
  p->slo_on = 1;
  p->slo_ttft = ttft_slo; p->slo_tpot = tpot_slo; p->slo_alpha = alpha;
  p->slo_window = window; p->slo_threshold = threshold;
  p->hist_n = p->hist_start = 0;
  return ORC_OK;
}

/* The whole history is kept and recounted at every call: of the observations made since the last
 * change of size, the newest `window` are looked at; `threshold` of them over the time-per-output-
 * token SLO shrink the buffer (that case first), else `threshold` over the time-to-first-token SLO
 * grow it. A negative latency is "none measured" and never a violation. */
int orc_pool_slo_observe(orc_pool* p, double ttft, double tpot, int32_t* logical_out) {
  if (!p->slo_on || ttft != ttft || tpot != tpot) return ORC_INVALID;
  if (p->hist_n == p->hist_cap) {
    p->hist_cap = p->hist_cap ? 2 * p->hist_cap : 64;
    p->hist_ttft = (double*)realloc(p->hist_ttft, sizeof(double) * (size_t)p->hist_cap);
    p->hist_tpot = (double*)realloc(p->hist_tpot, sizeof(double) * (size_t)p->hist_cap);
  }
  p->hist_ttft[p->hist_n] = ttft;
  p->hist_tpot[p->hist_n] = tpot;
  p->hist_n++;
  int64_t from = p->hist_n - p->slo_window;
#if ORC_MUTANT == 13
  from = p->hist_start;                                                    /* window never slides */
#endif
  if (from < p->hist_start) from = p->hist_start;
  int over_ttft = 0, over_tpot = 0;
  for (int64_t i = from; i < p->hist_n; i++) {
    if (p->hist_ttft[i] > p->slo_ttft) over_ttft++;
    if (p->hist_tpot[i] > p->slo_tpot) over_tpot++;
  }
  if (over_tpot >= p->slo_threshold) {
    p->logical_host = (int32_t)floor((double)p->logical_host / p->slo_alpha);
    p->hist_start = p->hist_n;
  } else if (over_ttft >= p->slo_threshold) {
    double base = p->logical_host < 1 ? 1.0 : (double)p->logical_host;
    double grown = ceil(base * p->slo_alpha);
    p->logical_host = grown > (double)p->n_host ? p->n_host : (int32_t)grown;
    p->hist_start = p->hist_n;
  }
  if (logical_out) *logical_out = p->logical_host;
  return ORC_OK;
}

/* ---- request turnover (Sec. 2.1.2 "Memory Management Strategy", Sec. 3.1 pre-mapping) -------- */

/* tokens a tensor can take without any new mapping: its leading run of device-resident slots */
static int32_t mapped_run(const orc_tensor* t) {
  int32_t run = 0;
  while (run < t->n_slots && t->table[run] >= 0) run++;
  return run;
}

/* The request is over: the tensor keeps its leading mapped slots and becomes available. What lies
 * behind the first slot without a device chunk (host copies, stray mappings) is given back. */
int orc_tensor_release(orc_pool* p, int32_t id) {
  orc_tensor* t = tensor_of(p, id);
  if (!t) return ORC_INVALID;
  int32_t keep = mapped_run(t);
#if ORC_MUTANT == 12
  keep = 0;                                                                /* nothing retained */
#endif
  for (int32_t s = keep; s < t->n_slots; s++) {
    release_entry(p, t->table[s]);
    t->table[s] = ENTRY_NONE;
  }
  t->len = 0;
  t->released = 1;
  return ORC_OK;
}

int orc_tensor_is_released(orc_pool* p, int32_t id) {
  orc_tensor* t = tensor_any(p, id);
  return t ? t->released : ORC_INVALID;
}

/* A new request that needs room for `need` tokens now and `max_tokens` at most. Best fit: of the
 * available tensors whose virtual range suffices and whose mapped size is at least `need`, the one
 * with the smallest mapped size (the paper's arg min); equal sizes: the lowest handle. Without
 * one, a fresh tensor (lowest unused handle) is mapped on demand: free KV chunks in ascending
 * order, then chunks taken back from available tensors (smallest mapped size first, equal sizes
 * lowest handle first, from its last mapped slot downwards), then, if allowed, free activation
 * chunks in ascending order. All or nothing. */
int orc_tensor_acquire(orc_pool* p, int64_t need, int64_t max_tokens, uint32_t flags, int32_t* out) {
  const int64_t Tc = p->tokens_per_chunk;
  if (need < 0 || max_tokens < 1 || need > max_tokens) return ORC_INVALID;
  if ((max_tokens + Tc - 1) / Tc > p->max_slots) return ORC_RANGE;
  int32_t best = -1;
  int64_t best_size = 0;
  for (int32_t i = 0; i < p->max_tensors; i++) {
    orc_tensor* t = &p->t[i];
    if (!t->used || !t->released || t->max_tokens < max_tokens) continue;
    int64_t size = (int64_t)mapped_run(t) * Tc;
    if (size < need) continue;
#if ORC_MUTANT == 11
    if (best < 0 || size > best_size) { best = i; best_size = size; }   /* worst fit */
    continue;
#endif
    if (best < 0 || size < best_size) { best = i; best_size = size; }
  }
  if (best >= 0) {
    p->t[best].released = 0;
    p->t[best].len = 0;
    *out = best;
    return ORC_OK;
  }
  /* on-demand mapping */
  int32_t n = (int32_t)((need + Tc - 1) / Tc), k = 0, handle = -1;
  for (int32_t i = 0; i < p->max_tensors && handle < 0; i++) if (!p->t[i].used) handle = i;
  if (handle < 0) return ORC_OOM;
  int32_t* pick = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n + 1));
  int32_t* taken = (int32_t*)calloc((size_t)p->max_tensors, sizeof(int32_t));   /* slots taken back per tensor */
  for (int32_t c = 0; c < p->n_chunks && k < n; c++)
    if (p->owner[c] == OWNER_KV && p->state[c] == ST_FREE) pick[k++] = c;
  while (k < n) {
    int32_t donor = -1, donor_left = 0;
    for (int32_t i = 0; i < p->max_tensors; i++) {
      orc_tensor* t = &p->t[i];
      if (!t->used || !t->released) continue;
      int32_t left = mapped_run(t) - taken[i];
      if (left > 0 && (donor < 0 || left < donor_left)) { donor = i; donor_left = left; }
    }
    if (donor < 0) break;
    while (k < n && donor_left > 0) {
      pick[k++] = p->t[donor].table[donor_left - 1];
      donor_left--;
      taken[donor]++;
    }
  }
  if (k < n && (flags & 1u))
    for (int32_t c = 0; c < p->n_chunks && k < n; c++)
      if (p->owner[c] == OWNER_ACT && p->state[c] == ST_FREE) pick[k++] = c;
  if (k < n) { free(pick); free(taken); return ORC_OOM; }
  for (int32_t i = 0; i < p->max_tensors; i++) {
    if (!taken[i]) continue;
    orc_tensor* t = &p->t[i];
    int32_t run = mapped_run(t);
    for (int32_t s = run - taken[i]; s < run; s++) { release_entry(p, t->table[s]); t->table[s] = ENTRY_NONE; }
  }
  free(taken);
  int32_t id = -1;
  int rc = orc_tensor_create(p, max_tokens, &id);
  if (rc || id != handle) { free(pick); return rc ? rc : ORC_INVALID; }
  orc_tensor* t = &p->t[id];
  for (int32_t i = 0; i < n; i++) {
    int32_t c = pick[i];
    p->owner[c] = OWNER_KV; p->state[c] = ST_MAPPED;
    p->map_tensor[c] = id; p->map_slot[c] = i;
    t->table[i] = c;
  }
  free(pick);
  *out = id;
  return ORC_OK;
}

/* Speculative pre-mapping (Sec. 3.1): every sequence is assumed to produce one more token, so a
 * request whose next token opens a slot that has no chunk gets one mapped now (pool-chosen, as in
 * map). All or nothing; *n_mapped counts the chunks. */
int orc_kv_premap_next(orc_pool* p, const int32_t* ids, int32_t batch, uint32_t flags, int32_t* n_mapped) {
  if (batch < 0) return ORC_INVALID;
  const int64_t Tc = p->tokens_per_chunk;
  int32_t need = 0;
  for (int32_t b = 0; b < batch; b++) {
    orc_tensor* t = tensor_of(p, ids[b]);
    if (!t) return ORC_INVALID;
    for (int32_t j = 0; j < b; j++) if (ids[j] == ids[b]) return ORC_INVALID;
    if (t->len < t->max_tokens && t->len % Tc == 0 && t->table[t->len / Tc] == ENTRY_NONE) need++;
  }
  int32_t* pick = (int32_t*)malloc(sizeof(int32_t) * (size_t)(need + 1));
  int rc = choose_chunks(p, need, (flags & 1u) != 0, pick);
  if (rc) { free(pick); return rc; }
  int32_t k = 0;
  for (int32_t b = 0; b < batch; b++) {
    orc_tensor* t = tensor_of(p, ids[b]);
    if (!(t->len < t->max_tokens && t->len % Tc == 0 && t->table[t->len / Tc] == ENTRY_NONE)) continue;
    int32_t c = pick[k++], s = (int32_t)(t->len / Tc);
    p->owner[c] = OWNER_KV; p->state[c] = ST_MAPPED;
    p->map_tensor[c] = ids[b]; p->map_slot[c] = s;
    t->table[s] = c;
  }
  free(pick);
  if (n_mapped) *n_mapped = need;
  return ORC_OK;
}

/* The same idea with a longer view (Sec. 3.1 maps "ahead of time"; how far is the caller's choice):
 * every listed sequence is assumed to produce tokens_ahead more tokens (as far as its max_tokens
 * allows), and every slot those tokens would be written to that has no chunk gets one now, in batch
 * order and, within a tensor, in slot order. Slots that hold a host copy are left alone. All or
 * nothing; *n_mapped counts the chunks. With tokens_ahead == 1 this is orc_kv_premap_next. */
int orc_kv_premap_ahead(orc_pool* p, const int32_t* ids, int32_t batch, int64_t tokens_ahead, uint32_t flags,
                        int32_t* n_mapped) {
  if (batch < 0 || tokens_ahead < 1) return ORC_INVALID;
  const int64_t Tc = p->tokens_per_chunk;
  int32_t need = 0;
  for (int32_t b = 0; b < batch; b++) {
    orc_tensor* t = tensor_of(p, ids[b]);
    if (!t) return ORC_INVALID;
    for (int32_t j = 0; j < b; j++) if (ids[j] == ids[b]) return ORC_INVALID;
    int64_t until = t->len + tokens_ahead;            /* tokens len .. until - 1 are the ones to come */
    if (until > t->max_tokens) until = t->max_tokens;
#if ORC_MUTANT == 17
    for (int64_t s = t->len / Tc; s <= until / Tc && s < t->n_slots; s++)
#else
    for (int64_t s = t->len / Tc; s * Tc < until; s++)
#endif
      if (t->table[s] == ENTRY_NONE) need++;
  }
  int32_t* pick = (int32_t*)malloc(sizeof(int32_t) * (size_t)(need + 1));
  int rc = choose_chunks(p, need, (flags & 1u) != 0, pick);
  if (rc) { free(pick); return rc; }
  int32_t k = 0;
  for (int32_t b = 0; b < batch; b++) {
    orc_tensor* t = tensor_of(p, ids[b]);
    int64_t until = t->len + tokens_ahead;
    if (until > t->max_tokens) until = t->max_tokens;
#if ORC_MUTANT == 17
    for (int64_t s = t->len / Tc; s <= until / Tc && s < t->n_slots; s++) {
#else
    for (int64_t s = t->len / Tc; s * Tc < until; s++) {
#endif
      if (t->table[s] != ENTRY_NONE) continue;
      int32_t c = pick[k++];
      p->owner[c] = OWNER_KV; p->state[c] = ST_MAPPED;
      p->map_tensor[c] = ids[b]; p->map_slot[c] = (int32_t)s;
      t->table[s] = c;
    }
  }
  free(pick);
  if (n_mapped) *n_mapped = need;
  return ORC_OK;
}

int orc_pool_transfer(orc_pool* p, const int32_t* ids, int32_t n, int new_owner) {
  if (n < 0 || (new_owner != OWNER_KV && new_owner != OWNER_ACT)) return ORC_INVALID;
  for (int32_t i = 0; i < n; i++) {
    int32_t c = ids[i];
    if (c < 0 || c >= p->n_chunks) return ORC_RANGE;
    if (p->state[c] != ST_FREE) return ORC_OWNED;
    for (int32_t j = 0; j < i; j++) if (ids[j] == c) return ORC_INVALID;
  }
  for (int32_t i = 0; i < n; i++) p->owner[ids[i]] = (uint8_t)new_owner;
  return ORC_OK;
}

int orc_pool_set_act_busy(orc_pool* p, const int32_t* ids, int32_t n, int busy) {
  if (n < 0) return ORC_INVALID;
  for (int32_t i = 0; i < n; i++) {
    int32_t c = ids[i];
    if (c < 0 || c >= p->n_chunks) return ORC_RANGE;
    if (p->owner[c] != OWNER_ACT) return ORC_OWNED;
    if (busy) { if (p->state[c] != ST_FREE) return ORC_OWNED; }
    else { if (p->state[c] != ST_BUSY) return ORC_INVALID; }
    for (int32_t j = 0; j < i; j++) if (ids[j] == c) return ORC_INVALID;
  }
#if ORC_MUTANT == 16
  if (!busy) return ORC_OK;                                                  /* chunks never given back */
#endif
  for (int32_t i = 0; i < n; i++) p->state[ids[i]] = busy ? ST_BUSY : ST_FREE;
  return ORC_OK;
}

/* append: k_new / v_new are [sum n_new][Hkv][D] bf16 bit patterns on the host */
int orc_kv_append(orc_pool* p, const int32_t* ids, int32_t batch, const int32_t* n_new,
                  const uint16_t* k_new, const uint16_t* v_new) {
  if (batch < 0) return ORC_INVALID;
  const int Tc = p->tokens_per_chunk;
  int64_t total = 0;
  for (int32_t b = 0; b < batch; b++) {
    orc_tensor* t = tensor_of(p, ids[b]);
    if (!t) return ORC_INVALID;
    for (int32_t j = 0; j < b; j++) if (ids[j] == ids[b]) return ORC_INVALID;
    int64_t n = n_new ? n_new[b] : 1;
    if (n < 0) return ORC_INVALID;
    if (t->len + n > t->max_tokens) return ORC_RANGE;
    if (n > 0) {
      for (int64_t s = t->len / Tc; s <= (t->len + n - 1) / Tc; s++) {
        if (t->table[s] == ENTRY_NONE) return ORC_UNMAPPED;
        if (t->table[s] <= -2) return ORC_NOT_RESIDENT;
      }
    }
    total += n;
  }
  if (total > 0 && (!k_new || !v_new)) return ORC_INVALID;
  const size_t row = (size_t)p->D * 2, tok = (size_t)p->Hkv * (size_t)p->D;
  int64_t src = 0;
  for (int32_t b = 0; b < batch; b++) {
    orc_tensor* t = &p->t[ids[b]];
    int64_t n = n_new ? n_new[b] : 1;
    if (p->keep_twin && n > 0) {
      if (t->len + n > t->twin_cap) {
        int64_t cap = t->twin_cap ? t->twin_cap : 64;
        while (cap < t->len + n) cap *= 2;
        t->twin_k = (uint16_t*)realloc(t->twin_k, (size_t)cap * tok * 2);
        t->twin_v = (uint16_t*)realloc(t->twin_v, (size_t)cap * tok * 2);
        t->twin_cap = cap;
      }
      memcpy(t->twin_k + (size_t)t->len * tok, k_new + (size_t)src * tok, (size_t)n * tok * 2);
      memcpy(t->twin_v + (size_t)t->len * tok, v_new + (size_t)src * tok, (size_t)n * tok * 2);
    }
    for (int64_t i = 0; i < n; i++, src++) {
      int64_t pos = t->len + i;
      uint8_t* img = chunk_bytes_of(p, t->table[pos / Tc]);
      int r = (int)(pos % Tc);
      for (int h = 0; h < p->Hkv; h++) {
        memcpy(img + row_offset(p, h, 0, r), k_new + (size_t)src * tok + (size_t)h * p->D, row);
        memcpy(img + row_offset(p, h, 1, r), v_new + (size_t)src * tok + (size_t)h * p->D, row);
      }
    }
    t->len += n;
  }
  return ORC_OK;
}

int orc_chunk_offload(orc_pool* p, int32_t id, int32_t first, int32_t n) {
  orc_tensor* t = tensor_of(p, id);
  if (!t || n < 0) return ORC_INVALID;
  if (n == 0) return ORC_OK;
  if (first < 0 || (int64_t)first + n > t->n_slots) return ORC_RANGE;
  for (int32_t i = 0; i < n; i++) {
    if (t->table[first + i] == ENTRY_NONE) return ORC_UNMAPPED;
    if (t->table[first + i] <= -2) return ORC_NOT_RESIDENT;
  }
  int32_t free_slots = 0;
  for (int32_t s = 0; s < p->n_host; s++) if (p->host_tensor[s] < 0) free_slots++;
  if (free_slots < n) return ORC_HOST_FULL;
  if (p->n_host - free_slots + n > p->logical_host) return ORC_HOST_FULL;   /* Sec. 2.3.2: logical buffer */
  int32_t hs = 0;
  for (int32_t i = 0; i < n; i++) {
    while (p->host_tensor[hs] >= 0) hs++;
    int32_t c = t->table[first + i];
    memcpy(host_bytes_of(p, hs), chunk_bytes_of(p, c), p->chunk_bytes);
    p->host_tensor[hs] = id; p->host_slot[hs] = first + i;
#if ORC_MUTANT != 9
    p->state[c] = ST_FREE; p->map_tensor[c] = p->map_slot[c] = -1;
#endif
    t->table[first + i] = -hs - 2;
  }
  return ORC_OK;
}

int orc_chunk_fetch(orc_pool* p, int32_t id, int32_t first, int32_t n, const int32_t* ids) {
  orc_tensor* t = tensor_of(p, id);
  if (!t || n < 0) return ORC_INVALID;
  if (n == 0) return ORC_OK;
  if (first < 0 || (int64_t)first + n > t->n_slots) return ORC_RANGE;
  for (int32_t i = 0; i < n; i++) {
    if (t->table[first + i] == ENTRY_NONE) return ORC_UNMAPPED;
    if (t->table[first + i] >= 0) return ORC_INVALID;
  }
  int32_t* pick = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
  int rc;
  if (ids) { rc = check_explicit(p, ids, n, 0); if (!rc) memcpy(pick, ids, sizeof(int32_t) * (size_t)n); }
  else rc = choose_chunks(p, n, 0, pick);
  if (rc) { free(pick); return rc; }
  for (int32_t i = 0; i < n; i++) {
    int32_t c = pick[i], hs = -t->table[first + i] - 2;
#if ORC_MUTANT != 10
    memcpy(chunk_bytes_of(p, c), host_bytes_of(p, hs), p->chunk_bytes);
#endif
    p->host_tensor[hs] = p->host_slot[hs] = -1;
    p->state[c] = ST_MAPPED; p->map_tensor[c] = id; p->map_slot[c] = first + i;
    t->table[first + i] = c;
  }
  free(pick);
  return ORC_OK;
}

/* ---- state read-out -------------------------------------------------------------------------- */
int orc_tensor_get_table(orc_pool* p, int32_t id, int32_t* out, int32_t cap, int32_t* n_slots, int64_t* len) {
  orc_tensor* t = tensor_any(p, id);
  if (!t) return ORC_INVALID;
  int32_t n = t->n_slots < cap ? t->n_slots : cap;
  if (out && n > 0) memcpy(out, t->table, sizeof(int32_t) * (size_t)n);
  if (n_slots) *n_slots = t->n_slots;
  if (len) *len = t->len;
  return ORC_OK;
}
void orc_pool_get_owner_state(orc_pool* p, uint8_t* owner, uint8_t* state, int32_t* mt, int32_t* ms) {
  if (owner) memcpy(owner, p->owner, p->n_chunks);
  if (state) memcpy(state, p->state, p->n_chunks);
  if (mt) memcpy(mt, p->map_tensor, sizeof(int32_t) * p->n_chunks);
  if (ms) memcpy(ms, p->map_slot, sizeof(int32_t) * p->n_chunks);
}
void orc_pool_get_host_slots(orc_pool* p, int32_t* tensor, int32_t* slot) {
  if (tensor) memcpy(tensor, p->host_tensor, sizeof(int32_t) * p->n_host);
  if (slot) memcpy(slot, p->host_slot, sizeof(int32_t) * p->n_host);
}
int orc_chunk_set_bytes(orc_pool* p, int32_t c, const uint8_t* src) {
  if (c < 0 || c >= p->n_chunks) return ORC_RANGE;
  memcpy(chunk_bytes_of(p, c), src, p->chunk_bytes);
  return ORC_OK;
}
int orc_chunk_get_bytes(orc_pool* p, int32_t c, uint8_t* dst) {
  if (c < 0 || c >= p->n_chunks) return ORC_RANGE;
  memcpy(dst, chunk_bytes_of(p, c), p->chunk_bytes);
  return ORC_OK;
}
int orc_host_slot_get_bytes(orc_pool* p, int32_t s, uint8_t* dst) {
  if (s < 0 || s >= p->n_host) return ORC_RANGE;
  memcpy(dst, host_bytes_of(p, s), p->chunk_bytes);
  return ORC_OK;
}

/* Structural invariants: every chunk id appears in at most one (tensor, slot); the chunk records
 * and the tables agree in both directions; host slots likewise. Returns 0 when all hold, else a
 * positive number naming the first rule broken. */
int orc_check_invariants(orc_pool* p) {
  int32_t* seen = (int32_t*)calloc(p->n_chunks, sizeof(int32_t));
  int32_t* hseen = (int32_t*)calloc(p->n_host > 0 ? p->n_host : 1, sizeof(int32_t));
  int bad = 0;
  for (int32_t i = 0; i < p->max_tensors && !bad; i++) {
    orc_tensor* t = &p->t[i];
    if (!t->used) continue;
    for (int32_t s = 0; s < t->n_slots && !bad; s++) {
      int32_t e = t->table[s];
      if (e >= 0) {
        if (e >= p->n_chunks) bad = 1;
        else if (seen[e]++) bad = 2;                                   /* chunk in two slots */
        else if (p->state[e] != ST_MAPPED || p->map_tensor[e] != i || p->map_slot[e] != s) bad = 3;
        else if (p->owner[e] != OWNER_KV) bad = 4;                     /* mapped chunk not KV-owned */
      } else if (e <= -2) {
        int32_t hs = -e - 2;
        if (hs >= p->n_host) bad = 5;
        else if (hseen[hs]++) bad = 6;
        else if (p->host_tensor[hs] != i || p->host_slot[hs] != s) bad = 7;
      }
    }
  }
  for (int32_t c = 0; c < p->n_chunks && !bad; c++) {
    if (p->state[c] == ST_MAPPED && !seen[c]) bad = 8;                 /* mapped chunk nobody names */
    if (p->state[c] == ST_BUSY && p->owner[c] != OWNER_ACT) bad = 9;
    if (p->state[c] != ST_MAPPED && (p->map_tensor[c] != -1 || p->map_slot[c] != -1)) bad = 10;
  }
  for (int32_t s = 0; s < p->n_host && !bad; s++)
    if (p->host_tensor[s] >= 0 && !hseen[s]) bad = 11;
  free(seen); free(hseen);
  return bad;
}

/* ---- attention -------------------------------------------------------------------------------- */
enum { MODE_CHUNKED = 0, MODE_TWIN = 1, MODE_ONLINE = 2 };

/* pointer to the D bf16 values of (token pos, kv head g, plane) of tensor t, read through the
 * table and the chunk image (MODE_CHUNKED / MODE_ONLINE) or from the dense twin (MODE_TWIN) */
static const uint16_t* kv_row(orc_pool* p, const orc_tensor* t, int64_t pos, int g, int plane, int mode) {
#if ORC_MUTANT == 3
  plane = 1 - plane;
#endif
  if (mode == MODE_TWIN)
    return (plane ? t->twin_v : t->twin_k) + ((size_t)pos * p->Hkv + (size_t)g) * (size_t)p->D;
  int32_t c = t->table[pos / p->tokens_per_chunk];
  return (const uint16_t*)(chunk_bytes_of(p, c) + row_offset(p, g, plane, (int)(pos % p->tokens_per_chunk)));
}

/* one (request, q head): the definition, two passes, fp64. w_out (len doubles) may be NULL. */
static void attend_two_pass(orc_pool* p, const orc_tensor* t, const uint16_t* q, int h, double scale,
                            int mode, double* out, double* w_out) {
#if ORC_MUTANT == 1
  const int D = p->D, g = h % p->Hkv;
#else
  const int D = p->D, g = h / p->G;
#endif
#if ORC_MUTANT == 2
  scale = 1.0;
#endif
  const int64_t L = t->len;
  double* s = (double*)malloc(sizeof(double) * (size_t)L);
  double smax = -INFINITY;
  for (int64_t pos = 0; pos < L; pos++) {
    const uint16_t* k = kv_row(p, t, pos, g, 0, mode);
    double dot = 0.0;
#if ORC_MUTANT == 7
    for (int d = 0; d < D - 1; d++) dot += bf16_to_f64(q[d]) * bf16_to_f64(k[d]);
#else
    for (int d = 0; d < D; d++) dot += bf16_to_f64(q[d]) * bf16_to_f64(k[d]);
#endif
    s[pos] = scale * dot;
    if (s[pos] > smax) smax = s[pos];
  }
  double denom = 0.0;
  for (int64_t pos = 0; pos < L; pos++) { s[pos] = exp(s[pos] - smax); denom += s[pos]; }
  for (int d = 0; d < D; d++) out[d] = 0.0;
  for (int64_t pos = 0; pos < L; pos++) {
#if ORC_MUTANT == 4
    double w = s[pos];
#elif ORC_MUTANT == 5
    double w = s[pos] / denom; if (pos == L - 1 && L > 1) w = 0.0;   /* newest token ignored */
#else
    double w = s[pos] / denom;
#endif
    if (w_out) w_out[pos] = w;
    const uint16_t* v = kv_row(p, t, pos, g, 1, mode);
    for (int d = 0; d < D; d++) out[d] += w * bf16_to_f64(v[d]);
  }
  free(s);
}

/* same result by another route: softmax statistics (max, sum, weighted V) computed per chunk-sized
 * slot and merged slot by slot with the usual rescaling. Used only to check that splitting the
 * sequence and merging partial softmaxes is exact up to rounding. */
static void attend_online(orc_pool* p, const orc_tensor* t, const uint16_t* q, int h, double scale, double* out) {
  const int D = p->D, g = h / p->G, Tc = p->tokens_per_chunk;
  double m = -INFINITY, l = 0.0;
  double* acc = (double*)calloc((size_t)D, sizeof(double));
  double* pacc = (double*)malloc(sizeof(double) * (size_t)D);
  for (int64_t t0 = 0; t0 < t->len; t0 += Tc) {
    int64_t t1 = t0 + Tc < t->len ? t0 + Tc : t->len;
    double pm = -INFINITY, pl = 0.0;
    double sc[t1 - t0];
    for (int64_t pos = t0; pos < t1; pos++) {
      const uint16_t* k = kv_row(p, t, pos, g, 0, MODE_CHUNKED);
      double dot = 0.0;
      for (int d = 0; d < D; d++) dot += bf16_to_f64(q[d]) * bf16_to_f64(k[d]);
      sc[pos - t0] = scale * dot;
      if (sc[pos - t0] > pm) pm = sc[pos - t0];
    }
    for (int d = 0; d < D; d++) pacc[d] = 0.0;
    for (int64_t pos = t0; pos < t1; pos++) {
      double e = exp(sc[pos - t0] - pm);
      pl += e;
      const uint16_t* v = kv_row(p, t, pos, g, 1, MODE_CHUNKED);
      for (int d = 0; d < D; d++) pacc[d] += e * bf16_to_f64(v[d]);
    }
    double nm = pm > m ? pm : m;
    double a = exp(m - nm), b = exp(pm - nm);
    l = l * a + pl * b;
    for (int d = 0; d < D; d++) acc[d] = acc[d] * a + pacc[d] * b;
    m = nm;
  }
  for (int d = 0; d < D; d++) out[d] = acc[d] / l;
  free(acc); free(pacc);
}

typedef struct {
  orc_pool* p; const int32_t* ids; int32_t batch; const uint16_t* q; double scale; int mode;
  double* out; int next; pthread_mutex_t mu;
} att_job;

static void* att_worker(void* arg) {
  att_job* j = (att_job*)arg;
  orc_pool* p = j->p;
  for (;;) {
    pthread_mutex_lock(&j->mu);
    int w = j->next++;
    pthread_mutex_unlock(&j->mu);
    if (w >= j->batch * p->Hq) break;
    int b = w / p->Hq, h = w % p->Hq;
    const orc_tensor* t = &p->t[j->ids[b]];
    const uint16_t* q = j->q + ((size_t)b * p->Hq + (size_t)h) * (size_t)p->D;
    double* o = j->out + ((size_t)b * p->Hq + (size_t)h) * (size_t)p->D;
    if (j->mode == MODE_ONLINE) attend_online(p, t, q, h, j->scale, o);
    else attend_two_pass(p, t, q, h, j->scale, j->mode, o, NULL);
  }
  return NULL;
}

/* q: [batch][Hq][D] bf16 bits (host); out: [batch][Hq][D] fp64. scale 0 selects 1/sqrt(D).
 * Work is spread over n_threads host threads, one (request, q head) at a time. */
int orc_decode_attention(orc_pool* p, const int32_t* ids, int32_t batch, const uint16_t* q, double scale,
                         int mode, int n_threads, double* out) {
  if (batch < 0 || !q || !out || !isfinite(scale)) return ORC_INVALID;
  const int Tc = p->tokens_per_chunk;
  for (int32_t b = 0; b < batch; b++) {
    orc_tensor* t = tensor_of(p, ids[b]);
    if (!t) return ORC_INVALID;
    if (t->len == 0) return ORC_EMPTY;
    for (int64_t s = 0; s <= (t->len - 1) / Tc; s++) {
      if (t->table[s] == ENTRY_NONE) return ORC_UNMAPPED;
      if (t->table[s] <= -2) return ORC_NOT_RESIDENT;
    }
    if (mode == MODE_TWIN && !p->keep_twin) return ORC_INVALID;
  }
  if (batch == 0) return ORC_OK;
  if (scale == 0.0) scale = 1.0 / sqrt((double)p->D);
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 256) n_threads = 256;
  /* materialise every chunk image first so worker threads only read */
  for (int32_t b = 0; b < batch; b++) {
    orc_tensor* t = &p->t[ids[b]];
    for (int64_t s = 0; s <= (t->len - 1) / Tc; s++) (void)chunk_bytes_of(p, t->table[s]);
  }
  att_job j = { p, ids, batch, q, scale, mode, out, 0, PTHREAD_MUTEX_INITIALIZER };
  pthread_t th[256];
  for (int i = 1; i < n_threads; i++) pthread_create(&th[i], NULL, att_worker, &j);
  att_worker(&j);
  for (int i = 1; i < n_threads; i++) pthread_join(th[i], NULL);
  return ORC_OK;
}

/* softmax weights of one (tensor, q head), for the sum-to-one check; q: [D] bf16 bits */
int orc_attention_weights(orc_pool* p, int32_t id, const uint16_t* q, int h, double scale, double* w_out) {
  orc_tensor* t = tensor_of(p, id);
  if (!t || h < 0 || h >= p->Hq) return ORC_INVALID;
  if (t->len == 0) return ORC_EMPTY;
  if (scale == 0.0) scale = 1.0 / sqrt((double)p->D);
  double o[128];
  attend_two_pass(p, t, q, h, scale, MODE_CHUNKED, o, w_out);
  return ORC_OK;
}
